// Scoring kernels of the token-recall path (paper Section 3.2, Eq. 4 and Eq. 5) for gfx950.
//
// Two passes over the key cache, both built on one MFMA skeleton:
//   pass 1 (MODE 0, row statistics)  S^T = K_tile . Q^T : tokens are the MFMA rows, query rows the
//           columns, so each lane owns one query row and sees 16 tokens of it per 32x32 block; the
//           running maximum and sum of exponentials of Eq. 4's softmax stay in that lane's registers.
//   pass 2 (MODE 1, column scores)   S = Q . K_tile^T : query rows are the MFMA rows, tokens the
//           columns, so each lane owns one token and the Eq. 5 reduction over heads and queries is
//           an in-lane sum (or max) over its 16 accumulator registers per block.
// In both passes a wavefront keeps the fragments of its 32*NB query rows in registers for the whole
// kernel.  K tiles are copied once per workgroup from HBM straight into LDS (buffer loads with the LDS
// flag, three buffers in flight, chunks XOR-swizzled so that the 16-byte fragment reads of 16
// consecutive rows fall in distinct banks) and shared by all query heads of the GQA group.  The loop is
// software pipelined: the MFMA chains of one 32-token block are interleaved, instruction by
// instruction, with the exponentials of the block before it and with the LDS reads of the block after
// it.  Logits leave the MFMA unscaled; scale*log2(e) is folded into the single fma that feeds
// v_exp_f32.  No atomics anywhere: every reduction has a fixed order.
#include "ilre_internal.h"

#include <math.h>

#include <mutex>

#include <type_traits>

namespace ilre {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr float kNegBig = -1.0e30f;
// a partial sum against a frozen reference beyond this is redone against the running maximum: far above anything
// a row with moderate logits reaches, far enough below the fp32 limit that merging 512 splits stays finite
constexpr float kFrozenSumLimit = 1.0e30f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int DT>
struct Traits;

// bf16: one 16-byte chunk holds 8 elements; v_mfma_f32_32x32x16_bf16 contracts 16 per issue
// (lanes 0-31 supply k = 0..7, lanes 32-63 k = 8..15 of the same row).
template <>
struct Traits<ILRE_BF16> {
    static constexpr int kElemBytes = 2;
    static constexpr int kSteps = 8;
    static constexpr int kChunksPerRow = 16;
    // tokens per LDS tile: four 16-byte chunks staged per thread
    static constexpr int tile_tokens(int waves) { return 16 * waves; }
    static __device__ __forceinline__ void mma(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
    }
};

// fp32: one chunk holds 4 elements; v_mfma_f32_32x32x2_f32 contracts 2 per issue (lanes 0-31 supply
// k = 0, lanes 32-63 k = 1).  Element j of both operands' chunks is contracted by issue j, which pairs
// identical k on the A and B side whatever order the k are visited in.
template <>
struct Traits<ILRE_F32> {
    static constexpr int kElemBytes = 4;
    static constexpr int kSteps = 16;
    static constexpr int kChunksPerRow = 32;
    static constexpr int tile_tokens(int waves) { return 16 * waves; }
    static __device__ __forceinline__ void mma(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Online update of one query row's running (max, sum of exponentials) with 16 new logits.
// Logits are raw dot products; c = scale*log2(e) turns them into base-2 exponents.
// A row's running sum is kept as four partial sums (accumulator registers v, v+4, v+8, v+12 feed
// partial v & 3), so that an element costs exactly one fma, one exp2 and one add; they are added up
// once, when the kernel ends.
template <bool MASKED>
__device__ __forceinline__ void row_update(const f32x16 &acc, float c, float &m, float (&z)[4], int64_t tok0, int64_t L)
{
    float s[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        s[v] = acc[v];
        if (MASKED) {
            const int64_t tok = tok0 + 8 * (v >> 2) + (v & 3);
            if (tok >= L) s[v] = -INFINITY;
        }
    }
    float smax = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) smax = fmaxf(smax, s[v]);
    const float mnew = fmaxf(m, smax * c);
    const float rescale = fast_exp2(m - mnew);
    m = mnew;
    const float nm = -mnew;
#pragma unroll
    for (int k = 0; k < 4; ++k) z[k] *= rescale;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v & 3] += fast_exp2(fmaf(s[v], c, nm));
}

// Asynchronous 16-byte-per-lane copy from a buffer resource straight into LDS: lane l of the
// wavefront lands at lds_addr + 16*l; bytes past the resource's num_records read as zero.  Tracked
// by vmcnt.  Issued as inline assembly so that the compiler's conservative alias handling does not
// put a full vmcnt wait in front of every later LDS read.
typedef __attribute__((ext_vector_type(4))) int i32x4;
__device__ __forceinline__ void lds_dma16(i32x4 rsrc, unsigned lds_addr, int voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}

__device__ __forceinline__ float quad_swap1(float x)  // lanes 0<->1, 2<->3 of every quad
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_swap2(float x)  // lanes 0<->2, 1<->3 of every quad
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, true));
}

// The same sum against a frozen reference m: no maximum, no rescale.  Any finite m gives the same
// (m, z) pair up to rounding as long as 2^(x - m) stays in range; a row whose later logits exceed m by
// more than ~2^7 base-2 units overflows to inf, which the kernel detects and redoes with row_update.
__device__ __forceinline__ void row_accumulate(const f32x16 &acc, float c, float m, float (&z)[4])
{
    const float nm = -m;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v & 3] += fast_exp2(fmaf(acc[v], c, nm));
}

// MODE 0: row statistics.  MODE 1: column scores (RMAX = 0 sum over rows, 1 max over rows).
template <int DT, int NB, int WAVES, int MODE, int RMAX>
__global__ __launch_bounds__(WAVES * 64, 2) void score_kernel(const ScoreArgs a)
{
    using T = Traits<DT>;
    constexpr int ES = T::kElemBytes;
    constexpr int STEPS = T::kSteps;
    constexpr int TN = T::tile_tokens(WAVES);
    constexpr int CPR = T::kChunksPerRow;
    constexpr int ROWB = CPR * 16;
    constexpr int TILE_BYTES = TN * ROWB;
    constexpr int NLW = TN * CPR / 64 / WAVES;  // 1 KiB DMA issues per wavefront and tile
    constexpr int TBLOCKS = TN / 32;
    constexpr int UNITS = TBLOCKS;              // pipeline units per tile: one per 32-token block
    constexpr int NPART = WAVES * 2;            // partial column results per token (pass 2)
    // Row pitch of the partial-result buffers.  The flush reads them with four lanes per token, lane group g
    // taking partials g*NPART/4 ..: the four groups of a half-wave must start 8 banks apart (8 tokens each)
    // to cover the 32 LDS banks once.  The stores (32 consecutive tokens of one partial) never conflict.
    constexpr int RSTR = TN + (NPART == 16 ? 34 : 36);
    static_assert((NPART / 4 * RSTR) % 32 == 8 || (NPART / 4 * RSTR) % 32 == 24, "flush lane groups 8 banks apart");
    static_assert(TN * CPR % (64 * WAVES) == 0, "tile must divide over the wavefronts");
    static_assert(UNITS % 2 == 0, "units alternate between two accumulators");
    static_assert(TN == 16 * WAVES && NPART % 4 == 0, "column flush: 16 tokens per wavefront, 4 lanes per token");

    extern __shared__ __align__(16) unsigned char smem[];

    // blockIdx -> (kv head, token split, query block).  Workgroups are dealt round-robin to the 8
    // XCDs, so the query blocks that stream the same K range are given ids with equal id % 8 and
    // consecutive id / 8: they run on one XCD at about the same time and share its L2.
    const int xcd = blockIdx.x % kNumXCD;
    const int slot = blockIdx.x / kNumXCD;
    const int qb = slot % a.nqb;
    const int64_t pair = (int64_t)(slot / a.nqb) * kNumXCD + xcd;
    // Pass 1 notes how long each workgroup ran (0: it had nothing to do); the merge kernel behind it turns the
    // times into pass 2's token ranges.
    const bool timed = MODE == 0 && a.wg_time != nullptr && threadIdx.x == 0;
    const unsigned long long t_begin = timed ? wall_clock64() : 0ull;
    if (timed) a.wg_time[blockIdx.x] = 0u;
    if (pair >= (int64_t)a.Hkv * a.nsplit) return;
    const int g = (int)(pair / a.nsplit);
    const int split = (int)(pair % a.nsplit);
    int64_t tile_lo = (int64_t)split * a.tiles_per_split;
    int64_t tile_hi = (tile_lo + a.tiles_per_split < a.ntiles) ? tile_lo + a.tiles_per_split : a.ntiles;
    if (MODE == 1 && a.split_table != nullptr) {
        // Pass 2's column results do not depend on how the tokens are cut into ranges, so the ranges may follow the
        // speed of the XCD they run on (the table's header says which launch shape it was made for; the table is
        // only used if it is a cut of the context, whatever the workspace holds).
        const int32_t *tb = a.split_table;
        if ((uint32_t)tb[0] == (uint32_t)a.table_tag && (uint32_t)tb[1] == (uint32_t)(a.table_tag >> 32)) {
            // every wavefront checks the whole table (a few loads a lane): edges from 0 to ntiles that never
            // step back cut the context into ranges that cover every tile once, whatever else they are
            bool bad = false;
            for (int i = threadIdx.x & 63; i <= a.nsplit; i += 64) {
                const int64_t e0 = tb[2 + i], e1 = i < a.nsplit ? (int64_t)tb[3 + i] : a.ntiles;
                bad = bad || e0 < 0 || e0 > e1 || e1 > a.ntiles || (i == 0 && e0 != 0) || (i == a.nsplit && e0 != a.ntiles);
            }
            if (!__any(bad)) {
                tile_lo = tb[2 + split];
                tile_hi = tb[3 + split];
            }
        }
    }
    const int64_t tile0 = tile_lo, tile1 = tile_hi;
    if (tile0 >= tile1) return;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const int rl0 = qb * (WAVES * NB * 32) + wave * (NB * 32);
    const int64_t nrows = (int64_t)a.Hq * a.Lq;

    // Query fragments, resident for the whole kernel: lane holds, for each of its NB blocks, row
    // l32 of the block, 16-byte chunk (2*step + half) of that row.
    uint4 qf[NB][STEPS];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int rl = rl0 + b * 32 + l32;
        if (rl < a.rows_per_group) {
            const int h = g * a.G + rl / a.Lq;
            const int i = rl % a.Lq;
            const unsigned char *src =
                (const unsigned char *)a.q + ((int64_t)h * a.q_stride_head + (int64_t)i * a.q_stride_token) * ES;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) qf[b][st] = *(const uint4 *)(src + (st * 2 + half) * 16);
        } else {
#pragma unroll
            for (int st = 0; st < STEPS; ++st) qf[b][st] = make_uint4(0, 0, 0, 0);
        }
    }

    // K tiles: three LDS buffers of TN rows, row r's 16-byte chunk c stored at chunk position
    // c ^ (r & 15), so that the fragment reads of 16 consecutive rows fall in distinct banks while a
    // wavefront's DMA still fills 1 KiB of consecutive LDS.
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned char *kbase = (const unsigned char *)a.k + (int64_t)g * a.k_stride_head * ES;
    const int64_t krow_bytes = a.k_stride_token * ES;
    int dma_voff[NLW];
#pragma unroll
    for (int j = 0; j < NLW; ++j) {
        const int pchunk = (wave * NLW + j) * 64 + lane;
        const int row = pchunk / CPR, cpos = pchunk % CPR;
        dma_voff[j] = (int)(row * krow_bytes) + (cpos ^ (row & 15)) * 16;
    }
    // Pass 2 walks its split backwards: pass 1 has just streamed the same split forwards, so what it read
    // last is what the memory-side cache still holds (an eighth of K at 1M tokens).  `tile` counts in
    // processing order everywhere; only the two places that turn it into tokens go through here.
    auto first_token = [&](int64_t tile) { return (MODE == 1 ? tile0 + tile1 - 1 - tile : tile) * TN; };
    auto issue_tile = [&](int64_t tile, int buf) {
        const int64_t tok0 = first_token(tile);
        const unsigned long long base = (unsigned long long)(kbase + tok0 * krow_bytes);
        long long avail = (a.L - tok0 - 1) * krow_bytes + ROWB;  // bytes up to the end of row L-1
        if (avail > 0xFFFFFFFFll) avail = 0xFFFFFFFFll;
        i32x4 rsrc;
        rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
        rsrc[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(base >> 32) & 0xFFFFu));
        rsrc[2] = __builtin_amdgcn_readfirstlane((int)(unsigned)avail);
        rsrc[3] = 0x00020000;
#pragma unroll
        for (int j = 0; j < NLW; ++j)
            lds_dma16(rsrc, __builtin_amdgcn_readfirstlane(lds0 + buf * TILE_BYTES + (wave * NLW + j) * 1024), dma_voff[j]);
    };

    // per-lane LDS byte offset of fragment chunk (2*st + half) of row l32 within a 32-row block,
    // relative to the tile buffer being read; advanced from buffer to buffer in place
    unsigned frag_addr[STEPS];

    // pass-1 state: one (max, sum) per owned query row, in base-2 exponent units
    float m[NB], z[NB][4];
    // pass-2 state: per accumulator register the row's exponent offset -(max*log2e + log2 sum)
    float noff[MODE == 1 ? NB : 1][16];
    float *red = (float *)(smem + 3 * TILE_BYTES);  // [3][NPART][RSTR], pass 2 only
    const int unit = g * a.nqb + qb;

    if (MODE == 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            m[b] = kNegBig;
#pragma unroll
            for (int k = 0; k < 4; ++k) z[b][k] = 0.f;
        }
    } else {
        // the workgroup's slice of the offset table (filled before this launch: one entry per query row in the
        // order the workgroups own them, -inf for padded rows, whose q = 0: exp2(0*c - inf) = 0); accumulator
        // registers 4j .. 4j+3 of a lane are four consecutive rows
        const float4 *off4 = (const float4 *)(a.row_off + (int64_t)unit * (WAVES * NB * 32) + wave * (NB * 32));
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 x = off4[(b * 32 + 8 * j + 4 * half) / 4];
                noff[b][4 * j + 0] = x.x;
                noff[b][4 * j + 1] = x.y;
                noff[b][4 * j + 2] = x.z;
                noff[b][4 * j + 3] = x.w;
            }
        }
    }

    // Pass 2: combine the NPART partial column results of a finished tile in a fixed order.  Wave w
    // takes tokens 16w..16w+15, four lanes per token, each lane NPART/4 partials, then the quad.
    // In the tile loop the LDS reads are issued inside the first unit and consumed in the last one, so
    // that their latency hides behind MFMAs.
    float fl[NPART / 4];
    auto flush_load = [&](int64_t tile) {
        const float *rb = red + (int)(tile - tile0) % 3 * NPART * RSTR;
        const int tl = wave * 16 + (lane >> 2), part0 = (lane & 3) * (NPART / 4);
#pragma unroll
        for (int k = 0; k < NPART / 4; ++k) fl[k] = rb[(part0 + k) * RSTR + tl];
    };
    // `live` false: nothing to flush yet.  Lanes with nothing to store write to a dump slot instead of
    // branching around the store, which would cut the tile body into separately scheduled pieces.
    auto flush_finish = [&](int64_t tile, bool live) {
        const int tl = wave * 16 + (lane >> 2);
        float acc = fl[0];
#pragma unroll
        for (int k = 1; k < NPART / 4; ++k) acc = RMAX ? fmaxf(acc, fl[k]) : acc + fl[k];
        const float x1 = quad_swap1(acc);
        acc = RMAX ? fmaxf(acc, x1) : acc + x1;
        const float x2 = quad_swap2(acc);
        acc = RMAX ? fmaxf(acc, x2) : acc + x2;
        const int64_t tok = first_token(tile) + tl;
        // after the quad reduction the four lanes of a token hold the same value and all store it
        float *dst = (live && tok < a.L) ? a.partial + ((int64_t)unit * a.L + tok) : a.dump + (lane & 15);
        *dst = acc;
    };
    auto flush_columns = [&](int64_t tile) {
        flush_load(tile);
        flush_finish(tile, true);
    };

    // The softmax arithmetic of one finished 32x32 block ("unit": token block tb, query block b).
    // It runs one unit behind the MFMAs, so that the matrix pipe works on unit u while the vector
    // pipe exponentiates unit u-1 from the other accumulator.
    float col = 0.f;  // pass 2: running column result of the token block over its NB query blocks
    // `rb` is the partial-result buffer (0..2) of the unit's tile, pass 2 only.
    auto finish_unit = [&](const f32x16 &acc, int b, int tb, int64_t tile, int rb, auto masked_tag, auto frozen_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool FROZEN = decltype(frozen_tag)::value;
        if (MODE == 0) {
            if (FROZEN)
                row_accumulate(acc, a.c, m[b], z[b]);
            else
                row_update<MASKED>(acc, a.c, m[b], z[b], tile * TN + tb * 32 + 4 * half, a.L);
        } else {
            float e[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) e[v] = fast_exp2(fmaf(acc[v], a.c, noff[b][v]));
            float p0 = e[0], p1 = e[1], p2 = e[2], p3 = e[3];
#pragma unroll
            for (int v = 4; v < 16; v += 4) {
                if (RMAX) {
                    p0 = fmaxf(p0, e[v]), p1 = fmaxf(p1, e[v + 1]), p2 = fmaxf(p2, e[v + 2]), p3 = fmaxf(p3, e[v + 3]);
                } else {
                    p0 += e[v], p1 += e[v + 1], p2 += e[v + 2], p3 += e[v + 3];
                }
            }
            const float part = RMAX ? fmaxf(fmaxf(p0, p1), fmaxf(p2, p3)) : (p0 + p1) + (p2 + p3);
            if (b == 0)
                col = part;
            else
                col = RMAX ? fmaxf(col, part) : col + part;
            // (the unit before a split's very first one stores zeros into a buffer that is rewritten
            // before it is read: no condition here, the tile body stays free of branches)
            if (b == NB - 1) red[(rb * NPART + wave * 2 + half) * RSTR + tb * 32 + l32] = col;
        }
    };

    f32x16 acc[2][NB];
    uint4 kf[STEPS];
    auto start_split = [&]() {
#pragma unroll
        for (int st = 0; st < STEPS; ++st) frag_addr[st] = lds0 + l32 * ROWB + (((2 * st + half) ^ (l32 & 15)) * 16);
        // Prologue: the first two tiles go to buffers 0 and 1.
        issue_tile(tile0, 0);
        if (tile0 + 1 < tile1) issue_tile(tile0 + 1, 1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        // acc[u & 1] receives unit u (a 32-token block against the wave's NB query blocks); the unit
        // before the very first one is all -inf, which the softmax arithmetic turns into zeros.
    #pragma unroll
        for (int b = 0; b < NB; ++b) {
    #pragma unroll
            for (int v = 0; v < 16; ++v) acc[1][b][v] = -INFINITY;
        }
    #pragma unroll
        for (int st = 0; st < STEPS; ++st)
            kf[st] = *(const uint4 *)(__attribute__((address_space(3))) unsigned char *)(size_t)frag_addr[st];
    };

    // One tile.  Its buffer and the next tile's are already published; the tile after that is
    // requested now and published by the barrier at the end.  Per 32-token block the NB independent
    // MFMA chains are interleaved step by step; as soon as a step's fragment has fed all chains it is
    // refilled from LDS for the next block (for the last block, from the next tile's buffer).
    // CUR_RAGGED is only ever true for the last tile of the context, and only in pass 1.
    auto do_tile = [&](int64_t tile, auto ragged_tag, auto frozen_tag) {
        constexpr bool CUR_RAGGED = decltype(ragged_tag)::value;
        constexpr bool FROZEN = decltype(frozen_tag)::value;  // pass 1: reference maxima no longer move
        const int it = (int)(tile - tile0);
        const int rb_cur = it % 3, rb_prev = (it + 2) % 3;
        if (tile + 2 < tile1) issue_tile(tile + 2, (it + 2) % 3);
        // byte distance from this tile's buffer to the next tile's
        const int to_next = (it % 3 == 2) ? -2 * TILE_BYTES : TILE_BYTES;

#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            if (u == UNITS - 1) {
#pragma unroll
                for (int st = 0; st < STEPS; ++st) frag_addr[st] += to_next;
            }
            const int next_block = (u == UNITS - 1) ? 0 : (u + 1) * 32 * ROWB;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[u & 1][b][v] = 0.f;
            }
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    if (MODE == 0)
                        T::mma(acc[u & 1][b], kf[st], qf[b][st]);
                    else
                        T::mma(acc[u & 1][b], qf[b][st], kf[st]);
                }
                kf[st] = *(const uint4 *)((__attribute__((address_space(3))) unsigned char *)(size_t)frag_addr[st] + next_block);
            }
            // column results of the tile before the previous one: LDS reads behind the first unit's
            // MFMAs (in straight-line code, so the fragment waits can leave them in flight), sums and
            // store in the tile's last unit
            if (MODE == 1 && u == 0) flush_load(it >= 2 ? tile - 2 : tile);
            if (MODE == 1 && u == UNITS - 1) flush_finish(tile - 2, it >= 2);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                if (u == 0)
                    finish_unit(acc[1][b], b, UNITS - 1, tile - 1, rb_prev, std::false_type{}, frozen_tag);
                else
                    finish_unit(acc[(u - 1) & 1][b], b, u - 1, tile, rb_cur, std::bool_constant<CUR_RAGGED>{}, frozen_tag);
            }
            // ask the scheduler for: one MFMA (group), a slice of the vector work, and a fragment
            // read after every NB-th MFMA
#pragma unroll
            for (int st = 0; st < 8; ++st) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    __builtin_amdgcn_sched_group_barrier(0x008, DT == ILRE_BF16 ? 1 : STEPS / 2, 0);
                    if (b == NB - 1) __builtin_amdgcn_sched_group_barrier(0x100, STEPS / 8, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (MODE == 0 && !FROZEN) ? 8 : 6, 0);
                }
            }
        }

        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    // Only pass 1 has to mask the tokens past L (in pass 2 a lane is a token and is simply not
    // stored); the ragged tile, if any, is the last tile of the last split.
    const bool last_ragged = MODE == 0 && tile1 * TN > a.L;
    const int64_t tile_full_end = last_ragged ? tile1 - 1 : tile1;
    // One walk over the split.  Pass 1 follows the running maximum for the first two tiles, then freezes each
    // row's reference and only accumulates -- unless `online_all`, the always-safe form.
    auto run_split = [&](bool online_all) {
    start_split();
    int64_t online_end = tile_full_end;
    if (MODE == 0 && !online_all && tile0 + 2 < tile_full_end) online_end = tile0 + 2;
    int64_t tile = tile0;
    for (; tile < online_end; ++tile) do_tile(tile, std::false_type{}, std::false_type{});
    if (MODE == 0)
        for (; tile < tile_full_end; ++tile) do_tile(tile, std::false_type{}, std::true_type{});
    if (last_ragged) do_tile(tile1 - 1, std::true_type{}, std::false_type{});
    // drain the pipeline: the last unit of the last tile
    const int rb_last = (int)((tile1 - 1 - tile0) % 3);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (last_ragged)
            finish_unit(acc[(UNITS - 1) & 1][b], b, UNITS - 1, tile1 - 1, rb_last, std::true_type{}, std::false_type{});
        else
            finish_unit(acc[(UNITS - 1) & 1][b], b, UNITS - 1, tile1 - 1, rb_last, std::false_type{}, std::false_type{});
    }
    };
    run_split(MODE == 0 && a.force_online);
    if (MODE == 0 && !a.force_online) {
        // A row whose later logits lie far above its frozen reference sums to inf (or to something a merge over
        // the splits could push out of range): the workgroup then walks its split again, following the maximum.
        bool bad = false;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int k = 0; k < 4; ++k) bad = bad || !(z[b][k] <= kFrozenSumLimit);
        if (__syncthreads_or(bad)) {  // uniform; also orders the last reads of the tile buffers before the new DMA
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                m[b] = kNegBig;
#pragma unroll
                for (int k = 0; k < 4; ++k) z[b][k] = 0.f;
            }
            run_split(true);
        }
    }

    if (MODE == 1) {
        __syncthreads();
        if (tile1 - tile0 >= 2) flush_columns(tile1 - 2);
        flush_columns(tile1 - 1);
    } else {
        // The two half-waves saw disjoint tokens of the same query rows: merge, then one partial
        // (max, sum) per row and split.
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float zb = (z[b][0] + z[b][1]) + (z[b][2] + z[b][3]);
            const float mo = __shfl_xor(m[b], 32);
            const float zo = __shfl_xor(zb, 32);
            const float mm = fmaxf(m[b], mo);
            const float zz = zb * fast_exp2(m[b] - mm) + zo * fast_exp2(mo - mm);
            const int rl = rl0 + b * 32 + l32;
            if (half == 0 && rl < a.rows_per_group) {
                const int64_t r = (int64_t)(g * a.G + rl / a.Lq) * a.Lq + rl % a.Lq;
                a.part_m[(int64_t)split * nrows + r] = mm;
                a.part_z[(int64_t)split * nrows + r] = zz;
            }
        }
        if (timed) {
            const unsigned long long dt = wall_clock64() - t_begin;  // 10 ns ticks
            a.wg_time[blockIdx.x] = dt < 0xFFFFFFFFull ? (uint32_t)(dt ? dt : 1) : 0xFFFFFFFFu;
        }
    }
}

// Pass 2's per-row exponent offsets, -(max*log2e + log2 sum), laid out in the order the workgroups own the rows:
// entry (unit, local) is row `qb*rows_per_wg + local` of kv head g's group, unit = g*nqb + qb; rows past the
// group's last one (padding of the last query block) get -inf.  Done once here rather than by every lane of
// every workgroup of the column-score kernel, whose row indices cost two integer divisions each.
__global__ __launch_bounds__(256) void row_offsets_kernel(const float *row_max, const float *row_sumexp, float *row_off, int entries,
                                                          int rows_per_wg, int nqb, int rows_per_group, int G, int Lq)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= entries) return;
    const int unit = e / rows_per_wg, local = e % rows_per_wg;
    const int g = unit / nqb, qb = unit % nqb;
    const int rl = qb * rows_per_wg + local;
    float off = -INFINITY;
    if (rl < rows_per_group) {
        const int64_t r = (int64_t)(g * G + rl / Lq) * Lq + rl % Lq;
        off = -(row_max[r] * kLog2e + __log2f(row_sumexp[r]));
    }
    row_off[e] = off;
}

// Merge the per-split partial statistics of each row (fixed order) and convert to the natural-log units of
// Eq. 4: row_max = a reference <= max_t logit, row_sumexp = sum_t exp(logit - row_max).
// Sixteen lanes share a row and the splits among them, so that all of a row's partials are fetched in one
// round of loads (a thread a row would fetch them in a chain of memory latencies: this kernel sits between
// the two scoring passes and is all latency).
constexpr int kCombineLanes = 16;
// Where the offset of row rl of kv head g's group sits in pass 2's table (see row_offsets_kernel).
// Pass 2's token ranges from pass 1's workgroup times.  The 8 XCDs of the chip do not run at one speed (their
// workgroups finish up to 6 % apart, the same dies ahead in every launch), and a launch lasts as long as its
// slowest XCD.  Split s of every kv head runs on the same XCD when the splits per head are a multiple of 8, so
// the ranges are sized by the mean time the workgroups of split s took in pass 1: range s gets a share of the
// tiles proportional to 1 / time, within 15 % of an even share (a workgroup that walked its split twice, or a
// disturbed launch, must not skew the next one).  Only pass 2 is cut this way: its results do not depend on the
// cut, pass 1's rounding would.
constexpr int kMaxBalancedSplits = 512;
struct BalanceArgs {
    const uint32_t *wg_time;  // null: no table wanted
    int32_t *table;           // [2 + nsplit + 1]: tag (low, high), then the first tile of every range and ntiles
    uint64_t tag;
    int grid, nqb, nsplit, Hkv;
    int64_t ntiles;
};
__device__ void make_split_table(const BalanceArgs &b)
{
    __shared__ uint32_t sum[kMaxBalancedSplits], cnt[kMaxBalancedSplits];
    for (int s = threadIdx.x; s < b.nsplit; s += blockDim.x) sum[s] = cnt[s] = 0;
    __syncthreads();
    for (int w = threadIdx.x; w < b.grid; w += blockDim.x) {
        const uint32_t t = b.wg_time[w];
        const int64_t pair = (int64_t)((w / kNumXCD) / b.nqb) * kNumXCD + w % kNumXCD;
        if (t != 0 && pair < (int64_t)b.Hkv * b.nsplit) {
            atomicAdd(&sum[pair % b.nsplit], t >> 4);  // 160 ns units: the sum over all workgroups of a split fits
            atomicAdd(&cnt[pair % b.nsplit], 1u);
        }
    }
    __syncthreads();
    // One wavefront, eight splits a lane: mean time per split, weight = mean of those over the split's own,
    // running sum of the weights, edges.  (One thread doing this in a loop was a 20 us chain at 32 splits.)
    if (threadIdx.x >= 64) return;
    constexpr int kPer = kMaxBalancedSplits / 64;
    const int lane = threadIdx.x;
    float d[kPer], lsum = 0.f, lcnt = 0.f;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int sp = lane * kPer + k;
        d[k] = (sp < b.nsplit && cnt[sp] && sum[sp]) ? (float)sum[sp] / (float)cnt[sp] : 0.f;
        lsum += d[k];
        lcnt += d[k] > 0.f ? 1.f : 0.f;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        lsum += __shfl_xor(lsum, o);
        lcnt += __shfl_xor(lcnt, o);
    }
    const float mean = lcnt > 0.f ? lsum / lcnt : 1.f;
    float w[kPer], lw = 0.f;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int sp = lane * kPer + k;
        float x = d[k] > 0.f ? mean / d[k] : 1.f;
        x = x < 0.85f ? 0.85f : (x > 1.15f ? 1.15f : x);
        w[k] = sp < b.nsplit ? x : 0.f;
        lw += w[k];
    }
    float incl = lw;  // inclusive running sum over the lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    const float weights = __shfl(incl, 63);
    float upto = incl - lw;
    if (lane == 0) {
        b.table[0] = (int32_t)(uint32_t)b.tag;
        b.table[1] = (int32_t)(uint32_t)(b.tag >> 32);
        b.table[2] = 0;
    }
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int sp = lane * kPer + k;
        upto += w[k];
        if (sp < b.nsplit) {
            int64_t edge = (int64_t)((double)b.ntiles * (double)(upto / weights) + 0.5);
            if (edge > b.ntiles || sp == b.nsplit - 1) edge = b.ntiles;
            b.table[3 + sp] = (int32_t)edge;  // non-decreasing: the running sum is, and so are the steps behind it
        }
    }
}

struct OffsetTable {
    float *row_off;  // null: not wanted
    int group_entries;  // nqb * rows_per_wg: entries per kv head, of which the first rows_per_group are rows
    int rows_per_group, G, Lq, Hkv;
};
__global__ __launch_bounds__(256) void combine_row_stats(const float *part_m, const float *part_z, int nsplit, int64_t nrows,
                                                         float *row_max, float *row_sumexp, const OffsetTable tab,
                                                         const BalanceArgs bal)
{
    constexpr int kBlock = 4;
    if (bal.wg_time && blockIdx.x == gridDim.x - 1) {  // the launch's last workgroup is there for the table alone
        make_split_table(bal);
        return;
    }
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = gid / kCombineLanes;
    const int sub = (int)(gid % kCombineLanes);
    const int64_t rr = r < nrows ? r : nrows - 1;  // surplus groups redo the last row and store no statistics
    float mm = kNegBig;
    for (int s0 = sub; s0 < nsplit; s0 += kCombineLanes * kBlock) {
        float m[kBlock];
#pragma unroll
        for (int i = 0; i < kBlock; ++i) {
            const int s = s0 + i * kCombineLanes;
            m[i] = part_m[(int64_t)(s < nsplit ? s : nsplit - 1) * nrows + rr];
        }
#pragma unroll
        for (int i = 0; i < kBlock; ++i) mm = fmaxf(mm, m[i]);
    }
#pragma unroll
    for (int o = 1; o < kCombineLanes; o <<= 1) mm = fmaxf(mm, __shfl_xor(mm, o));
    float zz = 0.f;
    for (int s0 = sub; s0 < nsplit; s0 += kCombineLanes * kBlock) {
        float m[kBlock], z[kBlock];
#pragma unroll
        for (int i = 0; i < kBlock; ++i) {
            const int s = s0 + i * kCombineLanes;
            const int64_t at = (int64_t)(s < nsplit ? s : nsplit - 1) * nrows + rr;
            m[i] = part_m[at];
            z[i] = part_z[at];
        }
#pragma unroll
        for (int i = 0; i < kBlock; ++i)
            if (s0 + i * kCombineLanes < nsplit) zz += z[i] * fast_exp2(m[i] - mm);
    }
#pragma unroll
    for (int o = 1; o < kCombineLanes; o <<= 1) zz += __shfl_xor(zz, o);
    if (sub != 0) return;
    if (r < nrows) {
        row_max[r] = mm * kLn2;
        row_sumexp[r] = zz;
        if (tab.row_off) {
            // the same value row_offsets_kernel derives from the two outputs just written
            const int h = (int)(r / tab.Lq), i = (int)(r % tab.Lq);
            const int rl = (h % tab.G) * tab.Lq + i;
            tab.row_off[(int64_t)(h / tab.G) * tab.group_entries + rl] = -((mm * kLn2) * kLog2e + __log2f(zz));
        }
    } else if (tab.row_off) {
        // surplus groups fill the table's padding (rows past a group's last one)
        const int pad_per_group = tab.group_entries - tab.rows_per_group;
        const int64_t p = r - nrows;
        if (p < (int64_t)pad_per_group * tab.Hkv)
            tab.row_off[(p / pad_per_group) * tab.group_entries + tab.rows_per_group + p % pad_per_group] = -INFINITY;
    }
}

// score[t] = sum (or max) over the (kv head, query block) units of their partial column results.
template <int RMAX>
__global__ void reduce_units(const float *partial, int nunits, int64_t L, float *score)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= L) return;
    // eight units at a time, their loads issued together; the sum runs in unit order
    constexpr int kBlock = 8;
    float acc = 0.f;
    for (int u0 = 0; u0 < nunits; u0 += kBlock) {
        float x[kBlock];
#pragma unroll
        for (int i = 0; i < kBlock; ++i) x[i] = partial[(int64_t)(u0 + i < nunits ? u0 + i : nunits - 1) * L + t];
#pragma unroll
        for (int i = 0; i < kBlock; ++i) {
            if (u0 + i >= nunits) break;
            if (u0 + i == 0)
                acc = x[i];
            else
                acc = RMAX ? fmaxf(acc, x[i]) : acc + x[i];
        }
    }
    score[t] = acc;
}

template <int DT>
constexpr size_t tile_lds_bytes(int waves)
{
    return 3 * (size_t)Traits<DT>::tile_tokens(waves) * (Traits<DT>::kChunksPerRow * 16);
}

// The dynamic-LDS ceiling of a kernel is raised once per process (to the most any plan asks of it: the
// 8-wavefront tiles plus the partial-result buffers of pass 2), not on every launch.
constexpr int kMaxDynamicLds = 144 * 1024;  // leaves room for the few bytes of static LDS a kernel may hold
hipError_t raise_lds_limit_once(const void *kernel)
{
    static std::mutex mutex;
    static const void *done[32];
    static int ndone = 0;
    std::lock_guard<std::mutex> lock(mutex);
    for (int i = 0; i < ndone; ++i)
        if (done[i] == kernel) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynamicLds);
    if (e == hipSuccess && ndone < 32) done[ndone++] = kernel;
    return e;
}

template <typename K>
hipError_t launch_score(K kernel, int grid, int threads, size_t lds, const ScoreArgs &a, hipStream_t s)
{
    hipError_t e = raise_lds_limit_once((const void *)kernel);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds, s, a);
    return hipGetLastError();
}

}  // namespace

ScorePlan make_score_plan(int dtype, int64_t L, int Lq, int Hq, int Hkv)
{
    ScorePlan p{};
    p.dtype = dtype;
    const int G = Hq / Hkv;
    p.rows_per_group = G * Lq;
    if (dtype == ILRE_F32) {
        p.waves = 4;
        p.nb = 1;
    } else {
        p.nb = 2;
        // 8 waves (512 rows) unless 4 waves (256 rows) leave fewer padded rows
        const int64_t pad8 = ((p.rows_per_group + 511) / 512) * 512;
        const int64_t pad4 = ((p.rows_per_group + 255) / 256) * 256;
        p.waves = pad4 < pad8 ? 4 : 8;
    }
    p.tile_tokens = dtype == ILRE_F32 ? Traits<ILRE_F32>::tile_tokens(p.waves) : Traits<ILRE_BF16>::tile_tokens(p.waves);
    p.rows_per_wg = p.waves * p.nb * 32;
    p.nqb = (p.rows_per_group + p.rows_per_wg - 1) / p.rows_per_wg;
    p.ntiles = (L + p.tile_tokens - 1) / p.tile_tokens;
    p.nunits = Hkv * p.nqb;
    // enough splits for one workgroup of 8 waves (two of 4 waves) per compute unit
    const int target = kNumCU * (p.waves == 8 ? 1 : 2);
    int64_t nsplit = (target + p.nunits / 2) / p.nunits;
    if (nsplit < 1) nsplit = 1;
    if (nsplit > p.ntiles) nsplit = p.ntiles;
    p.tiles_per_split = (p.ntiles + nsplit - 1) / nsplit;
    p.nsplit = (int)((p.ntiles + p.tiles_per_split - 1) / p.tiles_per_split);
    const int64_t pairs = (int64_t)Hkv * p.nsplit;
    p.grid = (int)(((pairs + kNumXCD - 1) / kNumXCD) * kNumXCD * p.nqb);
    const size_t tiles = dtype == ILRE_F32 ? tile_lds_bytes<ILRE_F32>(p.waves) : tile_lds_bytes<ILRE_BF16>(p.waves);
    // pass 2's ranges follow the XCDs' speed where a range is long enough for that to matter
    p.balanced = p.tiles_per_split >= 64 && p.nsplit >= kNumXCD && p.nsplit <= kMaxBalancedSplits;
    uint64_t tag = 0x494c52652d584344ull;  // what a table has to have been made for
    for (uint64_t v : {(uint64_t)L, (uint64_t)p.ntiles, (uint64_t)p.nsplit, (uint64_t)p.nqb, (uint64_t)Hkv, (uint64_t)p.tile_tokens,
                       (uint64_t)p.grid})
        tag = (tag ^ v) * 0x9E3779B97F4A7C15ull + 0x7F4A7C15ull;
    p.table_tag = tag;
    p.lds_bytes_stats = tiles;
    p.lds_bytes_cols = tiles + 3 * 2 * (size_t)p.waves * (p.tile_tokens + 36) * sizeof(float);  // pitch <= tokens + 36
    return p;
}

hipError_t launch_row_stats(const ScorePlan &p, const ScoreArgs &a, float *row_max, float *row_sumexp, hipStream_t s, bool offsets)
{
    // One launch: a workgroup whose sums against frozen references leave the safe range walks its split a second
    // time in the always-safe form before it writes its partials.
    const size_t lds = p.lds_bytes_stats;
    const int64_t nrows = (int64_t)a.Hq * a.Lq;
    hipError_t e;
    if (p.dtype == ILRE_F32)
        e = launch_score(score_kernel<ILRE_F32, 1, 4, 0, 0>, p.grid, 256, lds, a, s);
    else if (p.waves == 4)
        e = launch_score(score_kernel<ILRE_BF16, 2, 4, 0, 0>, p.grid, 256, lds, a, s);
    else
        e = launch_score(score_kernel<ILRE_BF16, 2, 8, 0, 0>, p.grid, 512, lds, a, s);
    if (e != hipSuccess) return e;
    const OffsetTable tab{offsets ? a.row_off : nullptr, p.nqb * p.rows_per_wg, p.rows_per_group, a.G, a.Lq, a.Hkv};
    // one 16-lane group per row, and with the table one more per padded table entry
    const int64_t groups = nrows + (offsets ? (int64_t)(tab.group_entries - tab.rows_per_group) * a.Hkv : 0);
    const bool balance = a.wg_time != nullptr && a.split_table != nullptr;
    const BalanceArgs bal{balance ? a.wg_time : nullptr, a.split_table, a.table_tag, p.grid, p.nqb, p.nsplit, a.Hkv, p.ntiles};
    hipLaunchKernelGGL(combine_row_stats, dim3((unsigned)((groups * kCombineLanes + 255) / 256) + (balance ? 1u : 0u)), dim3(256), 0, s,
                       a.part_m, a.part_z, a.nsplit, nrows, row_max, row_sumexp, tab, bal);
    return hipGetLastError();
}

hipError_t launch_reduce_units(const float *partial, int nunits, int64_t L, int rmax, float *out_scores, hipStream_t s)
{
    const unsigned blocks = (unsigned)((L + 255) / 256);
    if (rmax)
        hipLaunchKernelGGL(reduce_units<1>, dim3(blocks), dim3(256), 0, s, partial, nunits, L, out_scores);
    else
        hipLaunchKernelGGL(reduce_units<0>, dim3(blocks), dim3(256), 0, s, partial, nunits, L, out_scores);
    return hipGetLastError();
}

hipError_t launch_col_scores(const ScorePlan &p, const ScoreArgs &a, int score_mode, float *out_scores, hipStream_t s, bool reduce,
                             bool have_offsets)
{
    hipError_t e;
    const size_t lds = p.lds_bytes_cols;
    const bool mx = score_mode == ILRE_SCORE_MAX;
    if (!have_offsets) {
        const int entries = p.nunits * p.rows_per_wg;
        hipLaunchKernelGGL(row_offsets_kernel, dim3((unsigned)((entries + 255) / 256)), dim3(256), 0, s, a.row_max, a.row_sumexp,
                           a.row_off, entries, p.rows_per_wg, p.nqb, p.rows_per_group, a.G, a.Lq);
    }
    if (p.dtype == ILRE_F32)
        e = mx ? launch_score(score_kernel<ILRE_F32, 1, 4, 1, 1>, p.grid, 256, lds, a, s)
               : launch_score(score_kernel<ILRE_F32, 1, 4, 1, 0>, p.grid, 256, lds, a, s);
    else if (p.waves == 4)
        e = mx ? launch_score(score_kernel<ILRE_BF16, 2, 4, 1, 1>, p.grid, 256, lds, a, s)
               : launch_score(score_kernel<ILRE_BF16, 2, 4, 1, 0>, p.grid, 256, lds, a, s);
    else
        e = mx ? launch_score(score_kernel<ILRE_BF16, 2, 8, 1, 1>, p.grid, 512, lds, a, s)
               : launch_score(score_kernel<ILRE_BF16, 2, 8, 1, 0>, p.grid, 512, lds, a, s);
    if (e != hipSuccess || !reduce) return e;
    return launch_reduce_units(a.partial, p.nunits, a.L, mx ? 1 : 0, out_scores, s);
}

}  // namespace ilre
