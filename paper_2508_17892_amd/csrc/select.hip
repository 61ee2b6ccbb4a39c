// Context allocation (paper Section 3.2, Algorithm 1) for gfx950, in two forms: one stride-1 max
// pooling per kernel size (the "window-max" form), and the algorithm as printed (strided max pooling,
// then stride-1 average pooling, one combination per pair of kernel sizes, the best K_m cells only).
//
// Algorithm 1 pools the scores per combination, takes a ranked candidate list per combination and
// walks it, skipping tokens an earlier combination already allocated, until the combination's share
// is filled.  What a combination's candidates are does not depend on the combinations before it (in
// the window-max form its share can be met from its top K_j = B_j + (shares before it) ranked tokens,
// whatever the earlier ones took; in the printed form K_m is given), so the candidate sets are built
// for all combinations at once:
//
//   cell_max     printed form only: the strided max pooling, one cell array per max kernel
//   sel_init     clears histograms and counters, writes each combination's control block
//   pool_hist<1> wavefronts share out the 256-element "fine chunks" of the source array (the scores, or
//                a cell array): elements + halo into the wavefront's own LDS buffers, pooled value
//                (sliding maximum by doubling, or the average summed left to right), a 2048-bin LDS
//                histogram of the top 11 bits of the value's order-preserving key, added to the
//                combination's global histogram.  The last workgroup of a combination to finish
//                locates the bin holding its K_j-th largest key.
//   pool_hist<2> same pooling; histogram of the next 11 bits of the keys inside that bin; the last
//                workgroup locates the 22-bit prefix of the K_j-th largest key.
//   collect      keys above the prefix go to the combination's candidate list, keys that share it to
//                a boundary list (a few dozen on real scores; everything on all-equal scores)
//   refine       per combination: the boundary list is radix-selected down (8 bits a pass, survivors
//                compacted) to what is needed -- in the window-max form only while it is longer than
//                kSelSmall, extra candidates rank last and are harmless; in the printed form to
//                exactly K_m elements -- and joins the candidates
//   allocate     one workgroup walks the combinations in order: the tokens of the candidate elements
//                that are not yet allocated (LDS hash set), exact radix select of the B_j largest
//                among them in registers, then the allocated set sorted ascending behind the sink part.
//
// Long contexts in the window-max form (L >= 4M and >= 1024 tokens per budgeted token) start with a
// pruning pre-pass: the maximum of every fine chunk (one streaming read of the scores), the 22-bit
// prefix of the budget-th largest of those maxima (the same two histogram passes, run on the maxima),
// and the list of fine chunks that can still hold an admitted token; the three pooling passes then
// visit only that list.
//
// Ranking is (pooled value descending, token index ascending): the 64-bit key is the ordered value
// bits above the complemented element index, so all keys are distinct and every step is
// order-independent; the integer atomics only reserve list slots and build histograms, and the result
// is deterministic.  An element of m tokens ranks its tokens in ascending order, which is the order
// the same key gives them once the element index is replaced by the token index.
#include "ilre_internal.h"

namespace ilre {
namespace {

constexpr int kThreads = 1024;                    // refine, allocate: one large workgroup
constexpr int kPoolThreads = 256;                 // pooling passes: four wavefronts, one fine chunk each
constexpr int kPoolWaves = kPoolThreads / 64;
constexpr int kPerThread = kSelFine / 64;         // 4 tokens per lane
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kHashSlots = 16384;                 // >= 2 * ILRE_MAX_BUDGET
constexpr int kKeysPerThread = kCandCap / kThreads;
constexpr int kBuckets = 4096;                       // final counting sort (3 * kBuckets <= kHashSlots)

// Per-combination description, host -> sel_init (by value), which copies it into the control blocks.
struct SelParams {
    int n;
    uint32_t op, exact;
    uint32_t before[ILRE_MAX_POOL_KERNELS], after[ILRE_MAX_POOL_KERNELS];
    uint32_t share[ILRE_MAX_POOL_KERNELS], want[ILRE_MAX_POOL_KERNELS];
    uint32_t len[ILRE_MAX_POOL_KERNELS], cell[ILRE_MAX_POOL_KERNELS];
    uint64_t src_off[ILRE_MAX_POOL_KERNELS], tie_off[ILRE_MAX_POOL_KERNELS];
};

struct CellParams {
    int n;
    uint32_t m[ILRE_MAX_POOL_KERNELS], len[ILRE_MAX_POOL_KERNELS];
    uint64_t off[ILRE_MAX_POOL_KERNELS];
};

// Order-preserving map of a finite float onto uint32 (larger float -> larger key; the two zeros share one).
__device__ __forceinline__ uint32_t ordered_bits(float x)
{
    const uint32_t b = __float_as_uint(x + 0.0f);  // -0 ranks with +0
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ uint64_t make_key(float pooled, uint32_t token)
{
    return ((uint64_t)ordered_bits(pooled) << 32) | (uint64_t)(0xFFFFFFFFu - token);
}

__device__ __forceinline__ uint32_t key_token(uint64_t key) { return 0xFFFFFFFFu - (uint32_t)key; }

__device__ __forceinline__ uint32_t load_u32(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint64_t load_u64(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wavefront scans and reductions with DPP row shifts and row broadcasts: six plain vector instructions,
// where a shuffle-based version pays six trips through the LDS crossbar.
#define ILRE_DPP(old, x, ctrl, rows) __builtin_amdgcn_update_dpp((int)(old), (int)(x), ctrl, rows, 0xF, false)
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t x)  // inclusive prefix sum over the 64 lanes
{
    x += (uint32_t)ILRE_DPP(0, x, 0x111, 0xF);  // row_shr:1
    x += (uint32_t)ILRE_DPP(0, x, 0x112, 0xF);  // row_shr:2
    x += (uint32_t)ILRE_DPP(0, x, 0x114, 0xF);  // row_shr:4
    x += (uint32_t)ILRE_DPP(0, x, 0x118, 0xF);  // row_shr:8
    x += (uint32_t)ILRE_DPP(0, x, 0x142, 0xA);  // row_bcast:15 into rows 1 and 3
    x += (uint32_t)ILRE_DPP(0, x, 0x143, 0xC);  // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ uint32_t wave_total(uint32_t scanned)  // lane 63 of an inclusive scan, in every lane
{
    return (uint32_t)__builtin_amdgcn_readlane((int)scanned, 63);
}
template <bool IS_AND>
__device__ __forceinline__ uint32_t wave_bits32(uint32_t x)  // AND or OR over the 64 lanes, in every lane
{
    const uint32_t id = IS_AND ? 0xFFFFFFFFu : 0u;
#define ILRE_STEP(ctrl, rows)                                      \
    {                                                              \
        const uint32_t y = (uint32_t)ILRE_DPP(id, x, ctrl, rows);  \
        x = IS_AND ? (x & y) : (x | y);                            \
    }
    ILRE_STEP(0x111, 0xF) ILRE_STEP(0x112, 0xF) ILRE_STEP(0x114, 0xF) ILRE_STEP(0x118, 0xF) ILRE_STEP(0x142, 0xA) ILRE_STEP(0x143, 0xC)
#undef ILRE_STEP
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint64_t wave_and64(uint64_t x)
{
    return ((uint64_t)wave_bits32<true>((uint32_t)(x >> 32)) << 32) | wave_bits32<true>((uint32_t)x);
}
__device__ __forceinline__ uint64_t wave_or64(uint64_t x)
{
    return ((uint64_t)wave_bits32<false>((uint32_t)(x >> 32)) << 32) | wave_bits32<false>((uint32_t)x);
}

// Inclusive prefix sum over the THREADS threads of the block; wsum is THREADS / 64 words of LDS
// scratch.  Every thread also receives the block total.  Contains two barriers.
template <int THREADS>
__device__ __forceinline__ uint32_t block_scan_inclusive(uint32_t x, uint32_t *wsum, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    x = wave_scan_add(x);
    __syncthreads();  // protect wsum against a previous use
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) {
        const uint32_t s = wsum[w];
        if (w < wave) before += s;
        all += s;
    }
    total = all;
    return x + before;
}

__global__ __launch_bounds__(kThreads) void sel_init(const SelParams prm, uint32_t *hist, SelCtrl *ctrl, uint32_t *done)
{
    const int j = blockIdx.x;
    // hist holds [2][n][kSelBins]; block j clears its rows of both levels
    for (int i = threadIdx.x; i < kSelBins; i += kThreads) {
        hist[(size_t)j * kSelBins + i] = 0;
        hist[((size_t)prm.n + j) * kSelBins + i] = 0;
    }
    if (threadIdx.x == 0) {
        SelCtrl c{};
        c.want = prm.want[j];
        c.share = prm.share[j];
        c.before = prm.before[j];
        c.after = prm.after[j];
        c.bin1 = kSelBins;
        c.bin2 = kSelBins;
        c.len = prm.len[j];
        c.cell = prm.cell[j];
        c.op = prm.op;
        c.src_off = prm.src_off[j];
        c.tie_off = prm.tie_off[j];
        c.exact = prm.exact;
        ctrl[j] = c;
        done[j] = 0;          // [2][n]: workgroups finished per histogram level and combination
        done[prm.n + j] = 0;
    }
}

// MaxPooling of Algorithm 1 with size = stride = m: cell p = max(body[p*m .. p*m+m-1]) for the whole
// cells; the tokens after the last whole cell belong to none.  grid = (workgroups, max kernels).
__global__ __launch_bounds__(kPoolThreads) void cell_max(const float *body, const CellParams cp, float *cells)
{
    const int i = blockIdx.y;
    const uint32_t m = cp.m[i], len = cp.len[i];
    float *out = cells + cp.off[i];
    for (uint32_t p = blockIdx.x * kPoolThreads + threadIdx.x; p < len; p += gridDim.x * kPoolThreads) {
        const float *src = body + (size_t)p * m;
        float v = src[0];
        for (uint32_t u = 1; u < m; ++u) v = fmaxf(v, src[u]);
        out[p] = v;
    }
}

// The fine chunks (kSelFine elements) a pooling pass visits: all of the source array, or a list built
// by the pruning pre-pass.
struct Entries {
    const uint32_t *list;    // null: entry i is fine chunk i
    const uint32_t *list_n;  // device count of list entries
};
__device__ __forceinline__ uint32_t entry_count(const Entries &e, uint32_t len)
{
    return e.list ? load_u32(e.list_n) : (len + kSelFine - 1) / kSelFine;
}
__device__ __forceinline__ uint32_t entry_chunk(const Entries &e, uint32_t i) { return e.list ? e.list[i] : i; }

// A wavefront's LDS operations complete in order; waiting for them (and telling the compiler that
// memory changed) is all the synchronisation a wavefront-private buffer needs.
__device__ __forceinline__ void lds_wave_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// What a combination computes from its source array.
struct Pooling {
    const float *src;
    int64_t len;        // elements in src
    int before, after;  // window [e - before, e + after]
    int op;             // SelMode
};
__device__ __forceinline__ Pooling pooling_of(const float *vals, const SelCtrl &c)
{
    return Pooling{vals + c.src_off, (int64_t)c.len, (int)c.before, (int)c.after, (int)c.op};
}
__device__ __forceinline__ size_t pool_lds_floats(int before, int after) { return (size_t)(kSelFine + before + after); }

// Pooled values of this lane's kPerThread elements (lane + 64k) of fine chunk `fc`, computed by one
// wavefront in its own LDS buffers b0/b1 (kSelFine + before + after floats each).
//   kSelWindowMax: pooled[e] = max(src[u] : e - before <= u <= e + after, 0 <= u < len)  (MaxPooling at
//     stride 1, window clipped to the context).  Sliding maximum by doubling: m_p[i] = max(src[i ..
//     i+p-1]) for p = 1, 2, 4, ... <= w, then two overlapping windows of length p cover the window.
//   kSelMaxAvg: pooled[e] = (src[e-before] + ... + src[e+after]) / w with zeros outside the array,
//     summed left to right in fp32 and divided with round-to-nearest (AvgPooling at stride 1).
__device__ __forceinline__ void pooled_wave(const Pooling &pl, int64_t fc, float *b0, float *b1, float (&out)[kPerThread])
{
    const int lane = threadIdx.x & 63;
    const int len = kSelFine + pl.before + pl.after;
    const int64_t first = fc * kSelFine - pl.before;
    const float pad = pl.op == kSelMaxAvg ? 0.0f : -INFINITY;
    lds_wave_sync();  // the previous chunk's reads of these buffers are done
    // Loads are unconditional from a clamped address (padding is selected afterwards), so that a
    // lane's loads are all in flight together instead of one memory latency after the other.
    const int64_t last = pl.len - 1;
    auto clamped = [&](int64_t e) { return pl.src[e < 0 ? 0 : (e > last ? last : e)]; };
    {
        float v[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) v[k] = clamped(first + lane + k * 64);
        const int ih = kSelFine + lane;  // halo part: before + after <= 2 * 1023 elements
        const float vh = clamped(first + ih);
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int64_t e = first + lane + k * 64;
            b0[lane + k * 64] = (e >= 0 && e <= last) ? v[k] : pad;
        }
        if (ih < len) b0[ih] = (first + ih >= 0 && first + ih <= last) ? vh : pad;
        for (int i = ih + 64; i < len; i += 64) {
            const int64_t e = first + i;
            const float x = clamped(e);
            b0[i] = (e >= 0 && e <= last) ? x : pad;
        }
    }
    lds_wave_sync();
    const int w = pl.before + pl.after + 1;
    if (pl.op == kSelMaxAvg) {
        float sum[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) sum[k] = 0.0f;
        for (int u = 0; u < w; ++u) {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) sum[k] = sum[k] + b0[lane + k * 64 + u];
        }
        const float div = (float)w;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) out[k] = __fdiv_rn(sum[k], div);
        return;
    }
    int p = 1;
    float *src = b0, *dst = b1;
    while (2 * p <= w) {
        for (int i = lane; i < len; i += 64) dst[i] = (i + p < len) ? fmaxf(src[i], src[i + p]) : src[i];
        lds_wave_sync();
        float *t = src;
        src = dst;
        dst = t;
        p *= 2;
    }
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int tl = lane + k * 64;
        out[k] = fmaxf(src[tl], src[tl + w - p]);
    }
}

// For combination j: the bin b with  count(bins > b) < need <= count(bins >= b), by one wavefront.
// Lane l sums 32 bins (descending order of bins); a scan over the lanes finds the lane whose segment
// holds the crossing, and a second scan over that segment's 32 bins (one bin a lane) finds the bin.
// LEVEL 1 reads `want`, LEVEL 2 the remainder left by level 1.
template <int LEVEL>
__device__ void find_bins(const uint32_t *hist, SelCtrl *ctrl, int j)
{
    const int lane = threadIdx.x & 63;
    constexpr int BPL = kSelBins / 64;
    static_assert(BPL == 32, "the second scan maps one bin of a segment to each of 32 lanes");
    if (threadIdx.x < 64) {
        const uint32_t need = LEVEL == 1 ? ctrl[j].want : ctrl[j].need1;
        if (need == 0 || (LEVEL == 2 && ctrl[j].bin1 >= (uint32_t)kSelBins)) return;  // uniform in the wave
        const uint32_t *hj = hist + (size_t)j * kSelBins;
        uint32_t sum = 0;
#pragma unroll 16
        for (int k = 0; k < BPL; ++k) sum += load_u32(&hj[kSelBins - 1 - (lane * BPL + k)]);
        const uint32_t incl = wave_scan_add(sum);
        const uint64_t hit = __ballot(incl - sum < need && need <= incl);
        if (hit == 0) return;  // fewer than `need` keys in all (never: need <= number of elements)
        const int seg = __ffsll((unsigned long long)hit) - 1;
        const uint32_t seg_above = (uint32_t)__builtin_amdgcn_readlane((int)(incl - sum), seg);
        const uint32_t bin = kSelBins - 1 - (seg * BPL + (lane & 31));
        const uint32_t own = lane < 32 ? load_u32(&hj[bin]) : 0u;
        const uint32_t in2 = wave_scan_add(own);  // lanes 32.. hold zeros and are not looked at
        const uint32_t above = seg_above + in2 - own;
        if (lane < 32 && above < need && need <= above + own) {  // exactly one lane
            if (LEVEL == 1) {
                ctrl[j].bin1 = bin;
                ctrl[j].above1 = above;
                ctrl[j].need1 = need - above;
            } else {
                ctrl[j].bin2 = bin;
                ctrl[j].above2 = above;
                ctrl[j].need2 = need - above;
            }
        }
    }
}

// Append the selected items of a wavefront to a list: one slot reservation per wavefront.
template <typename T>
__device__ __forceinline__ void wave_append(bool pred, T item, T *list, uint32_t *counter)
{
    const uint64_t mask = __ballot(pred);
    if (mask == 0) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((unsigned long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(mask));
    base = (uint32_t)__builtin_amdgcn_readlane((int)base, leader);
    if (pred) list[base + __popcll(mask & ((1ull << lane) - 1ull))] = item;
}

// LEVEL 1: histogram of key bits 31..21 over the visited elements.  LEVEL 2: of bits 20..10 over the
// elements whose bits 31..21 equal the combination's level-1 bin.  grid = (workgroups, combinations);
// the wavefronts of a grid row share out the entries.
template <int LEVEL>
__global__ __launch_bounds__(kPoolThreads) void pool_hist(const float *vals, int n, SelCtrl *ctrl, uint32_t *hist_all,
                                                          uint32_t *done, const Entries ent)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t lh[kSelBins];
    __shared__ uint32_t is_last;
    const int j = blockIdx.y;
    const Pooling pl = pooling_of(vals, ctrl[j]);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t *hist = hist_all + (size_t)(LEVEL - 1) * n * kSelBins;
    float *b0 = (float *)smem + (size_t)wave * 2 * pool_lds_floats(pl.before, pl.after);
    float *b1 = b0 + pool_lds_floats(pl.before, pl.after);
    const uint32_t bin1 = LEVEL == 2 ? ctrl[j].bin1 : 0;
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) lh[i] = 0;
    __syncthreads();
    const uint32_t nent = entry_count(ent, (uint32_t)pl.len);
    for (uint32_t e = blockIdx.x * kPoolWaves + wave; e < nent; e += gridDim.x * kPoolWaves) {
        const int64_t fc = entry_chunk(ent, e);
        float pooled[kPerThread];
        pooled_wave(pl, fc, b0, b1, pooled);
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int64_t el = fc * kSelFine + lane + k * 64;
            const uint32_t key = ordered_bits(pooled[k]);
            if (LEVEL == 1) {
                // Real score distributions put most of a wavefront's 64 keys into one or two bins, and
                // same-address LDS atomics serialise: the two most common bins are counted with ballots
                // and added once, whatever is left goes one by one.
                const uint32_t bin = key >> 21;
                bool todo = el < pl.len;
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const uint64_t open = __ballot(todo);
                    if (open == 0) break;  // uniform
                    const int leader = __ffsll((unsigned long long)open) - 1;
                    const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
                    const uint64_t same = __ballot(todo && bin == b0);
                    if (lane == leader) atomicAdd(&lh[b0], (uint32_t)__popcll(same));
                    todo = todo && bin != b0;
                }
                if (todo) atomicAdd(&lh[bin], 1u);
            } else if (el < pl.len && (key >> 21) == bin1) {
                atomicAdd(&lh[(key >> 10) & (kSelBins - 1)], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hist[(size_t)j * kSelBins + i], c);
    }
    // The last workgroup of combination j to get here sees its histogram complete and locates the bin.  Each
    // thread waits until its histogram atomics have been performed, then one thread counts the workgroup in
    // (fences here cost tens of microseconds: an agent-scope release writes the L2 back).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        is_last = __hip_atomic_fetch_add(&done[(LEVEL - 1) * n + j], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                  gridDim.x - 1;
    __syncthreads();
    if (is_last) find_bins<LEVEL>(hist, ctrl, j);
}

__global__ __launch_bounds__(kPoolThreads) void collect(const float *vals, SelCtrl *ctrl, uint64_t *cand, uint64_t *tie,
                                                        const Entries ent)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int j = blockIdx.y;
    const Pooling pl = pooling_of(vals, ctrl[j]);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t bin1 = ctrl[j].bin1, bin2 = ctrl[j].bin2;
    if (bin1 >= (uint32_t)kSelBins || bin2 >= (uint32_t)kSelBins) return;  // nothing wanted from this combination
    const uint32_t prefix = (bin1 << 11) | bin2;  // 22-bit prefix of the K_j-th largest key
    float *b0 = (float *)smem + (size_t)wave * 2 * pool_lds_floats(pl.before, pl.after);
    float *b1 = b0 + pool_lds_floats(pl.before, pl.after);
    uint64_t *cand_j = cand + (size_t)j * kCandCap;
    uint64_t *tie_j = tie + ctrl[j].tie_off;
    const uint32_t nent = entry_count(ent, (uint32_t)pl.len);
    for (uint32_t e = blockIdx.x * kPoolWaves + wave; e < nent; e += gridDim.x * kPoolWaves) {
        const int64_t fc = entry_chunk(ent, e);
        float pooled[kPerThread];
        pooled_wave(pl, fc, b0, b1, pooled);
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int64_t el = fc * kSelFine + lane + k * 64;
            const bool valid = el < pl.len;
            const uint32_t p22 = valid ? ordered_bits(pooled[k]) >> 10 : 0;
            const uint64_t key = make_key(pooled[k], (uint32_t)el);
            wave_append(valid && p22 > prefix, key, cand_j, &ctrl[j].cand_n);
            wave_append(valid && p22 == prefix, key, tie_j, &ctrl[j].tie_n);
        }
    }
}

// Pruning pre-pass for long contexts, step 1: cm[c] = max of the scores of fine chunk c.  Pure
// streaming; a wavefront reads four chunks (4 KiB) per iteration.
__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true)));   // quad 1,0,3,2
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, true)));   // quad 2,3,0,1
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, true)));  // row_half_mirror
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, true)));  // row_mirror
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

__global__ __launch_bounds__(kPoolThreads) void chunk_max(const float *scores, int64_t L, uint32_t nfine, float *cm)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t stride = gridDim.x * kPoolWaves * 4;
    for (uint32_t c0 = (blockIdx.x * kPoolWaves + wave) * 4; c0 < nfine; c0 += stride) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t tok = (int64_t)(c0 + u) * kSelFine + lane * 4;
            if (tok + 3 < L) {
                v[u] = *(const float4 *)(scores + tok);
            } else {
                v[u].x = tok + 0 < L ? scores[tok + 0] : -INFINITY;
                v[u].y = tok + 1 < L ? scores[tok + 1] : -INFINITY;
                v[u].z = tok + 2 < L ? scores[tok + 2] : -INFINITY;
                v[u].w = -INFINITY;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float m = wave_max(fmaxf(fmaxf(v[u].x, v[u].y), fmaxf(v[u].z, v[u].w)));
            if (lane == 0 && c0 + u < nfine) cm[c0 + u] = m;
        }
    }
}

// Pruning pre-pass, step 3 (step 2 is the two-level histogram run on cm for the `budget`-th largest
// chunk maximum): at least `budget` tokens score at or above the lower edge of that maximum's 22-bit
// prefix, so no kernel admits a token whose pooled score is below it; a fine chunk can only hold such
// a token if a chunk maximum within `reach` chunks of it reaches the prefix.
__global__ __launch_bounds__(kPoolThreads) void mark_active(const float *cm, uint32_t nfine, int reach, SelCtrl *pctrl,
                                                            uint32_t *list)
{
    const uint32_t c = blockIdx.x * kPoolThreads + threadIdx.x;
    const uint32_t bin1 = pctrl->bin1, bin2 = pctrl->bin2;
    const uint32_t prefix = (bin1 >= (uint32_t)kSelBins || bin2 >= (uint32_t)kSelBins) ? 0u : (bin1 << 11) | bin2;
    bool active = false;
    if (c < nfine) {
        float m = cm[c];
        for (int d = 1; d <= reach; ++d) {
            if (c >= (uint32_t)d) m = fmaxf(m, cm[c - d]);
            if (c + d < nfine) m = fmaxf(m, cm[c + d]);
        }
        active = (ordered_bits(m) >> 10) >= prefix;
    }
    wave_append(active, c, list, &pctrl->cand_n);
}

// Boundary list -> candidates.  Window-max form: short lists (the normal case) are appended whole,
// candidates below the cut are harmless, they rank last; long ones are radix-selected down first.
// Printed form: the list is always cut to what the K_m-cell cap leaves.
__global__ __launch_bounds__(kThreads) void refine(SelCtrl *ctrl, uint64_t *cand, uint64_t *tie, uint32_t sort_n)
{
    __shared__ uint32_t h[256];
    __shared__ uint32_t cnt[2];
    __shared__ uint32_t pick[3];  // digit, count above it, count in it

    const int j = blockIdx.x;
    uint64_t *cand_j = cand + (size_t)j * kCandCap;
    uint64_t *A = tie + ctrl[j].tie_off;
    uint64_t *B = A + ctrl[j].len;
    uint32_t nA = ctrl[j].tie_n;
    uint32_t need = ctrl[j].need2;
    uint32_t candn = ctrl[j].cand_n;
    const uint32_t keep_small = ctrl[j].exact ? 0u : (uint32_t)kSelSmall;
    const int lane = threadIdx.x & 63;

    // The list shares its top 22 key bits (key64 bits 63..42).  Peel 8 more bits a pass.
    for (int shift = 40; shift >= 0 && nA > keep_small && need < nA; shift -= 8) {
        if (threadIdx.x < 256) h[threadIdx.x] = 0;
        if (threadIdx.x < 2) cnt[threadIdx.x] = 0;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < nA; i += kThreads) atomicAdd(&h[(load_u64(&A[i]) >> shift) & 255u], 1u);
        __syncthreads();
        if (threadIdx.x < 64) {
            // lane l owns digits 255-4l .. 252-4l (descending); find the digit holding the need-th key
            uint32_t own[4], sum = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                own[k] = h[255 - (lane * 4 + k)];
                sum += own[k];
            }
            const uint32_t incl = wave_scan_add(sum);
            uint32_t above = incl - sum;
            if (above < need && need <= incl) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (above < need && need <= above + own[k]) {
                        pick[0] = 255 - (lane * 4 + k);
                        pick[1] = above;
                        pick[2] = own[k];
                    }
                    above += own[k];
                }
            }
        }
        __syncthreads();
        const uint32_t digit = pick[0], above = pick[1], inside = pick[2];
        const uint32_t rounds = (nA + kThreads - 1) / kThreads;
        for (uint32_t it = 0; it < rounds; ++it) {
            const uint32_t i = it * kThreads + threadIdx.x;
            const bool valid = i < nA;
            const uint64_t key = valid ? load_u64(&A[i]) : 0;
            const uint32_t d = (uint32_t)(key >> shift) & 255u;
            wave_append(valid && d > digit, key, cand_j + candn, &cnt[0]);
            wave_append(valid && d == digit, key, B, &cnt[1]);
        }
        // The survivors go through global memory to the next pass of this same workgroup: wait until
        // the stores have reached the L2 and read them back past the L1 (load_u64).  A fence would do
        // too, at the price of an L2 write-back per pass.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        candn += above;
        need -= above;
        nA = inside;
        uint64_t *t = A;
        A = B;
        B = t;
    }
    for (uint32_t i = threadIdx.x; i < nA; i += kThreads) cand_j[candn + i] = load_u64(&A[i]);
    const uint32_t total = candn + nA;
    if (threadIdx.x == 0) ctrl[j].total_n = total;
    if (!ctrl[j].exact) return;  // uniform

    // Printed form: hand the candidates to the allocation walk in rank order.  Bitonic sort of the
    // keys (descending; padding keys of 0 sink to the end) in LDS, one barrier per stage.
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t *srt = (uint64_t *)smem;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this workgroup's stores to cand_j have reached the L2
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < sort_n; i += kThreads)
        srt[i] = i < total ? load_u64(&cand_j[i]) : 0ull;
    __syncthreads();
    for (uint32_t k = 2; k <= sort_n; k <<= 1) {
        for (uint32_t d = k >> 1; d > 0; d >>= 1) {
            for (uint32_t i = threadIdx.x; i < sort_n / 2; i += kThreads) {
                const uint32_t lo = ((i & ~(d - 1)) << 1) | (i & (d - 1)), hi = lo + d;
                const uint64_t a = srt[lo], b = srt[hi];
                const bool descending = (lo & k) == 0;
                if ((a < b) == descending) {
                    srt[lo] = b;
                    srt[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    // The allocation walk wants tokens: element e stands for tokens e*m .. e*m+m-1, in that order.  The
    // token list (uint32, total * m <= kCandCap entries) takes over the storage of the key list.
    uint32_t *tokens = (uint32_t *)cand_j;
    const uint32_t m = ctrl[j].cell;
    for (uint32_t r = threadIdx.x; r < total * m; r += kThreads) {
        const uint32_t el = r / m;
        tokens[r] = key_token(srt[el]) * m + (r - el * m);
    }
}

__device__ __forceinline__ uint32_t hash_slot(uint32_t token) { return (token * 0x9E3779B1u) >> 18; }

// The allocated set I of Algorithm 1 as an open-addressing hash set of token indices in LDS.
__device__ __forceinline__ bool is_allocated(const uint32_t *table, uint32_t token)
{
    uint32_t s = hash_slot(token);
    while (true) {
        const uint32_t t = table[s];
        if (t == kEmpty) return false;
        if (t == token) return true;
        s = (s + 1) & (kHashSlots - 1);
    }
}
__device__ __forceinline__ void mark_allocated(uint32_t *table, uint32_t token)
{
    uint32_t s = hash_slot(token);
    while (true) {
        const uint32_t old = atomicCAS(&table[s], kEmpty, token);
        if (old == kEmpty || old == token) break;
        s = (s + 1) & (kHashSlots - 1);
    }
}

// Last step of both allocation kernels: the sink indices, then the nsel allocated tokens in ascending
// order (counting sort on the high bits into kBuckets buckets, then each token's rank inside its bucket
// by counting the smaller ones: deterministic whatever order the tokens arrived in), then -1 up to
// sink + n_out.  table (the hash set, no longer needed) and the second half of sel are scratch.
template <int THREADS>
__device__ __forceinline__ void emit_ascending(uint32_t *table, uint32_t *sel, uint32_t *wsum, uint32_t nsel, int n_out,
                                               int sink, int bucket_shift, int32_t *out_idx, int32_t *out_count)
{
    uint32_t *cnt = table;                  // the hash set is no longer needed
    uint32_t *start = table + kBuckets;
    uint32_t *fill = table + 2 * kBuckets;
    uint32_t *grp = sel + ILRE_MAX_BUDGET;
    for (int i = threadIdx.x; i < kBuckets; i += THREADS) {
        cnt[i] = 0;
        fill[i] = 0;
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nsel; i += THREADS) atomicAdd(&cnt[sel[i] >> bucket_shift], 1u);
    __syncthreads();
    {
        constexpr int BPT = kBuckets / THREADS;
        uint32_t own[BPT], sum = 0;
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            own[k] = cnt[threadIdx.x * BPT + k];
            sum += own[k];
        }
        uint32_t total;
        uint32_t run = block_scan_inclusive<THREADS>(sum, wsum, total) - sum;
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            start[threadIdx.x * BPT + k] = run;
            run += own[k];
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nsel; i += THREADS) {
        const uint32_t t = sel[i], bkt = t >> bucket_shift;
        grp[start[bkt] + atomicAdd(&fill[bkt], 1u)] = t;
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nsel; i += THREADS) {
        const uint32_t t = grp[i], bkt = t >> bucket_shift;
        const uint32_t s0 = start[bkt], s1 = s0 + cnt[bkt];
        uint32_t rank = s0;
        for (uint32_t q = s0; q < s1; ++q) rank += grp[q] < t ? 1u : 0u;
        out_idx[sink + rank] = (int32_t)(t + sink);
    }
    for (int i = threadIdx.x; i < sink; i += THREADS) out_idx[i] = i;
    for (int i = nsel + threadIdx.x; i < n_out; i += THREADS) out_idx[sink + i] = -1;
    if (threadIdx.x == 0 && out_count) *out_count = sink + (int32_t)nsel;
}

// Algorithm 1's walk, window-max form: kernels in the order given; from kernel j's candidates the B_j
// largest keys whose tokens are not yet allocated; then the output.
__global__ __launch_bounds__(kThreads) void allocate(const SelCtrl *ctrl, const uint64_t *cand, int n, int n_out, int sink,
                                                     int bucket_shift, int32_t *out_idx, int32_t *out_count)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = (uint32_t *)smem;  // kHashSlots
    uint32_t *sel = table + kHashSlots;  // ILRE_MAX_BUDGET tokens, then as many again for the final sort
    __shared__ uint32_t wsum[kThreads / 64];
    __shared__ uint64_t red[2][3][kThreads / 64];  // per-wave (count, and, or), two generations
    __shared__ uint32_t h[3][256];                 // digit histograms, three generations
    __shared__ uint32_t nsel_ctr;
    constexpr int kDirect = 128;                   // a threshold bin this small is ranked directly
    __shared__ uint64_t small[kDirect];
    __shared__ uint64_t small_thr;
    __shared__ uint32_t small_n;

    for (int i = threadIdx.x; i < kHashSlots; i += kThreads) table[i] = kEmpty;
    if (threadIdx.x < 256) h[0][threadIdx.x] = h[1][threadIdx.x] = h[2][threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        nsel_ctr = 0;
        small_n = 0;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    uint64_t key[kKeysPerThread];
    auto fetch = [&](int j, uint64_t(&dst)[kKeysPerThread]) {
        const uint32_t cn = ctrl[j].total_n;
        const uint64_t *cand_j = cand + (size_t)j * kCandCap;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k) {
            const uint32_t i = threadIdx.x + k * kThreads;  // < kCandCap: always inside the list's storage
            dst[k] = cand_j[i];
        }
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k)
            if (threadIdx.x + k * kThreads >= cn) dst[k] = 0;  // 0 is below every real key
    };
    __syncthreads();

    uint32_t nsel = 0;
    int gen = 0, hgen = 0;  // generations of red[] and h[], advanced uniformly
    for (int j = 0; j < n; ++j) {
        uint32_t share = ctrl[j].share;
        if ((uint32_t)n_out - nsel < share) share = (uint32_t)n_out - nsel;
        if (share == 0) continue;  // uniform
        fetch(j, key);

        // which of this thread's candidates are still free
        uint32_t free_mask = 0, nfree = 0;
        uint64_t vand = ~0ull, vor = 0;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k) {
            if (key[k] == 0) continue;
            if (!is_allocated(table, key_token(key[k]))) {
                free_mask |= 1u << k;
                ++nfree;
                vand &= key[k];
                vor |= key[k];
            }
        }
        // block-wide count, AND and OR of the free keys: one exchange through LDS
        const uint64_t c64 = wave_total(wave_scan_add(nfree));
        vand = wave_and64(vand);
        vor = wave_or64(vor);
        if (lane == 0) {
            red[gen][0][wave] = c64;
            red[gen][1][wave] = vand;
            red[gen][2][wave] = vor;
        }
        __syncthreads();
        uint64_t total_free = 0, all_and = ~0ull, all_or = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) {
            total_free += red[gen][0][w];
            all_and &= red[gen][1][w];
            all_or |= red[gen][2][w];
        }
        gen ^= 1;
        const uint32_t take = share < (uint32_t)total_free ? share : (uint32_t)total_free;
        if (take == 0) continue;  // uniform

        // threshold: the take-th largest free key.  Radix select, 8 bits a pass, from the highest bit
        // in which the free keys differ; keys are distinct, so it ends with exactly `take` keys at or
        // above the threshold.  One barrier per pass: every wavefront locates the digit itself, and the
        // histogram two generations back is cleared while the current one fills.
        uint64_t thr = 0;
        if (take < (uint32_t)total_free) {
            const uint64_t diff = all_and ^ all_or;  // != 0: at least two distinct keys
            int shift = 63 - __clzll((long long)diff) - 7;
            if (shift < 0) shift = 0;
            uint64_t pmask = shift + 8 >= 64 ? 0ull : ~0ull << (shift + 8);
            uint64_t prefix = all_and & pmask;
            uint32_t need = take;
            bool direct = false;
            while (true) {
                uint32_t *hc = h[hgen];
                if (threadIdx.x < 256) h[(hgen + 1) % 3][threadIdx.x] = 0;
#pragma unroll
                for (int k = 0; k < kKeysPerThread; ++k)
                    if (((free_mask >> k) & 1u) && (key[k] & pmask) == prefix) atomicAdd(&hc[(key[k] >> shift) & 255u], 1u);
                __syncthreads();
                // lane l owns digits 255-4l .. 252-4l (descending)
                uint32_t own[4], sum = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    own[k] = hc[255 - (lane * 4 + k)];
                    sum += own[k];
                }
                const uint32_t incl = wave_scan_add(sum);
                uint32_t above = incl - sum;
                uint32_t found = 0;  // digit | inside << 8 (inside <= kCandCap) ; above kept separately
                uint32_t found_above = 0;
                if (above < need && need <= incl) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (above < need && need <= above + own[k]) {
                            found = (255u - (lane * 4 + k)) | (own[k] << 8) | 0x80000000u;
                            found_above = above;
                        }
                        above += own[k];
                    }
                }
                const uint64_t who = __ballot(found != 0);
                const int src_lane = __ffsll((unsigned long long)who) - 1;
                found = (uint32_t)__builtin_amdgcn_readlane((int)found, src_lane);
                found_above = (uint32_t)__builtin_amdgcn_readlane((int)found_above, src_lane);
                const uint32_t digit = found & 255u, inside = (found >> 8) & 0x7FFFFFu;
                hgen = (hgen + 1) % 3;
                prefix |= (uint64_t)digit << shift;
                pmask |= 255ull << shift;
                need -= found_above;
                if (need == inside || shift == 0) break;  // the whole digit bin is taken
                if (inside <= (uint32_t)kDirect) {
                    direct = true;  // few keys left in the bin: rank them against each other instead
                    break;
                }
                shift = shift >= 8 ? shift - 8 : 0;  // the last digit may overlap the one before: harmless
            }
            thr = prefix;
            if (direct) {  // uniform
                // The bin's keys go to a list; key i is the threshold if exactly need - 1 of the others
                // are larger (keys are distinct).  Two barriers instead of up to seven more passes when
                // the cut falls inside a plateau of equal pooled scores, where only index bits differ.
#pragma unroll
                for (int k = 0; k < kKeysPerThread; ++k)
                    if (((free_mask >> k) & 1u) && (key[k] & pmask) == prefix) small[atomicAdd(&small_n, 1u)] = key[k];
                __syncthreads();
                const uint32_t ns = small_n;  // == inside
                if (threadIdx.x < ns) {
                    const uint64_t mine = small[threadIdx.x];
                    uint32_t larger = 0;
                    for (uint32_t i = 0; i < ns; ++i) larger += small[i] > mine ? 1u : 0u;
                    if (larger == need - 1) small_thr = mine;
                }
                __syncthreads();
                thr = small_thr;
                if (threadIdx.x == 0) small_n = 0;  // next use lies behind the barrier that ends this kernel size
            }
        }

        // take every free key >= thr: one slot reservation per wavefront
        uint32_t take_mask = 0;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k)
            if (((free_mask >> k) & 1u) && key[k] >= thr) take_mask |= 1u << k;
        const uint32_t mine = (uint32_t)__popc(take_mask);
        const uint32_t incl = wave_scan_add(mine);
        uint32_t base = 0;
        if (lane == 63 && incl) base = atomicAdd(&nsel_ctr, incl);
        uint32_t pos = (uint32_t)__builtin_amdgcn_readlane((int)base, 63) + incl - mine;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k) {
            if ((take_mask >> k) & 1u) {
                const uint32_t token = key_token(key[k]);
                sel[pos++] = token;
                mark_allocated(table, token);
            }
        }
        __syncthreads();
        nsel = nsel_ctr;
    }
    __syncthreads();
    emit_ascending<kThreads>(table, sel, wsum, nsel, n_out, sink, bucket_shift, out_idx, out_count);
}

// LDS writes of this wavefront done, then the workgroup barrier; global loads in flight stay in flight.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Algorithm 1's walk, printed form.  refine left combination j's candidate tokens in rank order (a
// uint32 list in the storage of cand[j]).  Wavefront w owns the ranks [w*64*per,
// (w+1)*64*per), lane l the ranks w*64*per + 64*i + l.  Each wavefront counts its free tokens with
// ballots, one exchange through LDS gives every wavefront the number of free tokens ranked ahead of
// it, and the first B_j free tokens are taken.  The next combination's tokens are fetched meanwhile.
constexpr int kRankThreads = 1024;
constexpr int kRankWaves = kRankThreads / 64;
constexpr int kRankG = 5;                                                           // tokens of a lane are handled in groups
constexpr int kRankGroups = (kCandCap / kRankThreads + kRankG - 1) / kRankG;
constexpr int kRankPer = kRankGroups * kRankG;                                      // tokens per lane at most
static_assert(kRankPer <= 64, "free tokens of a lane are kept in a 64-bit mask");

__global__ __launch_bounds__(kRankThreads) void allocate_ranked(const SelCtrl *ctrl, const uint64_t *cand, int n, int n_out,
                                                                int sink, int bucket_shift, int32_t *out_idx,
                                                                int32_t *out_count)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = (uint32_t *)smem;  // kHashSlots
    uint32_t *sel = table + kHashSlots;  // ILRE_MAX_BUDGET tokens, then as many again for the final sort
    __shared__ uint32_t wsum[kRankWaves];
    __shared__ uint32_t wfree[2][kRankWaves];  // free tokens per wavefront, two generations
    __shared__ uint32_t c_share[ILRE_MAX_POOL_KERNELS], c_tokens[ILRE_MAX_POOL_KERNELS];

    for (int i = threadIdx.x; i < kHashSlots; i += kRankThreads) table[i] = kEmpty;
    if ((int)threadIdx.x < n) {
        c_share[threadIdx.x] = ctrl[threadIdx.x].share;
        c_tokens[threadIdx.x] = ctrl[threadIdx.x].total_n * ctrl[threadIdx.x].cell;  // <= kCandCap by the host's limits
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    __syncthreads();
    // At most (shares before j) tokens are allocated when combination j runs, so its B_j free tokens
    // are among its first (shares up to and including j) ranked ones: the rest is never looked at.
    if (threadIdx.x == 0) {
        uint32_t upto = 0;
        for (int j = 0; j < n; ++j) {
            upto += c_share[j];
            if (upto < c_tokens[j]) c_tokens[j] = upto;
        }
    }
    __syncthreads();

    // Loads are unconditional from a clamped slot of the list's storage, so that all are in flight
    // together; a whole group of kRankG tokens a lane is fetched when any of it is needed.
    auto fetch = [&](int j, uint32_t(&raw)[kRankPer]) {
        const uint32_t *list = (const uint32_t *)(cand + (size_t)j * kCandCap);
        const uint32_t per = (c_tokens[j] + kRankThreads - 1) / kRankThreads;
        const uint32_t base = (uint32_t)wave * per * 64u + (uint32_t)lane;
#pragma unroll
        for (int g = 0; g < kRankGroups; ++g) {
            if ((uint32_t)(g * kRankG) < per) {  // uniform
#pragma unroll
                for (int u = 0; u < kRankG; ++u) {
                    const uint32_t r = base + 64u * (g * kRankG + u);
                    raw[g * kRankG + u] = list[r < (uint32_t)kCandCap ? r : (uint32_t)kCandCap - 1u];
                }
            }
        }
    };

    uint32_t tok[kRankPer], nxt[kRankPer];
    if (n > 0) fetch(0, nxt);
    uint32_t nsel = 0;
    int gen = 0;
    for (int j = 0; j < n; ++j) {
#pragma unroll
        for (int i = 0; i < kRankPer; ++i) tok[i] = nxt[i];
        if (j + 1 < n) fetch(j + 1, nxt);
        uint32_t share = c_share[j];
        if ((uint32_t)n_out - nsel < share) share = (uint32_t)n_out - nsel;
        if (share == 0) continue;  // uniform
        const uint32_t cn = c_tokens[j];
        const uint32_t per = (cn + kRankThreads - 1) / kRankThreads;
        const uint32_t base = (uint32_t)wave * per * 64u + (uint32_t)lane;

        // Per group: the hash-set probes of all its tokens advance together, one round of LDS reads
        // per step of the longest probe chain, then the wavefront's count by ballots.
        uint64_t free_bits = 0;
        uint32_t run = 0;
#pragma unroll
        for (int g = 0; g < kRankGroups; ++g) {
            if ((uint32_t)(g * kRankG) < per) {  // uniform
                uint32_t slot[kRankG];
                uint32_t pend = 0;
#pragma unroll
                for (int u = 0; u < kRankG; ++u) {
                    const int i = g * kRankG + u;
                    slot[u] = hash_slot(tok[i]);
                    if ((uint32_t)i < per && base + 64u * i < cn) pend |= 1u << u;
                }
                while (__any(pend != 0)) {
                    uint32_t seen_tok[kRankG];
#pragma unroll
                    for (int u = 0; u < kRankG; ++u) seen_tok[u] = table[slot[u]];
#pragma unroll
                    for (int u = 0; u < kRankG; ++u) {
                        if ((pend >> u) & 1u) {
                            if (seen_tok[u] == kEmpty) {
                                free_bits |= 1ull << (g * kRankG + u);
                                pend &= ~(1u << u);
                            } else if (seen_tok[u] == tok[g * kRankG + u]) {
                                pend &= ~(1u << u);
                            } else {
                                slot[u] = (slot[u] + 1) & (kHashSlots - 1);
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kRankG; ++u) run += (uint32_t)__popcll(__ballot((free_bits >> (g * kRankG + u)) & 1ull));
            }
        }
        if (lane == 0) wfree[gen][wave] = run;
        lds_barrier();
        uint32_t before = 0, total_free = 0;
#pragma unroll
        for (int w = 0; w < kRankWaves; ++w) {
            const uint32_t c = wfree[gen][w];
            if (w < wave) before += c;
            total_free += c;
        }
        gen ^= 1;
        const uint32_t take = share < total_free ? share : total_free;
        const uint32_t quota = take > before ? take - before : 0u;  // of this wavefront's free tokens, in rank order
        uint32_t seen = 0;
#pragma unroll
        for (int g = 0; g < kRankGroups; ++g) {
            if ((uint32_t)(g * kRankG) < per && seen < quota) {  // uniform
#pragma unroll
                for (int u = 0; u < kRankG; ++u) {
                    const int i = g * kRankG + u;
                    const bool fr = (free_bits >> i) & 1ull;
                    const uint64_t mask = __ballot(fr);
                    const uint32_t pos = seen + (uint32_t)__popcll(mask & lanes_below);
                    if (fr && pos < quota) {
                        sel[nsel + before + pos] = tok[i];
                        mark_allocated(table, tok[i]);
                    }
                    seen += (uint32_t)__popcll(mask);
                }
            }
        }
        nsel += take;
        lds_barrier();  // the set is complete before the next combination probes it
    }
    __syncthreads();
    emit_ascending<kRankThreads>(table, sel, wsum, nsel, n_out, sink, bucket_shift, out_idx, out_count);
}

// Last line of Algorithm 1: the input IDs of the allocated tokens, C[I].  Unused index slots (-1) give -1.
__global__ __launch_bounds__(kPoolThreads) void gather_ids_kernel(const int32_t *ids, int64_t L, const int32_t *idx, int n,
                                                                  int32_t *out)
{
    const int i = blockIdx.x * kPoolThreads + threadIdx.x;
    if (i >= n) return;
    const int32_t t = idx[i];
    out[i] = (t >= 0 && t < L) ? ids[t] : -1;
}

}  // namespace

hipError_t launch_gather_ids(const int32_t *ids, int64_t L, const int32_t *idx, int n, int32_t *out, hipStream_t s)
{
    hipLaunchKernelGGL(gather_ids_kernel, dim3((n + kPoolThreads - 1) / kPoolThreads), dim3(kPoolThreads), 0, s, ids, L, idx, n, out);
    return hipGetLastError();
}

// Elements of combination j's source array and the tokens one element stands for.
static void combo_shape(const SelectJob &job, int j, int64_t &len, int &cell)
{
    if (job.mode == kSelMaxAvg) {
        cell = job.max_kernels[j / job.n_avg];
        len = job.L / cell;
    } else {
        cell = 1;
        len = job.L;
    }
}

SelectLayout make_select_layout(const SelectJob &job)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    SelectLayout lay{};
    const int n = job.combos() > 0 ? job.combos() : 1;
    const size_t nfine = (size_t)((job.L + kSelFine - 1) / kSelFine);
    size_t off = 0;
    lay.hist = off;
    off = up(off + 2 * (size_t)(n + 1) * kSelBins * sizeof(uint32_t));  // + the pre-pass's own pair
    lay.ctrl = off;
    off = up(off + (size_t)(n + 1) * sizeof(SelCtrl));
    lay.done = off;
    off = up(off + 2 * (size_t)(n + 1) * sizeof(uint32_t));
    lay.cmax = off;
    off = up(off + nfine * sizeof(float));
    lay.active = off;
    off = up(off + nfine * sizeof(uint32_t));
    lay.cells = off;
    size_t ncell = 0, ntie = 0;
    if (job.mode == kSelMaxAvg) {
        for (int i = 0; i < job.n_max; ++i) ncell += (size_t)(job.L / job.max_kernels[i]);
        ntie = 2 * ncell * (size_t)job.n_avg;
    } else {
        ntie = 2 * (size_t)job.L * (size_t)n;
    }
    off = up(off + ncell * sizeof(float));
    lay.cand = off;
    off = up(off + (size_t)n * kCandCap * sizeof(uint64_t));
    lay.tie = off;
    off = up(off + ntie * sizeof(uint64_t));
    lay.total = off;
    return lay;
}

hipError_t launch_select(const float *scores, const SelectJob &job, int32_t *out_idx, int32_t *out_count,
                         void *workspace, const SelectLayout &lay, hipStream_t s)
{
    const int64_t L = job.L;
    const int n = job.combos();
    const int budget = job.budget;
    const int n_out = (int)(budget < L ? budget : L);
    unsigned char *ws = (unsigned char *)workspace;
    uint32_t *hist = (uint32_t *)(ws + lay.hist);
    SelCtrl *ctrl = (SelCtrl *)(ws + lay.ctrl);
    uint32_t *done = (uint32_t *)(ws + lay.done);
    uint64_t *cand = (uint64_t *)(ws + lay.cand);
    uint64_t *tie = (uint64_t *)(ws + lay.tie);
    float *cells = (float *)(ws + lay.cells);
    const size_t alloc_lds = (size_t)kHashSlots * sizeof(uint32_t) + 2 * (size_t)ILRE_MAX_BUDGET * sizeof(uint32_t);
    int bucket_shift = 0;
    while (((int64_t)kBuckets << bucket_shift) < L) ++bucket_shift;

    // Dynamic LDS ceilings are the same constants on every call (idempotent, so concurrent callers agree).
    constexpr int kPoolLdsMax = kPoolWaves * 2 * (kSelFine + 2 * (ILRE_MAX_AVG_KERNEL > ILRE_MAX_POOL_KERNEL ? ILRE_MAX_AVG_KERNEL : ILRE_MAX_POOL_KERNEL)) * (int)sizeof(float);
    constexpr int kSortLdsMax = 16384 * (int)sizeof(uint64_t);  // >= ILRE_MAX_BUDGET + 1 keys, padded to a power of two
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void *)allocate, hipFuncAttributeMaxDynamicSharedMemorySize, (int)alloc_lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)allocate_ranked, hipFuncAttributeMaxDynamicSharedMemorySize, (int)alloc_lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)pool_hist<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)pool_hist<2>, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)collect, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)refine, hipFuncAttributeMaxDynamicSharedMemorySize, kSortLdsMax)) != hipSuccess) return e;
    if (L == 0) {  // nothing but the sink part
        hipLaunchKernelGGL(allocate_ranked, dim3(1), dim3(kRankThreads), alloc_lds, s, ctrl, cand, 0, 0, job.sink, 0, out_idx, out_count);
        return hipGetLastError();
    }

    // B_c: floor(B / n), the first B mod n combinations one more.  K_j: window-max form, what the
    // earlier shares could have taken plus the own share; printed form, K_m = B / m + 1 cells.
    SelParams prm{};
    CellParams cp{};
    prm.n = n;
    prm.op = (uint32_t)job.mode;
    prm.exact = job.mode == kSelMaxAvg ? 1u : 0u;
    const int base = budget / n, rem = budget % n;
    int64_t before = 0, tie_off = 0, len_max = 0;
    int halo_max = 0;
    uint64_t cell_off = 0;
    for (int j = 0; j < n; ++j) {
        const int share = base + (j < rem ? 1 : 0);
        int64_t len;
        int cell;
        combo_shape(job, j, len, cell);
        prm.share[j] = (uint32_t)share;
        prm.len[j] = (uint32_t)len;
        prm.cell[j] = (uint32_t)cell;
        prm.tie_off[j] = (uint64_t)tie_off;
        tie_off += 2 * len;
        if (job.mode == kSelMaxAvg) {
            const int i = j / job.n_avg, na = job.avg_kernels[j % job.n_avg];
            if (j % job.n_avg == 0) {
                cp.m[i] = (uint32_t)cell;
                cp.len[i] = (uint32_t)len;
                cp.off[i] = cell_off;
                cell_off += (uint64_t)len;
            }
            // K_m = B / m + 1 cells are candidates; of those the walk can only reach the first
            // ceil((shares up to and including this one) / m): at most (shares before) tokens are taken
            // when it starts and it stops after B_c free ones.  Only that many are found and sorted.
            int64_t km = (int64_t)budget / cell + 1;
            const int64_t reach = (before + share + cell - 1) / cell;
            if (reach < km) km = reach;
            prm.want[j] = (uint32_t)(km < len ? km : len);
            prm.before[j] = (uint32_t)((na - 1) / 2);
            prm.after[j] = (uint32_t)(na / 2);
            prm.src_off[j] = cp.off[i];
        } else {
            const int64_t want = before + share < L ? before + share : L;
            prm.want[j] = (uint32_t)want;
            prm.before[j] = prm.after[j] = (uint32_t)((job.max_kernels[j] - 1) / 2);
            prm.src_off[j] = 0;
        }
        before += share;
        if ((int)(prm.before[j] + prm.after[j]) > halo_max) halo_max = (int)(prm.before[j] + prm.after[j]);
        if (len > len_max) len_max = len;
    }
    cp.n = job.n_max;
    uint32_t sort_n = 0;  // printed form: candidates are sorted in LDS, padded to a power of two
    if (job.mode == kSelMaxAvg) {
        sort_n = 2;
        for (int j = 0; j < n; ++j)
            while (sort_n < prm.want[j]) sort_n *= 2;
    }
    const float *vals = job.mode == kSelMaxAvg ? cells : scores;
    const uint32_t nfine = (uint32_t)((len_max + kSelFine - 1) / kSelFine);
    const size_t pool_lds = (size_t)kPoolWaves * 2 * (size_t)(kSelFine + halo_max) * sizeof(float);
    // Workgroups per combination in the pooling passes; beyond the cap the wavefronts loop over the
    // entries.  A histogram workgroup carries fixed work (clearing and flushing 2048 bins, one atomic per
    // hot bin on a handful of addresses, about 13 ns each and serialised, the completion counter), so
    // those passes aim at about one resident round of workgroups over all combinations.
    auto pool_blocks = [](uint32_t entries, uint32_t cap) {
        const uint32_t want = (entries + kPoolWaves - 1) / kPoolWaves;
        return want < cap ? (want ? want : 1u) : cap;
    };
    auto clamp_u32 = [](uint32_t x, uint32_t lo, uint32_t hi) { return x < lo ? lo : (x > hi ? hi : x); };
    constexpr uint32_t kHistGrid = 2560, kCollectGrid = 8192;

    Entries ent{nullptr, nullptr};
    uint32_t entries = nfine;
    if (job.mode == kSelMaxAvg) {
        uint32_t cb = (uint32_t)((len_max + kPoolThreads - 1) / kPoolThreads);
        if (cb > 2048u) cb = 2048u;
        if (cb) hipLaunchKernelGGL(cell_max, dim3(cb, job.n_max), dim3(kPoolThreads), 0, s, scores, cp, cells);
    } else if ((int64_t)nfine >= 4 * (int64_t)n_out && nfine >= 16384) {
        // Long contexts: visit only the fine chunks that can hold an admitted token.
        float *cm = (float *)(ws + lay.cmax);
        uint32_t *active = (uint32_t *)(ws + lay.active);
        uint32_t *phist = hist + 2 * (size_t)n * kSelBins;
        SelCtrl *pctrl = ctrl + n;
        uint32_t *pdone = done + 2 * (size_t)n;
        SelParams pp{};
        pp.n = 1;
        pp.len[0] = nfine;
        pp.cell[0] = 1;
        pp.want[0] = (uint32_t)n_out;
        const uint32_t nfine2 = (nfine + kSelFine - 1) / kSelFine;
        const Entries all{nullptr, nullptr};
        const size_t lds0 = (size_t)kPoolWaves * 2 * kSelFine * sizeof(float);
        hipLaunchKernelGGL(chunk_max, dim3(2048), dim3(kPoolThreads), 0, s, scores, L, nfine, cm);
        hipLaunchKernelGGL(sel_init, dim3(1), dim3(kThreads), 0, s, pp, phist, pctrl, pdone);
        hipLaunchKernelGGL(pool_hist<1>, dim3(pool_blocks(nfine2, 1024), 1), dim3(kPoolThreads), lds0, s, cm, 1, pctrl, phist, pdone, all);
        hipLaunchKernelGGL(pool_hist<2>, dim3(pool_blocks(nfine2, 1024), 1), dim3(kPoolThreads), lds0, s, cm, 1, pctrl, phist, pdone, all);
        const int reach = (halo_max / 2 + kSelFine - 1) / kSelFine;
        hipLaunchKernelGGL(mark_active, dim3((nfine + kPoolThreads - 1) / kPoolThreads), dim3(kPoolThreads), 0, s, cm, nfine, reach, pctrl, active);
        ent = Entries{active, &pctrl->cand_n};
        // with a list the entry count is only known on the device: size the grid for the worst case the
        // pruning rule is meant for (a few times the budget) and let the wavefronts loop
        entries = 4u * (uint32_t)n_out + 1024u;
    }
    const uint32_t hcap = clamp_u32(kHistGrid / (uint32_t)n, 32u, 256u), ccap = clamp_u32(kCollectGrid / (uint32_t)n, 64u, 1024u);
    const uint32_t hblocks = pool_blocks(entries, hcap), cblocks = pool_blocks(entries, ccap);

    hipLaunchKernelGGL(sel_init, dim3(n), dim3(kThreads), 0, s, prm, hist, ctrl, done);
    hipLaunchKernelGGL(pool_hist<1>, dim3(hblocks, n), dim3(kPoolThreads), pool_lds, s, vals, n, ctrl, hist, done, ent);
    hipLaunchKernelGGL(pool_hist<2>, dim3(hblocks, n), dim3(kPoolThreads), pool_lds, s, vals, n, ctrl, hist, done, ent);
    hipLaunchKernelGGL(collect, dim3(cblocks, n), dim3(kPoolThreads), pool_lds, s, vals, ctrl, cand, tie, ent);
    hipLaunchKernelGGL(refine, dim3(n), dim3(kThreads), (size_t)sort_n * sizeof(uint64_t), s, ctrl, cand, tie, sort_n);
    if (job.mode == kSelMaxAvg)
        hipLaunchKernelGGL(allocate_ranked, dim3(1), dim3(kRankThreads), alloc_lds, s, ctrl, cand, n, n_out, job.sink, bucket_shift, out_idx, out_count);
    else
        hipLaunchKernelGGL(allocate, dim3(1), dim3(kThreads), alloc_lds, s, ctrl, cand, n, n_out, job.sink, bucket_shift, out_idx, out_count);
    return hipGetLastError();
}

}  // namespace ilre
