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
//   allocate_ranked   one workgroup walks the combinations in order over their rank-ordered token lists: a
//                token already allocated (LDS hash set) is skipped, the first B_j others are taken
//   emit_sorted  the allocated set in ascending order behind the sink part (each token counts the
//                tokens below it)
//
// The window-max form does not pool while it scans.  With B' = min(B, L), only the B' best raw scores by
// (score descending, token ascending), the "seeds", can decide anything: the K_j-th largest pooled value
// of any kernel size is at least the B'-th largest raw score (pooling only raises values and K_j <= B'),
// so every candidate token has a seed inside its window, and a seed that B' others outrank owns no token
// of any candidate prefix.  Hence:
//
//   sel_init, pool_hist<1>, pool_hist<2>, collect, refine    as above, for ONE combination with window 1:
//                the B' best raw scores (plus, harmlessly, up to kSelSmall more that share the 22-bit
//                prefix of the last one)
//   seed_rank    per seed: its rank among the seeds (counting: a wavefront's lanes share out the staged keys
//                and compare them with its four seeds) and the nearest seed that outranks it on either side
//                (a scan of the raw scores around it, 16 lanes a seed: whatever outranks a seed is a seed)
//   seed_lists   one workgroup per kernel size: seed u owns the tokens whose window holds u and no seed
//                that outranks u, an interval [max(u-r, a+r+1), min(u+r, b-r-1)]; their pooled value is
//                u's score.  Seeds in rank order, each interval ascending, is the kernel size's ranked
//                token list; its first K_j tokens are written out
//   allocate_ranked   the walk over those lists (shared with the printed form)
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

constexpr int kThreads = 1024;                    // refine, seed_lists: one large workgroup
constexpr int kPoolThreads = 256;                 // pooling passes: four wavefronts, one fine chunk each
constexpr int kPoolWaves = kPoolThreads / 64;
constexpr int kPerThread = kSelFine / 64;         // 4 tokens per lane
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kHashSlots = 16384;                 // >= 2 * ILRE_MAX_BUDGET
constexpr int kKeysPerThread = kCandCap / kThreads;

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
// Copy n items from global memory into LDS with the whole block, eight loads in flight per thread.
template <typename T, int THREADS>
__device__ __forceinline__ void stage_to_lds(T *dst, const T *src, uint32_t n)
{
    constexpr int kBatch = 8;
    for (uint32_t i0 = threadIdx.x; i0 < n; i0 += THREADS * kBatch) {
        T x[kBatch];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const uint32_t i = i0 + b * THREADS;
            x[b] = src[i < n ? i : n - 1];
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const uint32_t i = i0 + b * THREADS;
            if (i < n) dst[i] = x[b];
        }
    }
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

// Window 1 in the window-max form (the seed pass): the pooled value is the element.  kRawBatch fine chunks
// (entries e0 .. e0 + kRawBatch - 1 of the visit list) are fetched at once; fcs[u] < 0 marks a missing entry.
constexpr int kRawBatch = 4;
__device__ __forceinline__ bool raw_window(const Pooling &pl) { return pl.op == kSelWindowMax && pl.before + pl.after == 0; }
__device__ __forceinline__ void raw_fetch(const Pooling &pl, const Entries &ent, uint32_t e0, uint32_t nent, int64_t (&fcs)[kRawBatch],
                                          float (&vals)[kRawBatch][kPerThread])
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < kRawBatch; ++u) fcs[u] = e0 + u < nent ? (int64_t)entry_chunk(ent, e0 + u) : -1;
#pragma unroll
    for (int u = 0; u < kRawBatch; ++u)
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int64_t e = (fcs[u] < 0 ? 0 : fcs[u]) * kSelFine + lane + k * 64;
            vals[u][k] = pl.src[e < pl.len ? e : pl.len - 1];  // lanes past the end are ignored by the callers
        }
}

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

// The same for N items a lane (item g of every lane forms group g) and two lists at once: one slot reservation
// per list for the whole lot, both in flight together.  A reservation is a returning atomic on one address, a
// round trip to the memory side; one per group would chain N of them.
template <int N>
__device__ __forceinline__ void wave_append2(const bool (&pa)[N], const bool (&pb)[N], const uint64_t (&item)[N], uint64_t *la,
                                             uint32_t *ca, uint64_t *lb, uint32_t *cb)
{
    const int lane = threadIdx.x & 63;
    uint32_t na = 0, nb = 0;
#pragma unroll
    for (int g = 0; g < N; ++g) {
        na += (uint32_t)__popcll(__ballot(pa[g]));
        nb += (uint32_t)__popcll(__ballot(pb[g]));
    }
    if (na + nb == 0) return;  // uniform
    uint32_t base_a = 0, base_b = 0;
    if (lane == 0) {
        base_a = atomicAdd(ca, na);
        base_b = atomicAdd(cb, nb);
    }
    base_a = (uint32_t)__builtin_amdgcn_readfirstlane((int)base_a);
    base_b = (uint32_t)__builtin_amdgcn_readfirstlane((int)base_b);
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int g = 0; g < N; ++g) {
        const uint64_t ma = __ballot(pa[g]), mb = __ballot(pb[g]);
        if (pa[g]) la[base_a + (uint32_t)__popcll(ma & below)] = item[g];
        if (pb[g]) lb[base_b + (uint32_t)__popcll(mb & below)] = item[g];
        base_a += (uint32_t)__popcll(ma);
        base_b += (uint32_t)__popcll(mb);
    }
}

// Histogram accounting of a wavefront's kPerThread values per lane (element `first + lane + 64k`, valid while
// below `len`) into the workgroup's LDS histogram.  LEVEL 1: key bits 31..21.  LEVEL 2: bits 20..10 of the
// keys whose bits 31..21 equal bin1.
template <int LEVEL>
__device__ __forceinline__ void hist_account(uint32_t *lh, const float (&pooled)[kPerThread], int64_t first, int64_t len,
                                             uint32_t bin1)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int64_t el = first + lane + k * 64;
        const uint32_t key = ordered_bits(pooled[k]);
        if (LEVEL == 1) {
            // Real score distributions put most of a wavefront's 64 keys into one or two bins, and
            // same-address LDS atomics serialise: the two most common bins are counted with ballots
            // and added once, whatever is left goes one by one.
            const uint32_t bin = key >> 21;
            bool todo = el >= 0 && el < len;
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
        } else if (el >= 0 && el < len && (key >> 21) == bin1) {
            atomicAdd(&lh[(key >> 10) & (kSelBins - 1)], 1u);
        }
    }
}

// The workgroup's LDS histogram goes to the combination's global one; the last workgroup of combination j to
// get here sees it complete and locates the bin.  The bins are only ever touched by device-scope atomics (adds
// here, atomic loads in find_bins), which are performed at the memory side, common to all eight L2s.  Each
// thread waits until its adds have been performed (vmcnt counts them), then one thread counts the workgroup in
// with another device-scope atomic: whoever reads the final count reads, with atomic loads issued after it, bins
// that hold every add.  A device-scope release fence in their place would also write this L2's unrelated dirty
// lines back, tens of microseconds per workgroup; the acquire side, one workgroup per combination, is cheap and
// is there.  `counter` is the completion counter of this level and combination, `workgroups` how many count in.
template <int LEVEL>
__device__ __forceinline__ void hist_finish(uint32_t *lh, uint32_t *hist, SelCtrl *ctrl, int j, uint32_t *counter,
                                            uint32_t workgroups, uint32_t *is_last)
{
    __syncthreads();
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hist[(size_t)j * kSelBins + i], c);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        *is_last = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == workgroups - 1;
    __syncthreads();
    if (*is_last) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        find_bins<LEVEL>(hist, ctrl, j);
    }
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
    const int wave = threadIdx.x >> 6;
    uint32_t *hist = hist_all + (size_t)(LEVEL - 1) * n * kSelBins;
    float *b0 = (float *)smem + (size_t)wave * 2 * pool_lds_floats(pl.before, pl.after);
    float *b1 = b0 + pool_lds_floats(pl.before, pl.after);
    const uint32_t bin1 = LEVEL == 2 ? ctrl[j].bin1 : 0;
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) lh[i] = 0;
    __syncthreads();
    const uint32_t nent = entry_count(ent, (uint32_t)pl.len);
    if (raw_window(pl)) {
        // window 1: the elements themselves; a wavefront fetches kRawBatch fine chunks before it accounts for
        // any, so that their loads are in flight together
        for (uint32_t e0 = (blockIdx.x * kPoolWaves + wave) * kRawBatch; e0 < nent; e0 += gridDim.x * kPoolWaves * kRawBatch) {
            float vals_[kRawBatch][kPerThread];
            int64_t fcs[kRawBatch];
            raw_fetch(pl, ent, e0, nent, fcs, vals_);
#pragma unroll
            for (int u = 0; u < kRawBatch; ++u)
                if (fcs[u] >= 0) hist_account<LEVEL>(lh, vals_[u], fcs[u] * kSelFine, pl.len, bin1);  // uniform
        }
    } else {
        for (uint32_t e = blockIdx.x * kPoolWaves + wave; e < nent; e += gridDim.x * kPoolWaves) {
            const int64_t fc = entry_chunk(ent, e);
            float pooled[kPerThread];
            pooled_wave(pl, fc, b0, b1, pooled);
            hist_account<LEVEL>(lh, pooled, fc * kSelFine, pl.len, bin1);
        }
    }
    hist_finish<LEVEL>(lh, hist, ctrl, j, &done[(LEVEL - 1) * n + j], gridDim.x, &is_last);
}

// The whole path's first selection pass, fused with the last scoring step: score[t] = sum (or max) over the
// (kv head, query block) units of their partial column results, written out for every token, and the level-1
// histogram of the body's scores (tokens sink .. L-1) for the single seed combination, in one pass over the
// partial vectors.  The sum runs in unit order, as in the stand-alone reduction.
template <int RMAX>
__global__ __launch_bounds__(kPoolThreads) void reduce_hist1(const float *partial, int nunits, int64_t L, int sink, float *score,
                                                             SelCtrl *ctrl, uint32_t *hist, uint32_t *done)
{
    __shared__ uint32_t lh[kSelBins];
    __shared__ uint32_t is_last;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) lh[i] = 0;
    __syncthreads();
    const uint32_t nfine = (uint32_t)((L + kSelFine - 1) / kSelFine);
    // A wavefront takes kChunks fine chunks a round and the units eight at a time: 64 independent loads per lane
    // are in flight before the first sum (the partial vectors are 64 MiB at 1M tokens; this pass is their one
    // reader and must run at memory speed).
    constexpr int kChunks = 2, kUnits = 8;
    for (uint32_t fc0 = (blockIdx.x * kPoolWaves + wave) * kChunks; fc0 < nfine; fc0 += gridDim.x * kPoolWaves * kChunks) {
        float v[kChunks][kPerThread];
        int64_t tok[kChunks][kPerThread];
#pragma unroll
        for (int c = 0; c < kChunks; ++c)
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {
                const int64_t t = (int64_t)(fc0 + c) * kSelFine + lane + k * 64;
                tok[c][k] = t < L ? t : L - 1;
            }
        for (int u0 = 0; u0 < nunits; u0 += kUnits) {
            float x[kUnits][kChunks][kPerThread];
#pragma unroll
            for (int uu = 0; uu < kUnits; ++uu) {
                const int64_t u = u0 + uu < nunits ? u0 + uu : nunits - 1;
#pragma unroll
                for (int c = 0; c < kChunks; ++c)
#pragma unroll
                    for (int k = 0; k < kPerThread; ++k) x[uu][c][k] = partial[u * L + tok[c][k]];
            }
#pragma unroll
            for (int uu = 0; uu < kUnits; ++uu) {
                if (u0 + uu >= nunits) break;  // uniform
#pragma unroll
                for (int c = 0; c < kChunks; ++c)
#pragma unroll
                    for (int k = 0; k < kPerThread; ++k) {
                        if (u0 + uu == 0)
                            v[c][k] = x[uu][c][k];
                        else
                            v[c][k] = RMAX ? fmaxf(v[c][k], x[uu][c][k]) : v[c][k] + x[uu][c][k];
                    }
            }
        }
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            if (fc0 + c >= nfine) break;  // uniform
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {
                const int64_t t = (int64_t)(fc0 + c) * kSelFine + lane + k * 64;
                if (t < L) score[t] = v[c][k];
            }
            // body element of token t is t - sink; the sink tokens (negative elements) are not counted
            hist_account<1>(lh, v[c], (int64_t)(fc0 + c) * kSelFine - sink, L - sink, 0);
        }
    }
    hist_finish<1>(lh, hist, ctrl, 0, &done[0], gridDim.x, &is_last);
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
    // keys above the prefix are candidates, keys that share it go to the boundary list
    auto classify = [&](float pooled, int64_t fc, int k, bool &above, bool &same, uint64_t &key) {
        const int64_t el = fc * kSelFine + lane + k * 64;
        const bool valid = fc >= 0 && el < pl.len;
        const uint32_t p22 = valid ? ordered_bits(pooled) >> 10 : 0;
        key = make_key(pooled, (uint32_t)el);
        above = valid && p22 > prefix;
        same = valid && p22 == prefix;
    };
    if (raw_window(pl)) {
        for (uint32_t e0 = (blockIdx.x * kPoolWaves + wave) * kRawBatch; e0 < nent; e0 += gridDim.x * kPoolWaves * kRawBatch) {
            float vals_[kRawBatch][kPerThread];
            int64_t fcs[kRawBatch];
            raw_fetch(pl, ent, e0, nent, fcs, vals_);
            bool above[kRawBatch * kPerThread], same[kRawBatch * kPerThread];
            uint64_t key[kRawBatch * kPerThread];
#pragma unroll
            for (int u = 0; u < kRawBatch; ++u)
#pragma unroll
                for (int k = 0; k < kPerThread; ++k)
                    classify(vals_[u][k], fcs[u], k, above[u * kPerThread + k], same[u * kPerThread + k], key[u * kPerThread + k]);
            wave_append2<kRawBatch * kPerThread>(above, same, key, cand_j, &ctrl[j].cand_n, tie_j, &ctrl[j].tie_n);
        }
    } else {
        for (uint32_t e = blockIdx.x * kPoolWaves + wave; e < nent; e += gridDim.x * kPoolWaves) {
            const int64_t fc = entry_chunk(ent, e);
            float pooled[kPerThread];
            pooled_wave(pl, fc, b0, b1, pooled);
            bool above[kPerThread], same[kPerThread];
            uint64_t key[kPerThread];
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) classify(pooled[k], fc, k, above[k], same[k], key[k]);
            wave_append2<kPerThread>(above, same, key, cand_j, &ctrl[j].cand_n, tie_j, &ctrl[j].tie_n);
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
    const bool aligned = ((size_t)scores & 15) == 0;  // a sink part may shift the body off the 16-byte grid
    for (uint32_t c0 = (blockIdx.x * kPoolWaves + wave) * 4; c0 < nfine; c0 += stride) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t tok = (int64_t)(c0 + u) * kSelFine + lane * 4;
            if (aligned && tok + 3 < L) {
                v[u] = *(const float4 *)(scores + tok);
            } else {
                v[u].x = tok + 0 < L ? scores[tok + 0] : -INFINITY;
                v[u].y = tok + 1 < L ? scores[tok + 1] : -INFINITY;
                v[u].z = tok + 2 < L ? scores[tok + 2] : -INFINITY;
                v[u].w = tok + 3 < L ? scores[tok + 3] : -INFINITY;
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
// One slot reservation per workgroup (same-address atomics serialise at about 13 ns each, and a few thousand
// scattered hits would otherwise mean a few thousand of them): a thread looks at kMarkPerThread consecutive chunks.
constexpr int kMarkPerThread = 16;
__global__ __launch_bounds__(kPoolThreads) void mark_active(const float *cm, uint32_t nfine, int reach, SelCtrl *pctrl,
                                                            uint32_t *list)
{
    __shared__ uint32_t wsum[kPoolWaves];
    __shared__ uint32_t base_slot;
    const uint32_t c0 = (blockIdx.x * kPoolThreads + threadIdx.x) * kMarkPerThread;
    const uint32_t bin1 = pctrl->bin1, bin2 = pctrl->bin2;
    const uint32_t prefix = (bin1 >= (uint32_t)kSelBins || bin2 >= (uint32_t)kSelBins) ? 0u : (bin1 << 11) | bin2;
    uint32_t hits = 0;  // bit i: chunk c0 + i is active
#pragma unroll
    for (int i = 0; i < kMarkPerThread; ++i) {
        const uint32_t c = c0 + i;
        if (c < nfine) {
            float m = cm[c];
            for (int d = 1; d <= reach; ++d) {
                if (c >= (uint32_t)d) m = fmaxf(m, cm[c - d]);
                if (c + d < nfine) m = fmaxf(m, cm[c + d]);
            }
            if ((ordered_bits(m) >> 10) >= prefix) hits |= 1u << i;
        }
    }
    uint32_t total;
    const uint32_t mine = (uint32_t)__popc(hits);
    uint32_t at = block_scan_inclusive<kPoolThreads>(mine, wsum, total) - mine;
    if (total == 0) return;  // uniform
    if (threadIdx.x == 0) base_slot = atomicAdd(&pctrl->cand_n, total);
    __syncthreads();
    at += base_slot;
#pragma unroll
    for (int i = 0; i < kMarkPerThread; ++i)
        if ((hits >> i) & 1u) list[at++] = c0 + i;
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

// Last step of the allocation: the sink indices, then the nsel allocated tokens in ascending order, then -1
// up to sink + n_out.  The walk leaves the tokens in the order it took them; here every token counts the
// tokens below it, which is its place in the output whatever order they arrived in and however they
// cluster.  The list is staged in LDS; a wavefront owns kEmitPerWave tokens and its lanes read disjoint
// quarters of the list (every LDS word is fetched once per wavefront) and compare them with all of the
// wavefront's tokens.
constexpr int kEmitThreads = 512;
constexpr int kEmitPerWave = 4;
constexpr int kEmitPerBlock = kEmitThreads / 64 * kEmitPerWave;  // 32 tokens a workgroup
__global__ __launch_bounds__(kEmitThreads) void emit_sorted(const uint32_t *picked, const uint32_t *picked_n, int n_out, int sink,
                                                            int32_t *out_idx, int32_t *out_count)
{
    __shared__ __align__(16) uint32_t all[ILRE_MAX_BUDGET];
    static_assert(ILRE_MAX_BUDGET % 256 == 0, "the staged list is padded to whole rounds of 64 lanes x 4 tokens");
    const uint32_t nsel = *picked_n;
    const uint32_t gtid = blockIdx.x * kEmitThreads + threadIdx.x, gsize = gridDim.x * kEmitThreads;
    for (uint32_t i = gtid; i < (uint32_t)sink; i += gsize) out_idx[i] = (int32_t)i;
    for (uint32_t i = nsel + gtid; i < (uint32_t)n_out; i += gsize) out_idx[sink + i] = -1;
    if (gtid == 0 && out_count) *out_count = sink + (int32_t)nsel;
    if (blockIdx.x * kEmitPerBlock >= nsel) return;  // uniform
    stage_to_lds<uint32_t, kEmitThreads>(all, picked, nsel);
    const uint32_t padded = (nsel + 255u) & ~255u;  // the padding holds tokens no token is below
    if (threadIdx.x < 256 && nsel + threadIdx.x < padded) all[nsel + threadIdx.x] = 0xFFFFFFFFu;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t i0 = blockIdx.x * kEmitPerBlock + wave * kEmitPerWave;
    if (i0 >= nsel) return;  // whole wavefronts leave together, no barrier follows
    uint32_t t[kEmitPerWave], below[kEmitPerWave];
#pragma unroll
    for (int q = 0; q < kEmitPerWave; ++q) {
        t[q] = (uint32_t)__builtin_amdgcn_readfirstlane((int)all[i0 + q < nsel ? i0 + q : nsel - 1]);
        below[q] = 0;
    }
#pragma unroll 2
    for (uint32_t v = 4u * lane; v < padded; v += 256) {
        const uint4 x = *(const uint4 *)&all[v];
#pragma unroll
        for (int q = 0; q < kEmitPerWave; ++q)
            below[q] += (x.x < t[q] ? 1u : 0u) + (x.y < t[q] ? 1u : 0u) + (x.z < t[q] ? 1u : 0u) + (x.w < t[q] ? 1u : 0u);
    }
#pragma unroll
    for (int q = 0; q < kEmitPerWave; ++q) {
        const uint32_t place = wave_total(wave_scan_add(below[q]));
        if (lane == q && i0 + q < nsel) out_idx[sink + place] = (int32_t)(t[q] + (uint32_t)sink);
    }
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
                                                                uint32_t *picked, uint32_t *picked_n)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = (uint32_t *)smem;  // kHashSlots
    uint32_t *sel = table + kHashSlots;  // ILRE_MAX_BUDGET tokens
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
    // the allocated tokens, in the order they were taken, for emit_sorted
    for (uint32_t i = threadIdx.x; i < nsel; i += kRankThreads) picked[i] = sel[i];
    if (threadIdx.x == 0) *picked_n = nsel;
}


// ---------------------------------------------------------------- window-max form: seeds

// Per seed u (one of the ns best raw scores, keys distinct): rank[u] = number of seeds with a larger key,
// and the nearest token on either side, within `reach` tokens, whose key is larger (-1 / -1 if none; such a
// token is itself a seed, the seeds being the best keys).  A wavefront owns four seeds.  For the count its
// lanes read disjoint parts of the staged key list (every LDS word is fetched once per wavefront) and
// compare them with all four keys; for the scan 16 lanes share a seed and split its neighbourhood.
constexpr int kSeedRankThreads = 512;  // 32 seeds a workgroup
__global__ __launch_bounds__(kSeedRankThreads) void seed_rank(const float *scores, int64_t L, const SelCtrl *sc, const uint64_t *seeds,
                                                              int reach, uint32_t *rank, int32_t *dom_left, int32_t *dom_right)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t *all = (uint64_t *)smem;  // every seed's key, staged once per workgroup (kCandCap at most)
    const uint32_t ns = sc->total_n;
    if (blockIdx.x * (kSeedRankThreads / 16) >= ns) return;  // uniform
    // (the seeds were written by earlier kernels: plain loads, all in flight together)
    stage_to_lds<uint64_t, kSeedRankThreads>(all, seeds, ns);
    const uint32_t padded = (ns + 127u) & ~127u;  // whole rounds of 64 lanes x 2 keys; the padding outranks nothing
    if (threadIdx.x < 128 && ns + threadIdx.x < padded) all[ns + threadIdx.x] = 0ull;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const uint32_t u0 = blockIdx.x * (kSeedRankThreads / 16) + (threadIdx.x >> 6) * 4;  // the wavefront's first seed
    if (u0 >= ns) return;  // whole wavefronts leave together, no barrier follows
    uint64_t wkey[4];
    uint32_t wcnt[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint64_t k = all[u0 + q < ns ? u0 + q : ns - 1];
        wkey[q] = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(k >> 32)) << 32) |
                  (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)k);
        wcnt[q] = 0;
    }
#pragma unroll 2
    for (uint32_t v = 2u * lane; v < padded; v += 128) {
        const uint4 x = *(const uint4 *)&all[v];
        const uint64_t k0 = ((uint64_t)x.y << 32) | x.x, k1 = ((uint64_t)x.w << 32) | x.z;
#pragma unroll
        for (int q = 0; q < 4; ++q) wcnt[q] += (k0 > wkey[q] ? 1u : 0u) + (k1 > wkey[q] ? 1u : 0u);
    }
    uint32_t wtot[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) wtot[q] = wave_total(wave_scan_add(wcnt[q]));
    const int grp = lane >> 4;
    const uint32_t u = u0 + grp;
    const int sub = lane & 15;
    if (u >= ns) return;  // whole 16-lane groups leave together
    const uint64_t key = grp == 0 ? wkey[0] : (grp == 1 ? wkey[1] : (grp == 2 ? wkey[2] : wkey[3]));
    const uint32_t cnt = grp == 0 ? wtot[0] : (grp == 1 ? wtot[1] : (grp == 2 ? wtot[2] : wtot[3]));
    const int64_t pos = (int64_t)key_token(key);
    // nearest outranking token: distance d = 1 .. reach, 16 distances a round, both sides at once
    int32_t left = -1, right = -1;
    for (int d0 = 1; d0 <= reach; d0 += 16) {
        const int d = d0 + sub;
        const int64_t pl = pos - d, pr = pos + d;
        const bool hit_l = d <= reach && pl >= 0 && make_key(scores[pl < 0 ? 0 : pl], (uint32_t)(pl < 0 ? 0 : pl)) > key;
        const bool hit_r = d <= reach && pr < L && make_key(scores[pr < L ? pr : L - 1], (uint32_t)(pr < L ? pr : L - 1)) > key;
        // lowest lane of this 16-lane group with a hit = smallest distance
        const uint64_t bl = __ballot(left < 0 && hit_l), br = __ballot(right < 0 && hit_r);
        const int shift = (threadIdx.x & 63) & ~15;
        const uint32_t ml = (uint32_t)(bl >> shift) & 0xFFFFu, mr = (uint32_t)(br >> shift) & 0xFFFFu;
        if (left < 0 && ml) left = (int32_t)(pos - (d0 + __ffs((int)ml) - 1));
        if (right < 0 && mr) right = (int32_t)(pos + (d0 + __ffs((int)mr) - 1));
        if (left >= 0 && right >= 0) break;  // uniform within the group; ballots are wave-wide but only read per group
    }
    if (sub == 15) {
        rank[u] = cnt;
        dom_left[u] = left;
        dom_right[u] = right;
    }
}

// One workgroup per kernel size j: the first K_j tokens of its ranked token list (uint32, in the storage of
// cand list 1 + j) and its control block for the walk.  LDS: lo[kCandCap] and the running token counts
// pre[kCandCap], both indexed by seed rank.
struct SeedParams {
    int n;
    uint32_t radius[ILRE_MAX_POOL_KERNELS], share[ILRE_MAX_POOL_KERNELS], want[ILRE_MAX_POOL_KERNELS];
};
__global__ __launch_bounds__(kThreads) void seed_lists(const SeedParams prm, int64_t L, const SelCtrl *sc, const uint64_t *seeds,
                                                       const uint32_t *rank, const int32_t *dom_left, const int32_t *dom_right,
                                                       SelCtrl *kctrl, uint64_t *cand)
{
    extern __shared__ __align__(16) unsigned char smem[];
    int32_t *lo = (int32_t *)smem;
    uint32_t *pre = (uint32_t *)(lo + kCandCap);
    __shared__ uint32_t wsum[kThreads / 64];
    const int j = blockIdx.x;
    const uint32_t ns = sc->total_n;
    const int64_t r = prm.radius[j];
    for (uint32_t u = threadIdx.x; u < ns; u += kThreads) {
        const int64_t pos = (int64_t)key_token(seeds[u]);
        const int64_t a = dom_left[u], b = dom_right[u];
        int64_t first = pos - r, last = pos + r;
        if (first < 0) first = 0;
        if (last > L - 1) last = L - 1;
        if (a >= 0 && a + r + 1 > first) first = a + r + 1;
        if (b >= 0 && b - r - 1 < last) last = b - r - 1;
        const uint32_t rk = rank[u];
        lo[rk] = (int32_t)first;
        pre[rk] = last >= first ? (uint32_t)(last - first + 1) : 0u;
    }
    __syncthreads();
    // inclusive running sum of the interval lengths in rank order: thread t owns ranks t*kKeysPerThread ..
    uint32_t own[kKeysPerThread], sum = 0;
#pragma unroll
    for (int k = 0; k < kKeysPerThread; ++k) {
        const uint32_t i = threadIdx.x * kKeysPerThread + k;
        own[k] = i < ns ? pre[i] : 0u;
        sum += own[k];
    }
    uint32_t total;
    uint32_t run = block_scan_inclusive<kThreads>(sum, wsum, total) - sum;
#pragma unroll
    for (int k = 0; k < kKeysPerThread; ++k) {
        const uint32_t i = threadIdx.x * kKeysPerThread + k;
        run += own[k];
        if (i < ns) pre[i] = run;
    }
    __syncthreads();
    const uint32_t want = prm.want[j] < total ? prm.want[j] : total;
    uint32_t *tokens = (uint32_t *)(cand + (size_t)(1 + j) * kCandCap);
    for (uint32_t i = threadIdx.x; i < want; i += kThreads) {
        // the seed whose interval holds ranked token i: the first rank with pre[rank] > i
        uint32_t lo_r = 0, hi_r = ns - 1;
        while (lo_r < hi_r) {
            const uint32_t mid = (lo_r + hi_r) >> 1;
            if (pre[mid] > i) hi_r = mid; else lo_r = mid + 1;
        }
        const uint32_t before = lo_r ? pre[lo_r - 1] : 0u;
        tokens[i] = (uint32_t)lo[lo_r] + (i - before);
    }
    if (threadIdx.x == 0) {
        SelCtrl c{};
        c.share = prm.share[j];
        c.total_n = want;
        c.cell = 1;
        kctrl[j] = c;
    }
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
    const bool window = job.mode == kSelWindowMax;
    // histogram passes run per combination in the printed form, for the single seed combination in the
    // window-max form; one more set belongs to the pruning pre-pass
    const int nh = window ? 1 : n;
    const size_t nfine = (size_t)((job.L + kSelFine - 1) / kSelFine);
    size_t off = 0;
    lay.hist = off;
    off = up(off + 2 * (size_t)(nh + 1) * kSelBins * sizeof(uint32_t));
    lay.ctrl = off;
    off = up(off + (size_t)(nh + 1 + (window ? n : 0)) * sizeof(SelCtrl));
    lay.done = off;
    off = up(off + 2 * (size_t)(nh + 1) * sizeof(uint32_t));
    lay.cmax = off;
    off = up(off + nfine * sizeof(float));
    lay.active = off;
    off = up(off + nfine * sizeof(uint32_t));
    lay.cells = off;
    size_t ncell = 0, ntie = 0;
    if (!window) {
        for (int i = 0; i < job.n_max; ++i) ncell += (size_t)(job.L / job.max_kernels[i]);
        ntie = 2 * ncell * (size_t)job.n_avg;
    } else {
        ntie = 2 * (size_t)job.L;
    }
    off = up(off + ncell * sizeof(float));
    lay.picked = off;
    off = up(off + ((size_t)ILRE_MAX_BUDGET + 64) * sizeof(uint32_t));
    lay.seed = off;
    off = up(off + (window ? 3 * (size_t)kCandCap * sizeof(uint32_t) : 0));
    lay.cand = off;
    off = up(off + (size_t)(window ? n + 1 : n) * kCandCap * sizeof(uint64_t));
    lay.tie = off;
    off = up(off + ntie * sizeof(uint64_t));
    lay.total = off;
    return lay;
}

namespace {

// Dynamic LDS ceilings of the selection kernels: the same constants on every call, set once per process
// and device-independent.
hipError_t set_select_attributes()
{
    static hipError_t status = [] {
        constexpr int kAllocLds = kHashSlots * (int)sizeof(uint32_t) + ILRE_MAX_BUDGET * (int)sizeof(uint32_t);
        constexpr int kPoolLdsMax = kPoolWaves * 2 * (kSelFine + 2 * (ILRE_MAX_AVG_KERNEL > ILRE_MAX_POOL_KERNEL ? ILRE_MAX_AVG_KERNEL : ILRE_MAX_POOL_KERNEL)) * (int)sizeof(float);
        constexpr int kSortLdsMax = 16384 * (int)sizeof(uint64_t);  // >= ILRE_MAX_BUDGET + 1 keys, padded to a power of two
        constexpr int kSeedLds = 2 * kCandCap * (int)sizeof(uint32_t);
        constexpr int kSeedRankLds = kCandCap * (int)sizeof(uint64_t);
        hipError_t e;
        if ((e = hipFuncSetAttribute((const void *)allocate_ranked, hipFuncAttributeMaxDynamicSharedMemorySize, kAllocLds)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)pool_hist<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)pool_hist<2>, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)collect, hipFuncAttributeMaxDynamicSharedMemorySize, kPoolLdsMax)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)refine, hipFuncAttributeMaxDynamicSharedMemorySize, kSortLdsMax)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)seed_lists, hipFuncAttributeMaxDynamicSharedMemorySize, kSeedLds)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)seed_rank, hipFuncAttributeMaxDynamicSharedMemorySize, kSeedRankLds)) != hipSuccess) return e;
        return hipSuccess;
    }();
    return status;
}

uint32_t pool_blocks(uint32_t entries, uint32_t cap)
{
    const uint32_t want = (entries + kPoolWaves - 1) / kPoolWaves;
    return want < cap ? (want ? want : 1u) : cap;
}
uint32_t clamp_u32(uint32_t x, uint32_t lo, uint32_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Workgroups per combination in the pooling passes; beyond the cap the wavefronts loop over the entries.
// A histogram workgroup carries fixed work (clearing and flushing 2048 bins, one atomic per hot bin on a
// handful of addresses, about 13 ns each and serialised, the completion counter), so those passes aim at
// about one resident round of workgroups over all combinations.
constexpr uint32_t kHistGrid = 2560, kCollectGrid = 8192;

// Window-max form: the seeds (best raw scores), their ranks and neighbours, one ranked token list per
// kernel size, the walk.
hipError_t launch_select_window(const float *scores, const SelectJob &job, int32_t *out_idx, int32_t *out_count,
                                unsigned char *ws, const SelectLayout &lay, hipStream_t s, const FusedScores *fused)
{
    const int64_t L = job.L;
    const int n = job.combos();
    const int n_out = (int)(job.budget < L ? job.budget : L);
    uint32_t *hist = (uint32_t *)(ws + lay.hist);
    SelCtrl *ctrl = (SelCtrl *)(ws + lay.ctrl);  // [0] the seed combination, [1] the pruning pre-pass, [2 ..] the kernel sizes
    uint32_t *done = (uint32_t *)(ws + lay.done);
    uint64_t *cand = (uint64_t *)(ws + lay.cand);  // list 0: the seeds' keys; list 1 + j: kernel size j's ranked tokens
    uint64_t *tie = (uint64_t *)(ws + lay.tie);
    uint32_t *rank = (uint32_t *)(ws + lay.seed);
    int32_t *dom_left = (int32_t *)(rank + kCandCap), *dom_right = dom_left + kCandCap;
    const size_t alloc_lds = (size_t)kHashSlots * sizeof(uint32_t) + (size_t)ILRE_MAX_BUDGET * sizeof(uint32_t);
    uint32_t *picked = (uint32_t *)(ws + lay.picked), *picked_n = picked + ILRE_MAX_BUDGET;
    const dim3 emit_grid((unsigned)((n_out + kEmitPerBlock - 1) / kEmitPerBlock) + 1u);

    // the seed combination: window 1 on the scores, the n_out best wanted
    SelParams prm{};
    prm.n = 1;
    prm.op = (uint32_t)kSelWindowMax;
    prm.exact = 0;
    prm.share[0] = (uint32_t)n_out;
    prm.want[0] = (uint32_t)n_out;
    prm.len[0] = (uint32_t)L;
    prm.cell[0] = 1;
    // B_c: floor(B / n), the first B mod n kernel sizes one more.  K_j: what the earlier shares could have
    // taken plus the own share.
    SeedParams sp{};
    sp.n = n;
    const int base = job.budget / n, rem = job.budget % n;
    int64_t before = 0;
    int r_max = 0;
    for (int j = 0; j < n; ++j) {
        const int share = base + (j < rem ? 1 : 0);
        const int r = (job.max_kernels[j] - 1) / 2;
        const int64_t want = before + share < n_out ? before + share : n_out;
        sp.radius[j] = (uint32_t)r;
        sp.share[j] = (uint32_t)share;
        sp.want[j] = (uint32_t)want;
        before += share;
        if (r > r_max) r_max = r;
    }

    const uint32_t nfine = (uint32_t)((L + kSelFine - 1) / kSelFine);
    const size_t pool_lds = (size_t)kPoolWaves * 2 * (size_t)kSelFine * sizeof(float);
    Entries ent{nullptr, nullptr};
    uint32_t entries = nfine;
    const bool pruned = (int64_t)nfine >= 4 * (int64_t)n_out && nfine >= 16384;
    if (fused && pruned) {  // the pre-pass wants the finished scores
        const hipError_t e = launch_reduce_units(fused->partial, fused->nunits, fused->L, fused->rmax, fused->scores, s);
        if (e != hipSuccess) return e;
        fused = nullptr;
    }
    if (pruned) {
        // Long contexts: only fine chunks whose maximum reaches the n_out-th largest chunk maximum (up to its
        // 22-bit prefix) can hold one of the n_out best scores; visit only those.
        float *cm = (float *)(ws + lay.cmax);
        uint32_t *active = (uint32_t *)(ws + lay.active);
        uint32_t *phist = hist + 2 * (size_t)kSelBins;
        SelCtrl *pctrl = ctrl + 1;
        uint32_t *pdone = done + 2;
        SelParams pp{};
        pp.n = 1;
        pp.len[0] = nfine;
        pp.cell[0] = 1;
        pp.want[0] = (uint32_t)n_out;
        const uint32_t nfine2 = (nfine + kSelFine - 1) / kSelFine;
        const Entries all{nullptr, nullptr};
        hipLaunchKernelGGL(chunk_max, dim3(2048), dim3(kPoolThreads), 0, s, scores, L, nfine, cm);
        hipLaunchKernelGGL(sel_init, dim3(1), dim3(kThreads), 0, s, pp, phist, pctrl, pdone);
        const uint32_t pblocks = pool_blocks((nfine2 + kRawBatch - 1) / kRawBatch, 1024);
        hipLaunchKernelGGL(pool_hist<1>, dim3(pblocks, 1), dim3(kPoolThreads), pool_lds, s, cm, 1, pctrl, phist, pdone, all);
        hipLaunchKernelGGL(pool_hist<2>, dim3(pblocks, 1), dim3(kPoolThreads), pool_lds, s, cm, 1, pctrl, phist, pdone, all);
        hipLaunchKernelGGL(mark_active, dim3((nfine + kPoolThreads * kMarkPerThread - 1) / (kPoolThreads * kMarkPerThread)), dim3(kPoolThreads), 0, s, cm,
                           nfine, 0, pctrl, active);
        ent = Entries{active, &pctrl->cand_n};
        // with a list the entry count is only known on the device: size the grid for the worst case the
        // pruning rule is meant for (a few times the budget) and let the wavefronts loop
        entries = 4u * (uint32_t)n_out + 1024u;
    }
    // window 1: a wavefront takes kRawBatch fine chunks per round
    const uint32_t batches = (entries + kRawBatch - 1) / kRawBatch;
    const uint32_t hblocks = pool_blocks(batches, 256u), cblocks = pool_blocks(batches, 1024u);
    hipLaunchKernelGGL(sel_init, dim3(1), dim3(kThreads), 0, s, prm, hist, ctrl, done);
    if (fused) {
        // the last step of the scoring (sum of the partial score vectors) and the level-1 histogram in one pass
        const uint32_t rblocks = pool_blocks((uint32_t)((fused->L + kSelFine - 1) / kSelFine + 1) / 2, 512u);
        if (fused->rmax)
            hipLaunchKernelGGL(reduce_hist1<1>, dim3(rblocks), dim3(kPoolThreads), 0, s, fused->partial, fused->nunits, fused->L,
                               job.sink, fused->scores, ctrl, hist, done);
        else
            hipLaunchKernelGGL(reduce_hist1<0>, dim3(rblocks), dim3(kPoolThreads), 0, s, fused->partial, fused->nunits, fused->L,
                               job.sink, fused->scores, ctrl, hist, done);
    } else {
        hipLaunchKernelGGL(pool_hist<1>, dim3(hblocks, 1), dim3(kPoolThreads), pool_lds, s, scores, 1, ctrl, hist, done, ent);
    }
    hipLaunchKernelGGL(pool_hist<2>, dim3(hblocks, 1), dim3(kPoolThreads), pool_lds, s, scores, 1, ctrl, hist, done, ent);
    hipLaunchKernelGGL(collect, dim3(cblocks, 1), dim3(kPoolThreads), pool_lds, s, scores, ctrl, cand, tie, ent);
    hipLaunchKernelGGL(refine, dim3(1), dim3(kThreads), 0, s, ctrl, cand, tie, 0u);
    // at most n_out + kSelSmall <= kCandCap seeds
    const uint32_t max_seeds = (uint32_t)n_out + (uint32_t)kSelSmall;
    hipLaunchKernelGGL(seed_rank, dim3((max_seeds + kSeedRankThreads / 16 - 1) / (kSeedRankThreads / 16)), dim3(kSeedRankThreads),
                       (size_t)((max_seeds + 127u) & ~127u) * sizeof(uint64_t), s, scores, L, ctrl, cand, 2 * r_max, rank, dom_left, dom_right);
    hipLaunchKernelGGL(seed_lists, dim3(n), dim3(kThreads), 2 * (size_t)kCandCap * sizeof(uint32_t), s, sp, L, ctrl, cand, rank,
                       dom_left, dom_right, ctrl + 2, cand);
    hipLaunchKernelGGL(allocate_ranked, dim3(1), dim3(kRankThreads), alloc_lds, s, ctrl + 2, cand + kCandCap, n, n_out, picked, picked_n);
    hipLaunchKernelGGL(emit_sorted, emit_grid, dim3(kEmitThreads), 0, s, picked, picked_n, n_out, job.sink, out_idx, out_count);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_select(const float *scores, const SelectJob &job, int32_t *out_idx, int32_t *out_count,
                         void *workspace, const SelectLayout &lay, hipStream_t s, const FusedScores *fused)
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
    const size_t alloc_lds = (size_t)kHashSlots * sizeof(uint32_t) + (size_t)ILRE_MAX_BUDGET * sizeof(uint32_t);
    uint32_t *picked = (uint32_t *)(ws + lay.picked), *picked_n = picked + ILRE_MAX_BUDGET;
    const dim3 emit_grid((unsigned)((n_out + kEmitPerBlock - 1) / kEmitPerBlock) + 1u);

    hipError_t e = set_select_attributes();
    if (e != hipSuccess) return e;
    if (fused && (job.mode != kSelWindowMax || L == 0)) {  // only the window-max form takes the scores unreduced
        if ((e = launch_reduce_units(fused->partial, fused->nunits, fused->L, fused->rmax, fused->scores, s)) != hipSuccess) return e;
        fused = nullptr;
    }
    if (L == 0) {  // nothing but the sink part
        hipLaunchKernelGGL(allocate_ranked, dim3(1), dim3(kRankThreads), alloc_lds, s, ctrl, cand, 0, 0, picked, picked_n);
        hipLaunchKernelGGL(emit_sorted, emit_grid, dim3(kEmitThreads), 0, s, picked, picked_n, 0, job.sink, out_idx, out_count);
        return hipGetLastError();
    }
    if (job.mode == kSelWindowMax) return launch_select_window(scores, job, out_idx, out_count, ws, lay, s, fused);

    // The algorithm as printed.  B_c: floor(B / n), the first B mod n combinations one more; K_m = B / m + 1 cells.
    SelParams prm{};
    CellParams cp{};
    prm.n = n;
    prm.op = (uint32_t)job.mode;
    prm.exact = 1u;
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
        before += share;
        if ((int)(prm.before[j] + prm.after[j]) > halo_max) halo_max = (int)(prm.before[j] + prm.after[j]);
        if (len > len_max) len_max = len;
    }
    cp.n = job.n_max;
    uint32_t sort_n = 2;  // candidates are sorted in LDS, padded to a power of two
    for (int j = 0; j < n; ++j)
        while (sort_n < prm.want[j]) sort_n *= 2;
    const uint32_t nfine = (uint32_t)((len_max + kSelFine - 1) / kSelFine);
    const size_t pool_lds = (size_t)kPoolWaves * 2 * (size_t)(kSelFine + halo_max) * sizeof(float);
    const Entries ent{nullptr, nullptr};
    uint32_t cb = (uint32_t)((len_max + kPoolThreads - 1) / kPoolThreads);
    if (cb > 2048u) cb = 2048u;
    if (cb) hipLaunchKernelGGL(cell_max, dim3(cb, job.n_max), dim3(kPoolThreads), 0, s, scores, cp, cells);
    const uint32_t hcap = clamp_u32(kHistGrid / (uint32_t)n, 32u, 256u), ccap = clamp_u32(kCollectGrid / (uint32_t)n, 64u, 1024u);
    const uint32_t hblocks = pool_blocks(nfine, hcap), cblocks = pool_blocks(nfine, ccap);

    hipLaunchKernelGGL(sel_init, dim3(n), dim3(kThreads), 0, s, prm, hist, ctrl, done);
    hipLaunchKernelGGL(pool_hist<1>, dim3(hblocks, n), dim3(kPoolThreads), pool_lds, s, cells, n, ctrl, hist, done, ent);
    hipLaunchKernelGGL(pool_hist<2>, dim3(hblocks, n), dim3(kPoolThreads), pool_lds, s, cells, n, ctrl, hist, done, ent);
    hipLaunchKernelGGL(collect, dim3(cblocks, n), dim3(kPoolThreads), pool_lds, s, cells, ctrl, cand, tie, ent);
    hipLaunchKernelGGL(refine, dim3(n), dim3(kThreads), (size_t)sort_n * sizeof(uint64_t), s, ctrl, cand, tie, sort_n);
    hipLaunchKernelGGL(allocate_ranked, dim3(1), dim3(kRankThreads), alloc_lds, s, ctrl, cand, n, n_out, picked, picked_n);
    hipLaunchKernelGGL(emit_sorted, emit_grid, dim3(kEmitThreads), 0, s, picked, picked_n, n_out, job.sink, out_idx, out_count);
    return hipGetLastError();
}

}  // namespace ilre
