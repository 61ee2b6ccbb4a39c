// Context allocation (paper Section 3.2, Algorithm 1, stride-1 max-pool form) for gfx950.
//
// Algorithm 1 pools the scores per kernel size, takes a ranked candidate list per kernel and walks
// it, skipping tokens an earlier kernel already allocated, until the kernel's share is filled.  The
// share of kernel j can be met from its top K_j = B_j + (shares of the kernels before it) ranked
// candidates, whatever the earlier kernels took, so candidate lists are independent of each other:
//
//   pool_hist    all kernels at once: pooled score per token (sliding max by doubling, in LDS) and a
//                4096-bin histogram of the top 12 bits of its order-preserving key
//   find_bin     per kernel: the histogram bin in which the K_j-th largest key lies
//   collect      all kernels at once: keys above that bin go to the candidate list, keys inside it to
//                a boundary list
//   refine_sort  per kernel, one workgroup: radix-select (8 bits a pass, survivors compacted) the
//                boundary list down to what is still needed, then bitonic-sort the candidates in LDS
//   walk         one workgroup: kernels in order, first B_j candidates not yet allocated (LDS hash
//                set), then the allocated set sorted ascending
//
// Ranking is (pooled score descending, token index ascending): the 64-bit key is the ordered score
// bits above the complemented index, so all keys are distinct and every step is order-independent;
// the integer atomics only reserve list slots and build histograms, and the result is deterministic.
#include "ilre_internal.h"

namespace ilre {
namespace {

constexpr int kThreads = 1024;
constexpr int kPerThread = kSelChunk / kThreads;  // 4
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kHashSlots = 16384;                 // >= 2 * ILRE_MAX_BUDGET

struct SelParams {
    int n;
    int64_t L;
    uint32_t radius[ILRE_MAX_POOL_KERNELS];
    uint32_t share[ILRE_MAX_POOL_KERNELS];
    uint32_t want[ILRE_MAX_POOL_KERNELS];
};

// Order-preserving map of a finite float onto uint32 (larger float -> larger key).
__device__ __forceinline__ uint32_t ordered_bits(float x)
{
    const uint32_t b = __float_as_uint(x);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ uint64_t make_key(float pooled, uint32_t token)
{
    return ((uint64_t)ordered_bits(pooled) << 32) | (uint64_t)(0xFFFFFFFFu - token);
}

__device__ __forceinline__ uint32_t key_token(uint64_t key) { return 0xFFFFFFFFu - (uint32_t)key; }

// Inclusive prefix sum over the 1024 threads of the block; wsum is 16 words of LDS scratch.
// Every thread also receives the block total.  Contains two barriers.
__device__ __forceinline__ uint32_t block_scan_inclusive(uint32_t x, uint32_t *wsum, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();  // protect wsum against a previous use
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const uint32_t s = wsum[w];
        if (w < wave) before += s;
        all += s;
    }
    total = all;
    return x + before;
}

// Pooled scores of this thread's kPerThread tokens of chunk `chunk` for window radius r:
// pooled[t] = max(score[u] : |u - t| <= r, 0 <= u < L)   (MaxPooling step of Algorithm 1, stride 1,
// window clipped to the context).  b0/b1 are LDS arrays of kSelChunk + 2r floats.  Sliding maximum
// by doubling: m_p[i] = max(score[i .. i+p-1]) for p = 1, 2, 4, ... <= w, then two overlapping
// windows of length p cover the window of length w = 2r + 1.
__device__ __forceinline__ void pooled_chunk(const float *scores, int64_t L, int64_t chunk, int r, float *b0, float *b1,
                                             float (&out)[kPerThread])
{
    const int len = kSelChunk + 2 * r;
    const int64_t first = chunk * kSelChunk - r;
    for (int i = threadIdx.x; i < len; i += kThreads) {
        const int64_t tok = first + i;
        b0[i] = (tok >= 0 && tok < L) ? scores[tok] : -INFINITY;
    }
    __syncthreads();
    const int w = 2 * r + 1;
    int p = 1;
    float *src = b0, *dst = b1;
    while (2 * p <= w) {
        for (int i = threadIdx.x; i < len; i += kThreads) dst[i] = (i + p < len) ? fmaxf(src[i], src[i + p]) : src[i];
        __syncthreads();
        float *t = src;
        src = dst;
        dst = t;
        p *= 2;
    }
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int tl = threadIdx.x + k * kThreads;
        out[k] = fmaxf(src[tl], src[tl + w - p]);
    }
}

__global__ __launch_bounds__(kThreads) void sel_init(const SelParams prm, uint32_t *hist, SelCtrl *ctrl)
{
    const int j = blockIdx.x;
    for (int i = threadIdx.x; i < kSelBins; i += kThreads) hist[(size_t)j * kSelBins + i] = 0;
    if (threadIdx.x == 0) {
        SelCtrl c{};
        c.want = prm.want[j];
        c.share = prm.share[j];
        c.radius = prm.radius[j];
        c.bin = kSelBins;
        ctrl[j] = c;
    }
}

__global__ __launch_bounds__(kThreads) void pool_hist(const float *scores, int64_t L, const SelCtrl *ctrl, uint32_t *hist)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int j = blockIdx.y;
    const int r = (int)ctrl[j].radius;
    uint32_t *lh = (uint32_t *)smem;
    float *b0 = (float *)(smem + kSelBins * sizeof(uint32_t));
    float *b1 = b0 + kSelChunk + 2 * r;
    for (int i = threadIdx.x; i < kSelBins; i += kThreads) lh[i] = 0;
    float pooled[kPerThread];
    pooled_chunk(scores, L, blockIdx.x, r, b0, b1, pooled);  // has barriers: lh is cleared for all
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int64_t tok = (int64_t)blockIdx.x * kSelChunk + threadIdx.x + k * kThreads;
        if (tok < L) atomicAdd(&lh[ordered_bits(pooled[k]) >> 20], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kSelBins; i += kThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hist[(size_t)j * kSelBins + i], c);
    }
}

// Bin b with  count(bins > b) < want <= count(bins >= b).
__global__ __launch_bounds__(kThreads) void find_bin(const uint32_t *hist, SelCtrl *ctrl)
{
    __shared__ uint32_t wsum[kThreads / 64];
    const int j = blockIdx.x;
    const uint32_t want = ctrl[j].want;
    if (want == 0) return;  // ctrl.bin stays out of range: nothing is collected
    // thread i owns the 4 bins  top-4i, top-4i-1, ...  (top = kSelBins - 1), i.e. descending order
    uint32_t own[kPerThread], sum = 0;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        own[k] = hist[(size_t)j * kSelBins + (kSelBins - 1 - (threadIdx.x * kPerThread + k))];
        sum += own[k];
    }
    uint32_t total;
    const uint32_t incl = block_scan_inclusive(sum, wsum, total);
    uint32_t above = incl - sum;
    if (above < want && want <= incl) {
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            if (above < want && want <= above + own[k]) {
                ctrl[j].bin = kSelBins - 1 - (threadIdx.x * kPerThread + k);
                ctrl[j].above = above;
                ctrl[j].need = want - above;
            }
            above += own[k];
        }
    }
}

// Append the selected items of the block to a global list: one slot reservation per wavefront.
__device__ __forceinline__ void wave_append(bool pred, uint64_t key, uint64_t *list, uint32_t *counter)
{
    const uint64_t mask = __ballot(pred);
    if (mask == 0) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((unsigned long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(mask));
    base = __shfl(base, leader);
    if (pred) list[base + __popcll(mask & ((1ull << lane) - 1ull))] = key;
}

__global__ __launch_bounds__(kThreads) void collect(const float *scores, int64_t L, SelCtrl *ctrl, uint64_t *cand,
                                                    uint64_t *tie)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int j = blockIdx.y;
    const int r = (int)ctrl[j].radius;
    const uint32_t bin = ctrl[j].bin;
    if (bin >= (uint32_t)kSelBins) return;
    float *b0 = (float *)smem;
    float *b1 = b0 + kSelChunk + 2 * r;
    float pooled[kPerThread];
    pooled_chunk(scores, L, blockIdx.x, r, b0, b1, pooled);
    uint64_t *cand_j = cand + (size_t)j * kSortCap;
    uint64_t *tie_j = tie + (size_t)j * 2 * (size_t)L;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int64_t tok = (int64_t)blockIdx.x * kSelChunk + threadIdx.x + k * kThreads;
        const bool valid = tok < L;
        const uint32_t b = valid ? ordered_bits(pooled[k]) >> 20 : 0;
        const uint64_t key = make_key(pooled[k], (uint32_t)tok);
        wave_append(valid && b > bin, key, cand_j, &ctrl[j].cand_n);
        wave_append(valid && b == bin, key, tie_j, &ctrl[j].tie_n);
    }
}

// In-LDS bitonic sort, descending, of n (power of two) 64-bit keys by the whole block.
__device__ void bitonic_desc(uint64_t *s, int n)
{
    for (int k = 2; k <= n; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            for (int i = threadIdx.x; i < n; i += kThreads) {
                const int o = i ^ jj;
                if (o > i) {
                    const uint64_t x = s[i], y = s[o];
                    const bool down = (i & k) == 0;
                    if (down ? (x < y) : (x > y)) {
                        s[i] = y;
                        s[o] = x;
                    }
                }
            }
            __syncthreads();
        }
    }
}

__global__ __launch_bounds__(kThreads) void refine_sort(SelCtrl *ctrl, uint64_t *cand, uint64_t *tie, int64_t L)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t *sortbuf = (uint64_t *)smem;  // kSortCap keys
    __shared__ uint32_t h[256];
    __shared__ uint32_t cnt[2];
    __shared__ uint32_t pick[3];  // digit, count above it, count in it

    const int j = blockIdx.x;
    uint64_t *cand_j = cand + (size_t)j * kSortCap;
    uint64_t *A = tie + (size_t)j * 2 * (size_t)L;
    uint64_t *B = A + L;
    uint32_t nA = ctrl[j].tie_n;
    uint32_t need = ctrl[j].need;
    uint32_t candn = ctrl[j].cand_n;
    const int lane = threadIdx.x & 63;

    // The boundary list shares its top 12 key bits.  Peel 8 more bits a pass until few enough
    // survive (extra candidates below the cut are harmless: they rank last) or all are needed.
    for (int shift = 48; shift >= 0 && nA > (uint32_t)kSelSmall && need < nA; shift -= 8) {
        if (threadIdx.x < 256) h[threadIdx.x] = 0;
        if (threadIdx.x < 2) cnt[threadIdx.x] = 0;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < nA; i += kThreads) atomicAdd(&h[(A[i] >> shift) & 255u], 1u);
        __syncthreads();
        if (threadIdx.x < 64) {
            // lane l owns digits 255-4l .. 252-4l (descending); find the digit holding the need-th key
            uint32_t own[4], sum = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                own[k] = h[255 - (lane * 4 + k)];
                sum += own[k];
            }
            uint32_t incl = sum;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d);
                if (lane >= d) incl += y;
            }
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
            const uint64_t key = valid ? A[i] : 0;
            const uint32_t d = (uint32_t)(key >> shift) & 255u;
            wave_append(valid && d > digit, key, cand_j + candn, &cnt[0]);
            wave_append(valid && d == digit, key, B, &cnt[1]);
        }
        __threadfence();
        __syncthreads();
        candn += above;
        need -= above;
        nA = inside;
        uint64_t *t = A;
        A = B;
        B = t;
    }
    // what is left of the boundary list joins the candidates
    for (uint32_t i = threadIdx.x; i < nA; i += kThreads) cand_j[candn + i] = A[i];
    candn += nA;
    __threadfence();
    __syncthreads();

    int n2 = 1;
    while (n2 < (int)candn) n2 <<= 1;
    for (int i = threadIdx.x; i < n2; i += kThreads) sortbuf[i] = i < (int)candn ? cand_j[i] : 0ull;
    __syncthreads();
    bitonic_desc(sortbuf, n2);
    for (int i = threadIdx.x; i < (int)candn; i += kThreads) cand_j[i] = sortbuf[i];
    if (threadIdx.x == 0) ctrl[j].sorted_n = candn;
}

__device__ __forceinline__ uint32_t hash_slot(uint32_t token) { return (token * 0x9E3779B1u) >> 18; }

__global__ __launch_bounds__(kThreads) void walk(const SelCtrl *ctrl, const uint64_t *cand, int n, int n_out,
                                                 int32_t *out_idx)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = (uint32_t *)smem;                                  // kHashSlots
    uint64_t *sel = (uint64_t *)(smem + kHashSlots * sizeof(uint32_t));  // ILRE_MAX_BUDGET keys for the final sort
    __shared__ uint32_t wsum[kThreads / 64];

    for (int i = threadIdx.x; i < kHashSlots; i += kThreads) table[i] = kEmpty;
    __syncthreads();

    uint32_t nsel = 0;
    for (int j = 0; j < n; ++j) {
        const uint32_t cn = ctrl[j].sorted_n;
        const uint32_t share = ctrl[j].share;
        const uint64_t *cand_j = cand + (size_t)j * kSortCap;
        uint32_t taken = 0;
        for (uint32_t base = 0; base < cn && taken < share && nsel < (uint32_t)n_out; base += kThreads) {
            const uint32_t i = base + threadIdx.x;
            const bool valid = i < cn;
            const uint32_t token = valid ? key_token(cand_j[i]) : 0;
            bool free_tok = valid;
            if (valid) {
                uint32_t s = hash_slot(token);
                while (true) {
                    const uint32_t t = table[s];
                    if (t == kEmpty) break;
                    if (t == token) {
                        free_tok = false;
                        break;
                    }
                    s = (s + 1) & (kHashSlots - 1);
                }
            }
            uint32_t total;
            const uint32_t rank = block_scan_inclusive(free_tok ? 1u : 0u, wsum, total) - (free_tok ? 1u : 0u);
            uint32_t room = share - taken;
            if ((uint32_t)n_out - nsel < room) room = (uint32_t)n_out - nsel;
            if (free_tok && rank < room) {
                // descending order of the final bitonic sort = ascending token: key is the complement
                sel[nsel + rank] = (uint64_t)(0xFFFFFFFFu - token);
                uint32_t s = hash_slot(token);
                while (true) {
                    const uint32_t old = atomicCAS(&table[s], kEmpty, token);
                    if (old == kEmpty || old == token) break;
                    s = (s + 1) & (kHashSlots - 1);
                }
            }
            const uint32_t got = total < room ? total : room;
            taken += got;
            nsel += got;
            __syncthreads();
        }
    }

    int n2 = 1;
    while (n2 < (int)nsel) n2 <<= 1;
    for (int i = nsel + threadIdx.x; i < n2; i += kThreads) sel[i] = 0ull;
    __syncthreads();
    bitonic_desc(sel, n2);
    for (int i = threadIdx.x; i < n_out; i += kThreads)
        out_idx[i] = i < (int)nsel ? (int32_t)(0xFFFFFFFFu - (uint32_t)sel[i]) : -1;
}

}  // namespace

SelectLayout make_select_layout(int64_t L, int n_kernels)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    SelectLayout lay{};
    size_t off = 0;
    lay.hist = off;
    off = up(off + (size_t)n_kernels * kSelBins * sizeof(uint32_t));
    lay.ctrl = off;
    off = up(off + (size_t)n_kernels * sizeof(SelCtrl));
    lay.cand = off;
    off = up(off + (size_t)n_kernels * kSortCap * sizeof(uint64_t));
    lay.tie = off;
    off = up(off + (size_t)n_kernels * 2 * (size_t)L * sizeof(uint64_t));
    lay.total = off;
    return lay;
}

hipError_t launch_select(const float *scores, int64_t L, int budget, const int32_t *pool_kernels, int n_kernels,
                         int32_t *out_idx, void *workspace, const SelectLayout &lay, hipStream_t s)
{
    SelParams prm{};
    prm.n = n_kernels;
    prm.L = L;
    const int base = budget / n_kernels, rem = budget % n_kernels;
    int64_t before = 0;
    int rmax = 0;
    for (int j = 0; j < n_kernels; ++j) {
        const int share = base + (j < rem ? 1 : 0);
        const int64_t want = before + share < L ? before + share : L;
        prm.radius[j] = (uint32_t)((pool_kernels[j] - 1) / 2);
        prm.share[j] = (uint32_t)share;
        prm.want[j] = (uint32_t)want;
        before += share;
        if ((int)prm.radius[j] > rmax) rmax = (int)prm.radius[j];
    }
    unsigned char *ws = (unsigned char *)workspace;
    uint32_t *hist = (uint32_t *)(ws + lay.hist);
    SelCtrl *ctrl = (SelCtrl *)(ws + lay.ctrl);
    uint64_t *cand = (uint64_t *)(ws + lay.cand);
    uint64_t *tie = (uint64_t *)(ws + lay.tie);
    const unsigned nchunks = (unsigned)((L + kSelChunk - 1) / kSelChunk);
    const int n_out = (int)(budget < L ? budget : L);
    const size_t pool_lds = 2 * (size_t)(kSelChunk + 2 * rmax) * sizeof(float);
    const size_t hist_lds = pool_lds + kSelBins * sizeof(uint32_t);
    const size_t sort_lds = (size_t)kSortCap * sizeof(uint64_t);
    const size_t walk_lds = kHashSlots * sizeof(uint32_t) + (size_t)ILRE_MAX_BUDGET * sizeof(uint64_t);

    hipError_t e;
    if ((e = hipFuncSetAttribute((const void *)pool_hist, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hist_lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)collect, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pool_lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)refine_sort, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sort_lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)walk, hipFuncAttributeMaxDynamicSharedMemorySize, (int)walk_lds)) != hipSuccess) return e;

    hipLaunchKernelGGL(sel_init, dim3(n_kernels), dim3(kThreads), 0, s, prm, hist, ctrl);
    hipLaunchKernelGGL(pool_hist, dim3(nchunks, n_kernels), dim3(kThreads), hist_lds, s, scores, L, ctrl, hist);
    hipLaunchKernelGGL(find_bin, dim3(n_kernels), dim3(kThreads), 0, s, hist, ctrl);
    hipLaunchKernelGGL(collect, dim3(nchunks, n_kernels), dim3(kThreads), pool_lds, s, scores, L, ctrl, cand, tie);
    hipLaunchKernelGGL(refine_sort, dim3(n_kernels), dim3(kThreads), sort_lds, s, ctrl, cand, tie, L);
    hipLaunchKernelGGL(walk, dim3(1), dim3(kThreads), walk_lds, s, ctrl, cand, n_kernels, n_out, out_idx);
    return hipGetLastError();
}

}  // namespace ilre
