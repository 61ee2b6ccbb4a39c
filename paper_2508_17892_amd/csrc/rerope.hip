// DCA re-RoPE of the retrieval layer's key cache (paper Section 3.3, second DCA equation) for gfx950.
//
// Before the recall step the keys of prefill chunk i are turned by R(D_i), D_i = the distance in
// tokens between chunk i and chunk N_C - 1 (the positional base), for i < N_C - 1; the last two
// chunks stay as they are.  R(D) is the rotary embedding's rotation by D positions: pair j of a key
// vector turns by D * inv_freq[j].  One streaming pass: every key element is read once and written
// once (16-byte accesses), the rotation runs in fp32 and the result is rounded to the cache's type.
//
// A workgroup owns 1024 consecutive tokens of one kv head.  The angles depend on the chunk only:
// 64 lanes evaluate sin/cos of D * inv_freq[j] in fp64 (the angles reach 10^6 rad at 1M tokens, far
// beyond what an fp32 argument reduction resolves) once per chunk the workgroup touches, and every
// thread keeps the values of its own pairs in registers while it streams that chunk's tokens.
#include "ilre_internal.h"

namespace ilre {
namespace {

constexpr int kRopeThreads = 256;
constexpr int kRopeTokens = 1024;  // tokens per workgroup
constexpr int kPairs = ILRE_HEAD_DIM / 2;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
// round to nearest even; the inputs are finite
__device__ __forceinline__ uint32_t to_bf16(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// The NP pairs a thread owns, unpacked from one (interleaved) or two (half-split) 16-byte chunks.
template <int DT, int PAIRING>
struct Lanes {
    static constexpr int ES = DT == ILRE_BF16 ? 2 : 4;
    static constexpr int E = 16 / ES;                                   // elements per 16-byte chunk
    static constexpr int NP = PAIRING == ILRE_ROPE_HALF ? E : E / 2;    // pairs per thread
    static constexpr int TPT = kPairs / NP;                             // threads per token
};

template <int DT>
__device__ __forceinline__ void unpack(const uint4 &v, float (&f)[16 / (DT == ILRE_BF16 ? 2 : 4)])
{
    if (DT == ILRE_BF16) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = bf16_lo(w[i]);
            f[2 * i + 1] = bf16_hi(w[i]);
        }
    } else {
        f[0] = __uint_as_float(v.x);
        f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z);
        f[3] = __uint_as_float(v.w);
    }
}

template <int DT>
__device__ __forceinline__ uint4 pack(const float (&f)[16 / (DT == ILRE_BF16 ? 2 : 4)])
{
    uint4 v;
    if (DT == ILRE_BF16) {
        v.x = to_bf16(f[0]) | (to_bf16(f[1]) << 16);
        v.y = to_bf16(f[2]) | (to_bf16(f[3]) << 16);
        v.z = to_bf16(f[4]) | (to_bf16(f[5]) << 16);
        v.w = to_bf16(f[6]) | (to_bf16(f[7]) << 16);
    } else {
        v.x = __float_as_uint(f[0]);
        v.y = __float_as_uint(f[1]);
        v.z = __float_as_uint(f[2]);
        v.w = __float_as_uint(f[3]);
    }
    return v;
}

template <int DT, int PAIRING>
__global__ __launch_bounds__(kRopeThreads) void rerope_kernel(const RopeArgs a)
{
    using LN = Lanes<DT, PAIRING>;
    constexpr int ES = LN::ES, E = LN::E, NP = LN::NP, TPT = LN::TPT;
    constexpr int ROWS = kRopeThreads / TPT;  // tokens per sweep of the workgroup
    constexpr int UNROLL = 8;
    __shared__ float cs[2][kPairs];  // cos, sin of the current chunk

    const int head = blockIdx.y;
    const int64_t slice0 = (int64_t)blockIdx.x * kRopeTokens;
    const int64_t slice1 = slice0 + kRopeTokens < a.L ? slice0 + kRopeTokens : a.L;
    const int c = threadIdx.x % TPT, row = threadIdx.x / TPT;
    const int j0 = NP * c;  // first pair of this thread
    const int64_t head_off = (int64_t)head * a.stride_head * ES;
    const int64_t row_bytes = a.stride_token * ES;
    // byte offsets of the thread's chunk(s) inside a key row
    const int off_a = PAIRING == ILRE_ROPE_HALF ? j0 * ES : 2 * j0 * ES;
    const int off_b = (kPairs + j0) * ES;  // half-split only

    int64_t t = slice0;
    while (t < slice1) {  // one round per prefill chunk the slice touches (uniform)
        const int64_t first_len = (int64_t)a.first_extra + a.chunk;
        const int64_t ci = t < first_len ? 0 : (t - a.first_extra) / a.chunk;
        int64_t sub1 = (int64_t)a.first_extra + (ci + 1) * a.chunk;
        if (sub1 > slice1) sub1 = slice1;
        const int64_t dist = ci < (int64_t)a.nchunks - 2 ? ((int64_t)a.nchunks - 2 - ci) * a.chunk : 0;
        if (dist == 0 && a.in == a.out) {  // nothing to do in place
            t = sub1;
            continue;
        }
        __syncthreads();  // the previous round's readers of cs are done
        if (threadIdx.x < kPairs) {
            double s, co;
            sincos((double)dist * a.inv_freq[threadIdx.x], &s, &co);
            cs[0][threadIdx.x] = (float)co;
            cs[1][threadIdx.x] = (float)s;
        }
        __syncthreads();
        float co[NP], si[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            co[p] = cs[0][j0 + p];
            si[p] = cs[1][j0 + p];
        }
        for (int64_t tb = t + row; tb < sub1; tb += (int64_t)ROWS * UNROLL) {
            uint4 va[UNROLL], vb[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t tok = tb + (int64_t)u * ROWS;
                if (tok < sub1) {
                    const unsigned char *src = a.in + head_off + tok * row_bytes;
                    va[u] = *(const uint4 *)(src + off_a);
                    if (PAIRING == ILRE_ROPE_HALF) vb[u] = *(const uint4 *)(src + off_b);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t tok = tb + (int64_t)u * ROWS;
                if (tok < sub1) {
                    unsigned char *dst = a.out + head_off + tok * row_bytes;
                    float x[E], y[E];
                    unpack<DT>(va[u], x);
                    if (PAIRING == ILRE_ROPE_HALF) {
                        unpack<DT>(vb[u], y);
#pragma unroll
                        for (int p = 0; p < NP; ++p) {
                            const float xr = x[p] * co[p] - y[p] * si[p];
                            const float yr = y[p] * co[p] + x[p] * si[p];
                            x[p] = xr;
                            y[p] = yr;
                        }
                        *(uint4 *)(dst + off_a) = pack<DT>(x);
                        *(uint4 *)(dst + off_b) = pack<DT>(y);
                    } else {
#pragma unroll
                        for (int p = 0; p < NP; ++p) {
                            const float xr = x[2 * p] * co[p] - x[2 * p + 1] * si[p];
                            const float yr = x[2 * p + 1] * co[p] + x[2 * p] * si[p];
                            x[2 * p] = xr;
                            x[2 * p + 1] = yr;
                        }
                        *(uint4 *)(dst + off_a) = pack<DT>(x);
                    }
                }
            }
        }
        t = sub1;
    }
}

}  // namespace

hipError_t launch_rerope(const RopeArgs &a, int dtype, int pairing, hipStream_t s)
{
    const dim3 grid((unsigned)((a.L + kRopeTokens - 1) / kRopeTokens), (unsigned)a.Hkv);
    if (dtype == ILRE_BF16) {
        if (pairing == ILRE_ROPE_HALF)
            hipLaunchKernelGGL((rerope_kernel<ILRE_BF16, ILRE_ROPE_HALF>), grid, dim3(kRopeThreads), 0, s, a);
        else
            hipLaunchKernelGGL((rerope_kernel<ILRE_BF16, ILRE_ROPE_INTERLEAVED>), grid, dim3(kRopeThreads), 0, s, a);
    } else {
        if (pairing == ILRE_ROPE_HALF)
            hipLaunchKernelGGL((rerope_kernel<ILRE_F32, ILRE_ROPE_HALF>), grid, dim3(kRopeThreads), 0, s, a);
        else
            hipLaunchKernelGGL((rerope_kernel<ILRE_F32, ILRE_ROPE_INTERLEAVED>), grid, dim3(kRopeThreads), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace ilre
