// Measurement aid, not part of the recall path: register-only loops with the instruction mix of the scoring
// kernels (paper Section 3.2, Eq. 4 / Eq. 5: per 32x32 block of logits 8 bf16 MFMAs, and per logit one fma,
// one exp2 and one add), with no LDS, no global loads and no barriers in the loop.  What these loops reach
// on random bf16 operands is the most any kernel with this mix can reach on the chip at hand, which is
// what the measured rate of the scoring kernels is to be read against.
//
// A wavefront holds NB query-block fragments and one key fragment set in registers and runs, per
// iteration, two "units": NB chains of 8 MFMAs into one accumulator set while the vector work consumes
// the other set (the software pipeline of the scoring kernels).  The key fragments pass through an empty
// asm statement every unit, so the compiler treats them as new data and keeps every MFMA in the loop.
#include "ilre_internal.h"

namespace ilre {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

// 2^x without the transcendental unit: x = i + f with i = round(x), f in [-0.5, 0.5]; 2^f by a degree-4
// polynomial (relative error about 4e-6), times 2^i by adding i to the exponent field.
__device__ __forceinline__ float poly_exp2(float x)
{
    const float magic = 12582912.0f;  // 1.5 * 2^23: the sum's low mantissa bits hold round(x)
    const float t = x + magic;
    const float f = x - (t - magic);
    float p = 9.6181291e-3f;
    p = __builtin_fmaf(p, f, 5.5504109e-2f);
    p = __builtin_fmaf(p, f, 2.4022651e-1f);
    p = __builtin_fmaf(p, f, 6.9314718e-1f);
    p = __builtin_fmaf(p, f, 1.0f);
    return __uint_as_float(__float_as_uint(p) + (__float_as_uint(t) << 23));
}

// VALU: 0 none (MFMAs only), 1 fma + exp2 + add per accumulator element (the kernels' mix),
//       2 fma + add only, 3 exp2 + add only,
//       4 the mix with every exp2 computed on the plain vector pipe (round, subtract, degree-4 polynomial,
//         exponent add: 8 plain instructions in place of one transcendental), 5 every other exp2 so
// MFMA: false = the vector work alone, on accumulators the compiler must take as new data every unit
//       (rates are then quoted for the MFMAs that were left out)
template <int NB, int WAVES, int VALU, bool MFMA = true>
__global__ __launch_bounds__(WAVES * 64) void ceiling_kernel(const uint4 *src, int iters, float c, float *out,
                                                             unsigned long long *clocks)
{
    unsigned long long t0 = 0, w0 = 0;
    if (threadIdx.x == 0) {
        t0 = clock64();
        w0 = wall_clock64();
    }
    f32x16 acc[2][NB];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[u][b][i] = 0.f;
    uint4 q[NB][8], k[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        k[i] = src[(threadIdx.x + 64 * i) % 4096];
#pragma unroll
        for (int b = 0; b < NB; ++b) q[b][i] = src[(threadIdx.x * (2 * b + 3) + 64 * i + 1024 * (b + 1)) % 4096];
    }
    float z[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) z[b] = 0.f;
    const float off = -3.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int st = 0; st < 8; ++st) asm volatile("" : "+v"(k[st].x));
            if (MFMA) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[u][b][v] = 0.f;
#pragma unroll
                for (int st = 0; st < 8; ++st)
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[u][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q[b][st]),
                                                                            __builtin_bit_cast(bf16x8, k[st]), acc[u][b], 0, 0, 0);
            } else {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[u][b][v]));
            }
            if (VALU == 0) {
                // one read per accumulator set keeps the chains alive without vector work worth the name
#pragma unroll
                for (int b = 0; b < NB; ++b) z[b] += acc[u ^ 1][b][b];
            } else {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const f32x16 &a = acc[u ^ 1][b];  // the unit before this one
                    float p[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        if (VALU == 1) p[v & 3] += __builtin_amdgcn_exp2f(__builtin_fmaf(a[v], c, off));
                        if (VALU == 2) p[v & 3] += __builtin_fmaf(a[v], c, off);
                        if (VALU == 3) p[v & 3] += __builtin_amdgcn_exp2f(a[v]);
                        if (VALU == 4) p[v & 3] += poly_exp2(__builtin_fmaf(a[v], c, off));
                        if (VALU == 5)
                            p[v & 3] += (v & 1) ? poly_exp2(__builtin_fmaf(a[v], c, off))
                                                : __builtin_amdgcn_exp2f(__builtin_fmaf(a[v], c, off));
                    }
                    z[b] += (p[0] + p[1]) + (p[2] + p[3]);
                }
                // one MFMA, then its share of the vector work, as in the scoring kernels
                constexpr int kPerMfma = VALU == 1 ? 6 : (VALU == 4 ? 22 : (VALU == 5 ? 14 : 4));
                if (MFMA) {
#pragma unroll
                    for (int st = 0; st < 8; ++st)
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x002, kPerMfma, 0);
                        }
                }
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b) s += z[b];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) s += acc[u][b][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        clocks[blockIdx.x * 2 + 0] = clock64() - t0;
        clocks[blockIdx.x * 2 + 1] = wall_clock64() - w0;
    }
}

struct Variant {
    int nb, waves, valu;
    const char *what;
    bool mfma = true;
};
const Variant kVariants[] = {
    {2, 8, 0, "MFMAs only: 8 wavefronts x 64 query rows (the scoring kernels' shape), 2 per SIMD"},
    {2, 8, 1, "the scoring kernels' mix: 8 wavefronts x 64 rows, fma + exp2 + add per logit"},
    {4, 4, 0, "MFMAs only: 4 wavefronts x 128 rows, 1 per SIMD"},
    {4, 4, 1, "the mix: 4 wavefronts x 128 rows, 1 per SIMD"},
    {2, 8, 2, "8 wavefronts x 64 rows, fma + add per logit, no exp2"},
    {2, 8, 3, "8 wavefronts x 64 rows, exp2 + add per logit"},
    {1, 16, 1, "the mix: 16 wavefronts x 32 rows, 4 per SIMD"},
    {1, 16, 0, "MFMAs only: 16 wavefronts x 32 rows, 4 per SIMD"},
    {2, 8, 4, "8 wavefronts x 64 rows, the mix with exp2 as 8 plain vector instructions (no transcendental)"},
    {2, 8, 5, "8 wavefronts x 64 rows, the mix with every other exp2 as 8 plain vector instructions"},
    {2, 8, 1, "no MFMAs: the vector work of the mix alone (fma + exp2 + add per logit), 8 wavefronts; rate quoted for the MFMAs left out", false},
    {2, 8, 2, "no MFMAs: fma + add per logit alone, 8 wavefronts", false},
    {2, 8, 3, "no MFMAs: exp2 + add per logit alone, 8 wavefronts", false},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

}  // namespace

int probe_variants() { return kNumVariants; }

const char *probe_describe(int variant) { return variant >= 0 && variant < kNumVariants ? kVariants[variant].what : nullptr; }

hipError_t launch_probe(int variant, int iters, const void *operands, float *out, unsigned long long *clocks, double *flops,
                        hipStream_t s)
{
    const Variant &v = kVariants[variant];
    const dim3 grid(kNumCU), block(v.waves * 64);
    const uint4 *src = (const uint4 *)operands;
    const float c = 0.01f;
#define ILRE_PROBE(NB, WAVES, VALU)                                                                                  \
    if (v.nb == NB && v.waves == WAVES && v.valu == VALU && v.mfma)                                                  \
        hipLaunchKernelGGL((ceiling_kernel<NB, WAVES, VALU>), grid, block, 0, s, src, iters, c, out, clocks);
    ILRE_PROBE(2, 8, 0)
    ILRE_PROBE(2, 8, 1)
    ILRE_PROBE(4, 4, 0)
    ILRE_PROBE(4, 4, 1)
    ILRE_PROBE(2, 8, 2)
    ILRE_PROBE(2, 8, 3)
    ILRE_PROBE(1, 16, 1)
    ILRE_PROBE(1, 16, 0)
    ILRE_PROBE(2, 8, 4)
    ILRE_PROBE(2, 8, 5)
#undef ILRE_PROBE
    if (!v.mfma && v.valu == 1) hipLaunchKernelGGL((ceiling_kernel<2, 8, 1, false>), grid, block, 0, s, src, iters, c, out, clocks);
    if (!v.mfma && v.valu == 2) hipLaunchKernelGGL((ceiling_kernel<2, 8, 2, false>), grid, block, 0, s, src, iters, c, out, clocks);
    if (!v.mfma && v.valu == 3) hipLaunchKernelGGL((ceiling_kernel<2, 8, 3, false>), grid, block, 0, s, src, iters, c, out, clocks);
    // MFMAs: grid x wavefronts x iterations x 2 units x NB chains x 8, each 32*32*16*2 flop
    *flops = (double)kNumCU * v.waves * (double)iters * 2.0 * v.nb * 8.0 * 32768.0;
    return hipGetLastError();
}

}  // namespace ilre
