/*
 * libilre -- intermediate-layer token recall for context compression on MI355X (gfx950).
 *
 * Given the query states of a short question and the full-length key cache of one decoder
 * layer (the retrieval layer l_R of the paper), score every context token, pool the scores
 * with several kernel sizes, and return the indices of the tokens to keep.
 *
 *   Section 3.2, Eq. 4   A[h,i,t] = softmax_t( q[h,i,:] . K[g(h),t,:] * scale ), softmax over all L
 *                        context positions, no mask; GQA: g(h) = h / (Hq/Hkv) (consecutive groups).
 *   Section 3.2, Eq. 5   reduction over heads and queries to one score per context token:
 *                        ILRE_SCORE_SUM  score[t] = sum_{h,i} A[h,i,t]   (default of this library)
 *                        ILRE_SCORE_MAX  score[t] = max_{h,i} A[h,i,t]   (the equation as printed)
 *   Section 3.2, Algorithm 1 (Context Allocation), stride-1 max-pool form: for each kernel size
 *                        w_j in the order given, pooled_j[t] = max(score[u] : |u-t| <= (w_j-1)/2,
 *                        0 <= u < L); among tokens not yet allocated take the B_j with the largest
 *                        pooled_j (ties: lower index first); B_j = floor(B/n) (+1 for the first
 *                        B mod n kernels); finally the allocated set sorted ascending.
 *   Section 3.2, Algorithm 1 as printed (the *_max_avg entry points): the first `sink` tokens are
 *                        always allocated and the pooling sees body = score[sink..L).  For each max
 *                        kernel m_i (outer loop) and average kernel n_j (inner loop):
 *                        cell[p] = max(body[p*m_i .. p*m_i+m_i-1]) for the floor(len/m_i) whole cells;
 *                        avg[p] = (cell[p-a] + ... + cell[p+b]) / n_j, a = (n_j-1)/2, b = n_j/2 (integer
 *                        division), zeros outside the array, summed left to right in fp32; the
 *                        K_m = B/m_i + 1 cells with the largest avg (ties: lower cell first) are the
 *                        candidates, walked in that order, each as its m_i tokens in ascending order,
 *                        and the first B_c tokens not yet allocated are taken, B_c = floor(B/(N_M N_A))
 *                        (+1 for the first B mod (N_M N_A) combinations).  A combination whose
 *                        candidates run out takes fewer, so fewer than B tokens may come back.
 *
 * Conventions for every entry point
 *   - returns an ilre_status; never throws, never aborts, never synchronises the device;
 *   - "dev" pointers are device memory owned by the caller, "host" pointers host memory; the
 *     library keeps no pointer after a call returns and frees nothing of the caller's;
 *   - work is enqueued on opts->stream (NULL = the default stream) and the call returns at once;
 *   - the library allocates no device memory: scratch comes from opts->workspace, sized by
 *     ilre_workspace_bytes() for the same shape arguments; calls that share a workspace must be
 *     ordered on one stream;
 *   - inputs are read-only, outputs are fully overwritten, results are bitwise reproducible from
 *     run to run on the same device;
 *   - Q and K must hold finite values.
 *   - on error nothing is enqueued (argument errors) or the stream state is unspecified
 *     (ILRE_EHIP); ilre_last_error() describes the last error of the calling thread.
 */
#ifndef ILRE_H
#define ILRE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ILRE_OK = 0,
    ILRE_EINVAL = 1,        /* null pointer, non-positive size, Hq % Hkv != 0, even / non-positive kernel size, sink outside [0, L] */
    ILRE_EUNSUPPORTED = 2,  /* head_dim != 128, unknown dtype / score mode, budget or kernel size over the limits below */
    ILRE_ENOMEM = 3,        /* workspace missing or smaller than ilre_workspace_bytes() */
    ILRE_EHIP = 4           /* a HIP call failed; see ilre_last_error() */
} ilre_status;

typedef enum { ILRE_F32 = 0, ILRE_BF16 = 1 } ilre_dtype;
typedef enum { ILRE_SCORE_SUM = 0, ILRE_SCORE_MAX = 1 } ilre_score_mode;
/* which elements of a key vector form rotary pair j: (x[j], x[j + d/2]) or (x[2j], x[2j+1]) */
typedef enum { ILRE_ROPE_HALF = 0, ILRE_ROPE_INTERLEAVED = 1 } ilre_rope_pairing;

/* ilre_row_stats / ilre_recall: follow the running row maximum over the whole context, so that the
   reference written to row_ref is exactly max_t logit (a few percent slower).  Without it the
   reference is a maximum over part of the context, which normalises just as well. */
#define ILRE_FLAG_EXACT_ROW_MAX 1

#define ILRE_HEAD_DIM 128        /* the only supported head dimension */
#define ILRE_MAX_BUDGET 8192     /* largest budget when budget < L (budget >= L needs L <= 8192) */
#define ILRE_MAX_POOL_KERNEL 2047 /* largest pooling kernel size */
#define ILRE_MAX_POOL_KERNELS 64 /* most kernel sizes (or max/average combinations) in one call */
#define ILRE_MAX_MAX_KERNEL 1024 /* largest strided max-pooling kernel (the *_max_avg entry points) */
#define ILRE_MAX_AVG_KERNEL 1024 /* largest average-pooling kernel */
#define ILRE_STATIC_SCRATCH_BYTES (4u << 20) /* scratch built into the library for ilre_row_stats_static, per GPU */

typedef struct {
    int32_t struct_size;     /* sizeof(ilre_opts), for versioning */
    int32_t dtype;           /* ilre_dtype of q and k_cache */
    int32_t n_pool_kernels;  /* length of pool_kernels (selection entry points) */
    int32_t score_mode;      /* ilre_score_mode */
    float scale;             /* softmax scale; 0 means 1/sqrt(d) */
    int32_t flags;           /* ILRE_FLAG_* bits */
    int64_t k_stride_head;   /* elements between kv heads of k_cache;  0 = contiguous [Hkv, L, d] */
    int64_t k_stride_token;  /* elements between tokens of k_cache;    0 = contiguous */
    int64_t q_stride_head;   /* elements between heads of q;           0 = contiguous [Hq, Lq, d] */
    int64_t q_stride_token;  /* elements between query tokens of q;    0 = contiguous */
    void *workspace;         /* dev, 256-byte aligned */
    size_t workspace_bytes;
    void *stream;            /* hipStream_t */
    int32_t sink;            /* ilre_recall / ilre_select: leading tokens that are always kept (the sink part of
                                Algorithm 1); the pooling sees score[sink..L) and the budget counts the other tokens */
    int32_t reserved;        /* 0 */
} ilre_opts;

/* Bytes of device workspace any entry point needs for this shape (host computation only).
   out_bytes: host. */
int ilre_workspace_bytes(int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                         int32_t n_pool_kernels, int32_t dtype, size_t *out_bytes);

/* The whole path: Eq. 4, Eq. 5, Algorithm 1.
   q          dev  [Hq, Lq, d] (strides in opts), element type opts->dtype, innermost d contiguous
   k_cache    dev  [Hkv, L, d] (strides in opts; token-major [L, Hkv, d] is expressible)
   pool_kernels host, opts->n_pool_kernels odd sizes >= 1, processed in this order
   out_idx    dev  opts->sink + min(budget, L - opts->sink) int32, ascending, unique: the sink indices
                   0 .. sink-1, then the allocated tokens
   out_scores dev  L float, 16-byte aligned, the un-pooled per-token score of Eq. 5 (all positions, the
                   sink part included: the softmax of Eq. 4 runs over all L) */
int ilre_recall(const void *q, const void *k_cache,
                int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                int32_t budget, const int32_t *pool_kernels,
                int32_t *out_idx, float *out_scores, const ilre_opts *opts);

/* Stage 1 (Eq. 4 row statistics): for every row r = h*Lq + i a reference logit and the sum of
   exponentials against it, i.e. the softmax normaliser in two parts:
       row_sumexp[r] = sum_t exp(logit[r,t] - row_ref[r]),   log sum_t exp(logit[r,t]) = row_ref[r] + log row_sumexp[r].
   row_ref[r] <= max_t logit[r,t]; it equals the maximum with ILRE_FLAG_EXACT_ROW_MAX, otherwise it is
   the maximum over the first tokens of the row's context splits (row_sumexp stays finite: a part of the
   context whose sums would leave the safe range is walked again against the running maximum).  Both dev, Hq*Lq float.
   Needs the head of the workspace only (the partial statistics); given a workspace of ilre_workspace_bytes it
   also leaves there, on long contexts, how fast each part of the chip ran, for a later ilre_col_scores. */
int ilre_row_stats(const void *q, const void *k_cache,
                   int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                   float *row_ref, float *row_sumexp, const ilre_opts *opts);

/* ilre_row_stats for callers that cannot allocate device memory or pass a workspace: code running under HIP
   graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
   bit-identical results; the per-split partial statistics live in a buffer of
   ILRE_STATIC_SCRATCH_BYTES built into the library (one copy per GPU, held until the process ends) instead
   of opts->workspace, which is not read.  Makes no allocating call.  ILRE_EUNSUPPORTED when the shape needs
   more scratch than the buffer holds (2 * 4 bytes per query row and token split, plus 512; the 1M-token
   workload with 8192 rows needs 1 MiB).  Every call on a GPU shares that GPU's buffer: calls that overlap
   on one GPU (different streams, or different threads without ordering) race; calls ordered on one stream
   do not.  Nothing in the buffer needs to start at zero and nothing of an earlier call is read. */
int ilre_row_stats_static(const void *q, const void *k_cache,
                          int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                          float *row_ref, float *row_sumexp, const ilre_opts *opts);

/* Stage 2 (Eq. 4 normalised, Eq. 5): recompute the logits, normalise with the given row
   statistics (any pair with the right row_ref + log row_sumexp) and reduce over heads and queries.
   row_ref,row_sumexp: dev, as written by ilre_row_stats.  out_scores: dev, L float.
   On long contexts, a workspace in which an ilre_row_stats call of the same shape left its timings lets this call
   size each workgroup's token range by the speed of the XCD it runs on; the scores are the same bits with or
   without (the table is recognised by a header and ignored otherwise, whatever the workspace holds). */
int ilre_col_scores(const void *q, const void *k_cache,
                    int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                    const float *row_ref, const float *row_sumexp,
                    float *out_scores, const ilre_opts *opts);

/* Stages 3-4 (Algorithm 1): pooling, budgeted top-k with skip-allocated, ascending output.
   scores: dev, L finite floats, 16-byte aligned.  pool_kernels: host.
   out_idx: dev, opts->sink + min(budget, L - opts->sink) int32. */
int ilre_select(const float *scores, int64_t L, int32_t budget, const int32_t *pool_kernels,
                int32_t *out_idx, const ilre_opts *opts);

/* Algorithm 1 as printed (strided max pooling, stride-1 average pooling, K_m cap, sink part); see the
   top of this file for the exact definition.  The paper's default is max kernels {2,4,8}, average
   kernels {1..16}, sink 4.
   scores      dev  L finite floats (all positions, the sink part included)
   sink        leading tokens always kept, 0 <= sink <= L; budget counts the other tokens
   max_kernels host n_max sizes in [1, ILRE_MAX_MAX_KERNEL]; avg_kernels host n_avg sizes in
               [1, ILRE_MAX_AVG_KERNEL]; n_max * n_avg <= ILRE_MAX_POOL_KERNELS
   out_idx     dev  sink + min(budget, L - sink) int32: the sink indices, then the allocated tokens
               ascending, then -1 in the slots a run of exhausted candidates left unused
   out_count   dev  one int32, the number of valid leading entries of out_idx; may be NULL
   workspace   sized by ilre_workspace_bytes_max_avg for the same L, sink and max kernels */
int ilre_select_max_avg(const float *scores, int64_t L, int32_t sink, int32_t budget,
                        const int32_t *max_kernels, int32_t n_max,
                        const int32_t *avg_kernels, int32_t n_avg,
                        int32_t *out_idx, int32_t *out_count, const ilre_opts *opts);

/* The whole path with Algorithm 1 as printed: Eq. 4 over all L positions, Eq. 5, then
   ilre_select_max_avg on the scores.  q, k_cache, out_scores as for ilre_recall; the other arguments
   as for ilre_select_max_avg.  opts->n_pool_kernels is not read. */
int ilre_recall_max_avg(const void *q, const void *k_cache,
                        int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                        int32_t sink, int32_t budget,
                        const int32_t *max_kernels, int32_t n_max,
                        const int32_t *avg_kernels, int32_t n_avg,
                        int32_t *out_idx, int32_t *out_count, float *out_scores, const ilre_opts *opts);

/* Workspace bytes for the two *_max_avg entry points (host computation only; the sizes of the
   average kernels do not matter).  max_kernels, out_bytes: host. */
int ilre_workspace_bytes_max_avg(int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d, int32_t sink,
                                 const int32_t *max_kernels, int32_t n_max, int32_t n_avg,
                                 int32_t dtype, size_t *out_bytes);

/* Last line of Algorithm 1: the compressed prompt C[I], i.e. out[i] = input_ids[idx[i]] for the n entries
   of an index list written by one of the selection entry points; entries that are -1 (unused slots of the
   printed form) or out of range give -1.  input_ids: dev, L int32.  idx: dev, n int32.  out: dev, n int32
   (must not overlap idx).  Needs no workspace; opts supplies the stream. */
int ilre_gather_ids(const int32_t *input_ids, int64_t L, const int32_t *idx, int32_t n, int32_t *out,
                    const ilre_opts *opts);

/* DCA re-RoPE of the retrieval layer's key cache (Section 3.3, second DCA equation), to be run before
   the recall step when DCA is on.  The context is the sequence of prefill chunks 1..N_C: chunk 1 holds
   first_extra + chunk_tokens tokens (the sink part rides with it), the others chunk_tokens, the last one
   what is left; N_C = max(1, ceil((L - first_extra) / chunk_tokens)).  The keys of chunk i < N_C - 1 are
   turned by R(D_i), D_i = (N_C - 1 - i) * chunk_tokens: pair j of a key vector (see ilre_rope_pairing)
   goes from (x, y) to (x cos a - y sin a, y cos a + x sin a) with a = D_i * inv_freq[j], which moves a key
   embedded at position p to p + D_i.  Chunks N_C - 1 and N_C are copied unchanged.  Angles are evaluated
   in fp64, the rotation in fp32, the result is rounded to the cache's element type (nearest even).
   k_in      dev  [Hkv, L, d], element type opts->dtype, layout by opts->k_stride_head / k_stride_token
   k_out     dev  same shape, type and strides; may be k_in itself (in place), must not overlap it otherwise
   inv_freq  host d/2 doubles, or NULL for rope_base^(-2j/d) (rope_base > 0)
   Needs no workspace. */
int ilre_rerope_keys(const void *k_in, void *k_out, int64_t L, int32_t Hkv, int32_t d,
                     int32_t chunk_tokens, int32_t first_extra, double rope_base, const double *inv_freq,
                     int32_t pairing, const ilre_opts *opts);

/* Measurement aid, not a step of the method: register-only loops with the instruction mix of the two scoring
   passes (Section 3.2, Eq. 4 / Eq. 5: 8 bf16 MFMAs per 32x32 block of logits; one fma, one exp2 and one add per
   logit), no LDS, no loads and no barriers inside the loop, one workgroup per compute unit.  The rate such a
   loop reaches on the caller's operands bounds what the scoring kernels can reach on the same chip.
   variant    0 .. (number of variants - 1); ilre_probe_describe(variant) names it, NULL past the last one
   iters      loop iterations per wavefront (>= 1); one iteration is 2 units of 8 MFMAs per 32 query rows
   operands   dev  ILRE_PROBE_OPERAND_BYTES of bf16 values the MFMA fragments are read from (once, before the loop)
   out        dev  ILRE_PROBE_OUT_BYTES, 256-byte aligned: 1 MiB of floats nobody needs (they keep the loop alive),
                   then per workgroup two uint64: shader clock cycles and 100 MHz wall ticks the workgroup ran for
   out_flops  host the MFMA flops of the launch
   Needs no workspace; opts supplies the stream. */
#define ILRE_PROBE_OPERAND_BYTES 65536
#define ILRE_PROBE_OUT_BYTES ((1u << 20) + 4096)
int ilre_probe_mfma_ceiling(int32_t variant, int32_t iters, const void *operands, void *out, double *out_flops,
                            const ilre_opts *opts);
const char *ilre_probe_describe(int32_t variant);

/* Message for the last non-OK status returned to the calling thread (static storage, never NULL). */
const char *ilre_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ILRE_H */
