// C ABI of libilre: argument validation, workspace carving and kernel launches on the caller's
// stream.  Host code only; the kernels live in scoring.hip and select.hip.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "ilre_internal.h"

// Scratch of ilre_row_stats_static: the per-split partial row statistics live here
// instead of in a caller's workspace.  One copy per GPU the library runs on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; the device address it yields is what
// the kernels are given.
static __device__ __align__(256) unsigned char scratch[ILRE_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

int fail(int status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return status;
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
    size_t part_m, part_z, flag, row_max, row_sumexp, row_off, wg_time, split_table, partial, select, total;
    ilre::SelectLayout sel;
};

ilre::SelectJob window_job(int64_t L, int sink, int budget, const int32_t *pool_kernels, int n_kernels)
{
    ilre::SelectJob job{};
    job.mode = ilre::kSelWindowMax;
    job.L = L - sink;
    job.sink = sink;
    job.budget = budget;
    job.n_max = n_kernels;
    job.n_avg = 1;
    job.max_kernels = pool_kernels;
    return job;
}

ilre::SelectJob max_avg_job(int64_t L, int sink, int budget, const int32_t *max_kernels, int n_max,
                            const int32_t *avg_kernels, int n_avg)
{
    ilre::SelectJob job{};
    job.mode = ilre::kSelMaxAvg;
    job.L = L - sink;
    job.sink = sink;
    job.budget = budget;
    job.n_max = n_max;
    job.n_avg = n_avg;
    job.max_kernels = max_kernels;
    job.avg_kernels = avg_kernels;
    return job;
}

Layout make_layout(const ilre::ScorePlan &p, int64_t L, int64_t nrows, const ilre::SelectJob &job)
{
    Layout l{};
    size_t off = 0;
    l.part_m = off;
    off = up256(off + (size_t)p.nsplit * nrows * sizeof(float));
    l.part_z = off;
    off = up256(off + (size_t)p.nsplit * nrows * sizeof(float));
    l.flag = off;
    off = up256(off + sizeof(uint32_t));
    l.row_max = off;
    off = up256(off + (size_t)nrows * sizeof(float));
    l.row_sumexp = off;
    off = up256(off + (size_t)nrows * sizeof(float));
    l.row_off = off;
    off = up256(off + (size_t)p.nunits * p.rows_per_wg * sizeof(float));
    l.wg_time = off;
    off = up256(off + (size_t)p.grid * sizeof(uint32_t));
    l.split_table = off;
    off = up256(off + ((size_t)p.nsplit + 3) * sizeof(int32_t));
    l.partial = off;
    off = up256(off + (size_t)p.nunits * (size_t)L * sizeof(float));
    l.select = off;
    l.sel = ilre::make_select_layout(job);
    off += l.sel.total;
    l.total = off;
    return l;
}

int check_shape(int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d, int32_t dtype)
{
    if (L < 1 || Lq < 1 || Hq < 1 || Hkv < 1) return fail(ILRE_EINVAL, "L, Lq, Hq, Hkv must be positive");
    if (Hq % Hkv != 0) return fail(ILRE_EINVAL, "Hq (%d) must be a multiple of Hkv (%d)", Hq, Hkv);
    if (L > 0x7FFFFFFFll) return fail(ILRE_EUNSUPPORTED, "L must fit an int32 index");
    if (d != ILRE_HEAD_DIM) return fail(ILRE_EUNSUPPORTED, "head_dim %d unsupported (only %d)", d, ILRE_HEAD_DIM);
    if (dtype != ILRE_F32 && dtype != ILRE_BF16) return fail(ILRE_EUNSUPPORTED, "unknown dtype %d", dtype);
    if ((int64_t)Hq * Lq > 0x3FFFFFFF) return fail(ILRE_EUNSUPPORTED, "too many query rows");
    return ILRE_OK;
}

int check_kernels(int64_t L, int32_t budget, const int32_t *pool_kernels, int32_t n)
{
    if (!pool_kernels) return fail(ILRE_EINVAL, "pool_kernels is null");
    if (n < 1) return fail(ILRE_EINVAL, "n_pool_kernels must be positive");
    if (n > ILRE_MAX_POOL_KERNELS) return fail(ILRE_EUNSUPPORTED, "more than %d pooling kernels", ILRE_MAX_POOL_KERNELS);
    if (budget < 1) return fail(ILRE_EINVAL, "budget must be positive");
    for (int j = 0; j < n; ++j) {
        if (pool_kernels[j] < 1 || pool_kernels[j] % 2 == 0)
            return fail(ILRE_EINVAL, "pooling kernel size %d must be odd and >= 1", pool_kernels[j]);
        if (pool_kernels[j] > ILRE_MAX_POOL_KERNEL)
            return fail(ILRE_EUNSUPPORTED, "pooling kernel size %d over the limit %d", pool_kernels[j], ILRE_MAX_POOL_KERNEL);
    }
    const int64_t n_out = budget < L ? budget : L;
    if (n_out > ILRE_MAX_BUDGET)
        return fail(ILRE_EUNSUPPORTED, "min(budget, L) = %lld over the limit %d", (long long)n_out, ILRE_MAX_BUDGET);
    return ILRE_OK;
}

// Kernel sizes of the printed form of Algorithm 1 (the arrays may be null only when the sizes
// themselves are not needed: n_avg sizes never are for workspace sizing).
int check_max_avg(int64_t L, int32_t sink, int32_t budget, const int32_t *max_kernels, int32_t n_max,
                  const int32_t *avg_kernels, int32_t n_avg, bool sizing)
{
    if (L < 1 || L > 0x7FFFFFFFll) return fail(ILRE_EINVAL, "L must be in [1, 2^31)");
    if (sink < 0 || sink > L) return fail(ILRE_EINVAL, "sink must be in [0, L]");
    if (!max_kernels || (!sizing && !avg_kernels)) return fail(ILRE_EINVAL, "max_kernels or avg_kernels is null");
    if (n_max < 1 || n_avg < 1) return fail(ILRE_EINVAL, "n_max and n_avg must be positive");
    if ((int64_t)n_max * n_avg > ILRE_MAX_POOL_KERNELS)
        return fail(ILRE_EUNSUPPORTED, "more than %d pooling combinations", ILRE_MAX_POOL_KERNELS);
    for (int i = 0; i < n_max; ++i) {
        if (max_kernels[i] < 1) return fail(ILRE_EINVAL, "max-pooling kernel size %d must be >= 1", max_kernels[i]);
        if (max_kernels[i] > ILRE_MAX_MAX_KERNEL)
            return fail(ILRE_EUNSUPPORTED, "max-pooling kernel size %d over the limit %d", max_kernels[i], ILRE_MAX_MAX_KERNEL);
    }
    if (sizing) return ILRE_OK;
    for (int i = 0; i < n_avg; ++i) {
        if (avg_kernels[i] < 1) return fail(ILRE_EINVAL, "average-pooling kernel size %d must be >= 1", avg_kernels[i]);
        if (avg_kernels[i] > ILRE_MAX_AVG_KERNEL)
            return fail(ILRE_EUNSUPPORTED, "average-pooling kernel size %d over the limit %d", avg_kernels[i], ILRE_MAX_AVG_KERNEL);
    }
    if (budget < 1) return fail(ILRE_EINVAL, "budget must be positive");
    const int64_t n_out = budget < L - sink ? budget : L - sink;
    if (n_out > ILRE_MAX_BUDGET)
        return fail(ILRE_EUNSUPPORTED, "min(budget, L - sink) = %lld over the limit %d", (long long)n_out, ILRE_MAX_BUDGET);
    return ILRE_OK;
}

int check_opts(const ilre_opts *o)
{
    if (!o) return fail(ILRE_EINVAL, "opts is null");
    if (o->struct_size != (int32_t)sizeof(ilre_opts))
        return fail(ILRE_EINVAL, "opts->struct_size %d != %zu", o->struct_size, sizeof(ilre_opts));
    if (o->score_mode != ILRE_SCORE_SUM && o->score_mode != ILRE_SCORE_MAX)
        return fail(ILRE_EUNSUPPORTED, "unknown score_mode %d", o->score_mode);
    if (!(o->scale >= 0.f) || isinf(o->scale)) return fail(ILRE_EINVAL, "scale must be finite and >= 0 (0 = 1/sqrt(d))");
    if (o->flags & ~ILRE_FLAG_EXACT_ROW_MAX) return fail(ILRE_EUNSUPPORTED, "unknown flag bits 0x%x", o->flags);
    if (o->sink < 0) return fail(ILRE_EINVAL, "sink must be non-negative");
    if (o->reserved != 0) return fail(ILRE_EINVAL, "opts->reserved must be 0");
    return ILRE_OK;
}

int check_workspace(const ilre_opts *o, size_t need)
{
    if (!o->workspace) return fail(ILRE_ENOMEM, "workspace is null (%zu bytes needed)", need);
    if (((uintptr_t)o->workspace & 255) != 0) return fail(ILRE_EINVAL, "workspace must be 256-byte aligned");
    if (o->workspace_bytes < need)
        return fail(ILRE_ENOMEM, "workspace has %zu bytes, %zu needed", o->workspace_bytes, need);
    return ILRE_OK;
}

// Fills the part of ScoreArgs that describes Q and K; validates strides and alignment (the kernels
// read 16-byte chunks).
int fill_qk(ilre::ScoreArgs &a, const void *q, const void *k, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
            const ilre_opts *o)
{
    if (!q || !k) return fail(ILRE_EINVAL, "q or k_cache is null");
    const int es = o->dtype == ILRE_BF16 ? 2 : 4;
    a.q = q;
    a.k = k;
    a.L = L;
    a.Lq = Lq;
    a.Hq = Hq;
    a.Hkv = Hkv;
    a.G = Hq / Hkv;
    a.q_stride_token = o->q_stride_token ? o->q_stride_token : d;
    a.q_stride_head = o->q_stride_head ? o->q_stride_head : (int64_t)Lq * d;
    a.k_stride_token = o->k_stride_token ? o->k_stride_token : d;
    a.k_stride_head = o->k_stride_head ? o->k_stride_head : L * (int64_t)d;
    const int64_t strides[4] = {a.q_stride_token, a.q_stride_head, a.k_stride_token, a.k_stride_head};
    for (int64_t s : strides) {
        if (s < d)
            return fail(ILRE_EINVAL, "strides must be >= d (rows may not overlap)");
        if ((s * es) % 16 != 0) return fail(ILRE_EINVAL, "strides must be multiples of 16 bytes");
    }
    if (((uintptr_t)q & 15) || ((uintptr_t)k & 15)) return fail(ILRE_EINVAL, "q and k_cache must be 16-byte aligned");
    const float scale = o->scale > 0.f ? o->scale : 1.0f / sqrtf((float)d);
    a.c = scale * 1.4426950408889634f;
    a.force_online = (o->flags & ILRE_FLAG_EXACT_ROW_MAX) ? 1 : 0;
    return ILRE_OK;
}

// The key stream addresses a tile's rows with 32-bit byte offsets from the tile's first token.
int check_tile_span(const ilre::ScoreArgs &a, const ilre::ScorePlan &p, int dtype)
{
    const int64_t es = dtype == ILRE_BF16 ? 2 : 4;
    const int64_t span = a.k_stride_token * es * (int64_t)(p.tile_tokens - 1) + (int64_t)ILRE_HEAD_DIM * es;
    if (span > 0x7FFFFFFFll)
        return fail(ILRE_EUNSUPPORTED, "k_stride_token %lld too large: a tile of %d tokens would span %lld bytes (limit 2^31 - 1)",
                    (long long)a.k_stride_token, p.tile_tokens, (long long)span);
    return ILRE_OK;
}

void fill_plan(ilre::ScoreArgs &a, const ilre::ScorePlan &p)
{
    a.rows_per_group = p.rows_per_group;
    a.nqb = p.nqb;
    a.nsplit = p.nsplit;
    a.ntiles = p.ntiles;
    a.tiles_per_split = p.tiles_per_split;
    a.table_tag = p.table_tag;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(ILRE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Device address of the static scratch array on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(ILRE_EUNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return fail(ILRE_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return ILRE_OK;
}

// Eq. 4 row statistics with the partial results in `scratch_base` (scratch_bytes long; a caller's workspace or
// the static array).  static_buf only words the error message.
int row_stats_into(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                   float *row_max, float *row_sumexp, const ilre_opts *opts, bool static_buf)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if ((rc = check_shape(L, Lq, Hq, Hkv, d, opts->dtype))) return rc;
    if (!row_max || !row_sumexp) return fail(ILRE_EINVAL, "row_max or row_sumexp is null");
    const ilre::ScorePlan p = ilre::make_score_plan(opts->dtype, L, Lq, Hq, Hkv);
    const int64_t nrows = (int64_t)Hq * Lq;
    const Layout lay = make_layout(p, L, nrows, window_job(L, 0, 1, nullptr, 0));
    unsigned char *ws;
    if (static_buf) {
        if (lay.row_max > (size_t)ILRE_STATIC_SCRATCH_BYTES)
            return fail(ILRE_EUNSUPPORTED, "this shape needs %zu bytes of scratch, the static buffer holds %zu; use ilre_row_stats",
                        lay.row_max, (size_t)ILRE_STATIC_SCRATCH_BYTES);
        void *ptr = nullptr;
        if ((rc = static_scratch(&ptr))) return rc;
        ws = (unsigned char *)ptr;
    } else {
        if ((rc = check_workspace(opts, lay.row_max))) return rc;
        ws = (unsigned char *)opts->workspace;
    }
    ilre::ScoreArgs a{};
    if ((rc = fill_qk(a, q, k_cache, L, Lq, Hq, Hkv, d, opts))) return rc;
    if ((rc = check_tile_span(a, p, opts->dtype))) return rc;
    fill_plan(a, p);
    a.part_m = (float *)(ws + lay.part_m);
    a.part_z = (float *)(ws + lay.part_z);
    // a workspace that also serves ilre_col_scores is told how fast each XCD was (that call sizes its token
    // ranges by it); one that only holds this call's scratch is not
    if (!static_buf && p.balanced && opts->workspace_bytes >= lay.partial) {
        a.wg_time = (uint32_t *)(ws + lay.wg_time);
        a.split_table = (int32_t *)(ws + lay.split_table);
    }
    const hipError_t e = ilre::launch_row_stats(p, a, row_max, row_sumexp, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "row-statistics launch");
    return ILRE_OK;
}

}  // namespace

extern "C" {

const char *ilre_last_error(void) { return g_err; }

int ilre_workspace_bytes(int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_pool_kernels,
                         int32_t dtype, size_t *out_bytes)
{
    if (!out_bytes) return fail(ILRE_EINVAL, "out_bytes is null");
    int rc = check_shape(L, Lq, Hq, Hkv, d, dtype);
    if (rc) return rc;
    if (n_pool_kernels < 0 || n_pool_kernels > ILRE_MAX_POOL_KERNELS)
        return fail(ILRE_EINVAL, "n_pool_kernels out of range");
    const ilre::ScorePlan p = ilre::make_score_plan(dtype, L, Lq, Hq, Hkv);
    *out_bytes = make_layout(p, L, (int64_t)Hq * Lq, window_job(L, 0, 1, nullptr, n_pool_kernels)).total;
    return ILRE_OK;
}

int ilre_workspace_bytes_max_avg(int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d, int32_t sink,
                                 const int32_t *max_kernels, int32_t n_max, int32_t n_avg, int32_t dtype,
                                 size_t *out_bytes)
{
    if (!out_bytes) return fail(ILRE_EINVAL, "out_bytes is null");
    int rc = check_shape(L, Lq, Hq, Hkv, d, dtype);
    if (rc) return rc;
    if ((rc = check_max_avg(L, sink, 1, max_kernels, n_max, nullptr, n_avg, true))) return rc;
    const ilre::ScorePlan p = ilre::make_score_plan(dtype, L, Lq, Hq, Hkv);
    *out_bytes = make_layout(p, L, (int64_t)Hq * Lq, max_avg_job(L, sink, 1, max_kernels, n_max, nullptr, n_avg)).total;
    return ILRE_OK;
}

int ilre_row_stats(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                   float *row_max, float *row_sumexp, const ilre_opts *opts)
{
    return row_stats_into(q, k_cache, L, Lq, Hq, Hkv, d, row_max, row_sumexp, opts, false);
}

int ilre_row_stats_static(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                          float *row_max, float *row_sumexp, const ilre_opts *opts)
{
    return row_stats_into(q, k_cache, L, Lq, Hq, Hkv, d, row_max, row_sumexp, opts, true);
}

int ilre_col_scores(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                    const float *row_max, const float *row_sumexp, float *out_scores, const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if ((rc = check_shape(L, Lq, Hq, Hkv, d, opts->dtype))) return rc;
    if (!row_max || !row_sumexp || !out_scores) return fail(ILRE_EINVAL, "row_max, row_sumexp or out_scores is null");
    const ilre::ScorePlan p = ilre::make_score_plan(opts->dtype, L, Lq, Hq, Hkv);
    const int64_t nrows = (int64_t)Hq * Lq;
    const Layout lay = make_layout(p, L, nrows, window_job(L, 0, 1, nullptr, 0));
    if ((rc = check_workspace(opts, lay.select))) return rc;
    ilre::ScoreArgs a{};
    if ((rc = fill_qk(a, q, k_cache, L, Lq, Hq, Hkv, d, opts))) return rc;
    if ((rc = check_tile_span(a, p, opts->dtype))) return rc;
    fill_plan(a, p);
    unsigned char *ws = (unsigned char *)opts->workspace;
    a.row_max = row_max;
    a.row_sumexp = row_sumexp;
    a.row_off = (float *)(ws + lay.row_off);
    if (p.balanced) a.split_table = (int32_t *)(ws + lay.split_table);  // taken only if an ilre_row_stats of this shape left it there
    a.partial = (float *)(ws + lay.partial);
    a.dump = (float *)(ws + lay.flag) + 16;
    const hipError_t e = ilre::launch_col_scores(p, a, opts->score_mode, out_scores, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "column-score launch");
    return ILRE_OK;
}

int ilre_select(const float *scores, int64_t L, int32_t budget, const int32_t *pool_kernels, int32_t *out_idx,
                const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if (L < 1 || L > 0x7FFFFFFFll) return fail(ILRE_EINVAL, "L must be in [1, 2^31)");
    if (!scores || !out_idx) return fail(ILRE_EINVAL, "scores or out_idx is null");
    if ((uintptr_t)scores & 15) return fail(ILRE_EINVAL, "scores must be 16-byte aligned");
    if (opts->sink > L) return fail(ILRE_EINVAL, "sink must be in [0, L]");
    if ((rc = check_kernels(L - opts->sink, budget, pool_kernels, opts->n_pool_kernels))) return rc;
    // The selection region sits at the end of the workspace whatever the scoring shape was; used
    // alone it starts at the workspace base.  Sized for the whole context, so that one workspace serves
    // every sink size.
    const ilre::SelectLayout sized = ilre::make_select_layout(window_job(L, 0, budget, pool_kernels, opts->n_pool_kernels));
    if ((rc = check_workspace(opts, sized.total))) return rc;
    const ilre::SelectJob job = window_job(L, opts->sink, budget, pool_kernels, opts->n_pool_kernels);
    const ilre::SelectLayout sel = ilre::make_select_layout(job);
    const hipError_t e = ilre::launch_select(scores + opts->sink, job, out_idx, nullptr, opts->workspace, sel, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "selection launch");
    return ILRE_OK;
}

int ilre_select_max_avg(const float *scores, int64_t L, int32_t sink, int32_t budget, const int32_t *max_kernels,
                        int32_t n_max, const int32_t *avg_kernels, int32_t n_avg, int32_t *out_idx, int32_t *out_count,
                        const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if (!scores || !out_idx) return fail(ILRE_EINVAL, "scores or out_idx is null");
    if ((uintptr_t)scores & 3) return fail(ILRE_EINVAL, "scores must be 4-byte aligned");
    if ((rc = check_max_avg(L, sink, budget, max_kernels, n_max, avg_kernels, n_avg, false))) return rc;
    const ilre::SelectJob job = max_avg_job(L, sink, budget, max_kernels, n_max, avg_kernels, n_avg);
    const ilre::SelectLayout sel = ilre::make_select_layout(job);
    if ((rc = check_workspace(opts, sel.total))) return rc;
    const hipError_t e = ilre::launch_select(scores + sink, job, out_idx, out_count, opts->workspace, sel, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "selection launch");
    return ILRE_OK;
}

namespace {

// Eq. 4 and Eq. 5 (the part the two forms of the whole path share).  The scores are left as per-unit partial
// vectors, described by `fused`, for the selection to reduce into out_scores on its way.
int run_scoring(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                float *out_scores, const ilre_opts *opts, const ilre::ScorePlan &p, const Layout &lay, ilre::FusedScores &fused)
{
    int rc;
    ilre::ScoreArgs a{};
    if ((rc = fill_qk(a, q, k_cache, L, Lq, Hq, Hkv, d, opts))) return rc;
    if ((rc = check_tile_span(a, p, opts->dtype))) return rc;
    fill_plan(a, p);
    unsigned char *ws = (unsigned char *)opts->workspace;
    hipStream_t s = (hipStream_t)opts->stream;
    a.part_m = (float *)(ws + lay.part_m);
    a.part_z = (float *)(ws + lay.part_z);
    float *row_max = (float *)(ws + lay.row_max);
    float *row_sumexp = (float *)(ws + lay.row_sumexp);
    a.row_off = (float *)(ws + lay.row_off);
    if (p.balanced) {
        a.wg_time = (uint32_t *)(ws + lay.wg_time);
        a.split_table = (int32_t *)(ws + lay.split_table);
    }
    hipError_t e = ilre::launch_row_stats(p, a, row_max, row_sumexp, s, true);
    if (e != hipSuccess) return hip_fail(e, "row-statistics launch");
    a.row_max = row_max;
    a.row_sumexp = row_sumexp;
    a.partial = (float *)(ws + lay.partial);
    a.dump = (float *)(ws + lay.flag) + 16;
    e = ilre::launch_col_scores(p, a, opts->score_mode, out_scores, s, false, true);
    if (e != hipSuccess) return hip_fail(e, "column-score launch");
    fused = ilre::FusedScores{a.partial, p.nunits, opts->score_mode == ILRE_SCORE_MAX ? 1 : 0, out_scores, L};
    return ILRE_OK;
}

}  // namespace

int ilre_gather_ids(const int32_t *input_ids, int64_t L, const int32_t *idx, int32_t n, int32_t *out, const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if (L < 1 || L > 0x7FFFFFFFll) return fail(ILRE_EINVAL, "L must be in [1, 2^31)");
    if (n < 0) return fail(ILRE_EINVAL, "n must be non-negative");
    if (!input_ids || !idx || !out) return fail(ILRE_EINVAL, "input_ids, idx or out is null");
    if (n == 0) return ILRE_OK;
    const hipError_t e = ilre::launch_gather_ids(input_ids, L, idx, n, out, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "ID gather launch");
    return ILRE_OK;
}

int ilre_rerope_keys(const void *k_in, void *k_out, int64_t L, int32_t Hkv, int32_t d, int32_t chunk_tokens,
                     int32_t first_extra, double rope_base, const double *inv_freq, int32_t pairing, const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if ((rc = check_shape(L, 1, Hkv, Hkv, d, opts->dtype))) return rc;
    if (!k_in || !k_out) return fail(ILRE_EINVAL, "k_in or k_out is null");
    if (Hkv > 65535) return fail(ILRE_EUNSUPPORTED, "more than 65535 kv heads");
    if (chunk_tokens < 1 || first_extra < 0) return fail(ILRE_EINVAL, "chunk_tokens must be positive, first_extra non-negative");
    if (pairing != ILRE_ROPE_HALF && pairing != ILRE_ROPE_INTERLEAVED) return fail(ILRE_EUNSUPPORTED, "unknown pairing %d", pairing);
    if (!inv_freq && !(rope_base > 0.0 && isfinite(rope_base))) return fail(ILRE_EINVAL, "rope_base must be positive and finite");
    const int es = opts->dtype == ILRE_BF16 ? 2 : 4;
    ilre::RopeArgs a{};
    a.in = (const unsigned char *)k_in;
    a.out = (unsigned char *)k_out;
    a.L = L;
    a.Hkv = Hkv;
    a.stride_token = opts->k_stride_token ? opts->k_stride_token : d;
    a.stride_head = opts->k_stride_head ? opts->k_stride_head : L * (int64_t)d;
    if (a.stride_token < d || a.stride_head < d) return fail(ILRE_EINVAL, "strides must be >= d (rows may not overlap)");
    if ((a.stride_token * es) % 16 != 0 || (a.stride_head * es) % 16 != 0) return fail(ILRE_EINVAL, "strides must be multiples of 16 bytes");
    if (((uintptr_t)k_in & 15) || ((uintptr_t)k_out & 15)) return fail(ILRE_EINVAL, "k_in and k_out must be 16-byte aligned");
    a.chunk = chunk_tokens;
    a.first_extra = first_extra;
    const int64_t body = L - first_extra;
    const int64_t nchunks = body > 0 ? (body + chunk_tokens - 1) / chunk_tokens : 1;
    a.nchunks = (int)nchunks;
    for (int j = 0; j < d / 2; ++j) {
        const double f = inv_freq ? inv_freq[j] : pow(rope_base, -2.0 * j / d);
        if (!isfinite(f)) return fail(ILRE_EINVAL, "inv_freq[%d] is not finite", j);
        a.inv_freq[j] = f;
    }
    const hipError_t e = ilre::launch_rerope(a, opts->dtype, pairing, (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "re-RoPE launch");
    return ILRE_OK;
}

const char *ilre_probe_describe(int32_t variant) { return ilre::probe_describe(variant); }

int ilre_probe_mfma_ceiling(int32_t variant, int32_t iters, const void *operands, void *out, double *out_flops,
                            const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if (variant < 0 || variant >= ilre::probe_variants()) return fail(ILRE_EINVAL, "no probe variant %d", variant);
    if (iters < 1) return fail(ILRE_EINVAL, "iters must be positive");
    if (!operands || !out || !out_flops) return fail(ILRE_EINVAL, "operands, out or out_flops is null");
    if (((uintptr_t)operands & 15) || ((uintptr_t)out & 255)) return fail(ILRE_EINVAL, "operands must be 16-byte, out 256-byte aligned");
    const hipError_t e = ilre::launch_probe(variant, iters, operands, (float *)out,
                                            (unsigned long long *)((unsigned char *)out + (1u << 20)), out_flops,
                                            (hipStream_t)opts->stream);
    if (e != hipSuccess) return hip_fail(e, "probe launch");
    return ILRE_OK;
}

int ilre_recall(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                int32_t budget, const int32_t *pool_kernels, int32_t *out_idx, float *out_scores, const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if ((rc = check_shape(L, Lq, Hq, Hkv, d, opts->dtype))) return rc;
    if (!out_idx || !out_scores) return fail(ILRE_EINVAL, "out_idx or out_scores is null");
    if ((uintptr_t)out_scores & 15) return fail(ILRE_EINVAL, "out_scores must be 16-byte aligned");
    if (opts->sink > L) return fail(ILRE_EINVAL, "sink must be in [0, L]");
    if ((rc = check_kernels(L - opts->sink, budget, pool_kernels, opts->n_pool_kernels))) return rc;
    const ilre::ScorePlan p = ilre::make_score_plan(opts->dtype, L, Lq, Hq, Hkv);
    // workspace sized for the whole context (what ilre_workspace_bytes reports); the selection then runs on the body
    const Layout lay = make_layout(p, L, (int64_t)Hq * Lq, window_job(L, 0, budget, pool_kernels, opts->n_pool_kernels));
    if ((rc = check_workspace(opts, lay.total))) return rc;
    ilre::FusedScores fused{};
    if ((rc = run_scoring(q, k_cache, L, Lq, Hq, Hkv, d, out_scores, opts, p, lay, fused))) return rc;
    unsigned char *ws = (unsigned char *)opts->workspace;
    const ilre::SelectJob job = window_job(L, opts->sink, budget, pool_kernels, opts->n_pool_kernels);
    const hipError_t e = ilre::launch_select(out_scores + opts->sink, job, out_idx, nullptr, ws + lay.select,
                                             ilre::make_select_layout(job), (hipStream_t)opts->stream, &fused);
    if (e != hipSuccess) return hip_fail(e, "selection launch");
    return ILRE_OK;
}

int ilre_recall_max_avg(const void *q, const void *k_cache, int64_t L, int32_t Lq, int32_t Hq, int32_t Hkv, int32_t d,
                        int32_t sink, int32_t budget, const int32_t *max_kernels, int32_t n_max,
                        const int32_t *avg_kernels, int32_t n_avg, int32_t *out_idx, int32_t *out_count,
                        float *out_scores, const ilre_opts *opts)
{
    int rc = check_opts(opts);
    if (rc) return rc;
    if ((rc = check_shape(L, Lq, Hq, Hkv, d, opts->dtype))) return rc;
    if (!out_idx || !out_scores) return fail(ILRE_EINVAL, "out_idx or out_scores is null");
    if ((rc = check_max_avg(L, sink, budget, max_kernels, n_max, avg_kernels, n_avg, false))) return rc;
    const ilre::ScorePlan p = ilre::make_score_plan(opts->dtype, L, Lq, Hq, Hkv);
    const ilre::SelectJob job = max_avg_job(L, sink, budget, max_kernels, n_max, avg_kernels, n_avg);
    const Layout lay = make_layout(p, L, (int64_t)Hq * Lq, job);
    if ((rc = check_workspace(opts, lay.total))) return rc;
    ilre::FusedScores fused{};
    if ((rc = run_scoring(q, k_cache, L, Lq, Hq, Hkv, d, out_scores, opts, p, lay, fused))) return rc;
    unsigned char *ws = (unsigned char *)opts->workspace;
    const hipError_t e = ilre::launch_select(out_scores + sink, job, out_idx, out_count, ws + lay.select, lay.sel,
                                             (hipStream_t)opts->stream, &fused);
    if (e != hipSuccess) return hip_fail(e, "selection launch");
    return ILRE_OK;
}

}  // extern "C"
