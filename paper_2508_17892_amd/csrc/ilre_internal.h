// Internal declarations shared by the translation units of libilre (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ilre.h"

namespace ilre {

constexpr int kHeadDim = ILRE_HEAD_DIM;
constexpr int kNumCU = 256;  // MI355X: 256 compute units in 8 XCDs
constexpr int kNumXCD = 8;

// ---------------------------------------------------------------- scoring (Eq. 4 / Eq. 5)

// How one scoring pass is cut into workgroups.  A workgroup owns (kv head g, query block qb,
// token split s): `waves` wavefronts of 32*nb query rows each, streaming its token tiles.
struct ScorePlan {
    int dtype;            // ilre_dtype
    int waves;            // wavefronts per workgroup (4 or 8)
    int nb;               // 32-row query blocks per wavefront
    int rows_per_group;   // G * Lq query rows served by one kv head
    int rows_per_wg;      // waves * nb * 32
    int nqb;              // query blocks per kv group
    int tile_tokens;      // tokens per LDS tile
    int64_t ntiles;       // ceil(L / tile_tokens)
    int nsplit;           // token splits per (g, qb)
    int64_t tiles_per_split;
    int nunits;           // Hkv * nqb  (partial score vectors of pass 2)
    int grid;             // workgroups launched (a few may be idle padding for the XCD mapping)
    bool balanced;        // pass 2's token ranges are sized by the XCDs' speed in pass 1
    uint64_t table_tag;   // header of a range table made for this plan
    size_t lds_bytes_stats, lds_bytes_cols;
};

struct ScoreArgs {
    const void *q;
    const void *k;
    int64_t L;
    int Lq, Hq, Hkv, G;
    int64_t q_stride_head, q_stride_token, k_stride_head, k_stride_token;  // in elements
    float c;  // scale * log2(e): logits leave the MFMA in raw units and are exponentiated base 2
    int rows_per_group, nqb, nsplit;
    int64_t ntiles, tiles_per_split;
    // pass 1 (row statistics): per-split partial maxima (base-2 units) and sums
    float *part_m, *part_z;  // [nsplit][Hq*Lq]
    int force_online;        // 1: follow the running maximum throughout (the always-safe form)
    uint32_t *wg_time;       // [grid] how long each workgroup of pass 1 ran, 10 ns ticks (null: not recorded)
    int32_t *split_table;    // [2 + nsplit + 1] pass 2's token ranges: written behind pass 1, read by pass 2 (null: even ranges)
    uint64_t table_tag;
    // pass 2 (column scores)
    const float *row_max, *row_sumexp;  // [Hq*Lq]
    float *row_off;                     // [nunits][rows_per_wg]: pass 2's exponent offsets in workgroup order
    float *partial;                     // [nunits][L]
    float *dump;                        // 16 floats nobody reads: target of stores that have nothing to store
};

ScorePlan make_score_plan(int dtype, int64_t L, int Lq, int Hq, int Hkv);

// offsets = true also fills a.row_off, the table of pass 2's per-row exponent offsets, for a launch_col_scores
// with have_offsets = true behind it (otherwise launch_col_scores derives the table from row_max / row_sumexp).
hipError_t launch_row_stats(const ScorePlan &p, const ScoreArgs &a, float *row_max, float *row_sumexp,
                            hipStream_t s, bool offsets = false);
// reduce = false leaves the per-unit partial score vectors in a.partial for launch_reduce_units (or for the
// selection's first pass, which can do the reduction on its way).
hipError_t launch_col_scores(const ScorePlan &p, const ScoreArgs &a, int score_mode, float *out_scores,
                             hipStream_t s, bool reduce = true, bool have_offsets = false);
hipError_t launch_reduce_units(const float *partial, int nunits, int64_t L, int rmax, float *out_scores, hipStream_t s);

// ---------------------------------------------------------------- selection (Algorithm 1)

constexpr int kSelFine = 256;       // elements a wavefront pools at a time ("fine chunk")
constexpr int kSelBins = 2048;      // histogram bins per level: 11 key bits
constexpr int kSelSmall = 2048;     // boundary lists up to this long join the candidates unrefined
constexpr int kCandCap = 10240;     // candidate capacity in tokens (>= ILRE_MAX_BUDGET + kSelSmall)

// Two forms of Algorithm 1 share the selection kernels.  A "combination" j ranks the elements of a
// source array (value descending, element ascending) and offers the tokens of its best elements:
//   kSelWindowMax  stride-1 max pooling: source = the scores, element = token, value = maximum over a
//                  window of radius r_j clipped to the context; candidates are never exhausted.
//   kSelMaxAvg     the algorithm as printed: source = the cells of a strided max pooling (size = stride
//                  = m), value = stride-1 average over n cells (zeros outside), element p stands for
//                  tokens p*m .. p*m+m-1, and only the best K_m = B/m + 1 cells are candidates.
enum SelMode { kSelWindowMax = 0, kSelMaxAvg = 1 };

struct SelectJob {
    int mode;                    // SelMode
    int64_t L;                   // tokens the pooling sees (the context without its sink part)
    int sink;                    // leading tokens that are always allocated (indices are offset by it)
    int budget;
    int n_max, n_avg;            // kSelWindowMax: n_max window sizes, n_avg = 1
    const int32_t *max_kernels;  // host: window sizes w_j, or max-pooling sizes m_i
    const int32_t *avg_kernels;  // host: average-pooling sizes n_j (kSelMaxAvg only)
    int combos() const { return n_max * n_avg; }
};

struct SelectLayout {
    size_t hist;      // uint32 [2][n][kSelBins]  (level 1, level 2), then [2][kSelBins] of the pre-pass
    size_t ctrl;      // SelCtrl [n + 1]  (the last one belongs to the pre-pass)
    size_t done;      // uint32 [2][n], then [2] of the pre-pass: workgroups finished per level and combination
    size_t cmax;      // float [ceil(L / kSelFine)]: fine-chunk maxima (pruning pre-pass)
    size_t active;    // uint32 [ceil(L / kSelFine)]: fine chunks left after pruning
    size_t cells;     // float: the max-pooled cell arrays, one per max kernel (kSelMaxAvg)
    size_t picked;    // uint32 [ILRE_MAX_BUDGET] the allocated tokens in the order they were taken, then their count
    size_t seed;      // kSelWindowMax: uint32 rank[kCandCap], int32 dom_left[kCandCap], int32 dom_right[kCandCap]
    size_t cand;      // uint64 [n][kCandCap]; kSelWindowMax: [1 + n][kCandCap], list 0 the seeds, then a token list per kernel size
    size_t tie;       // uint64: per combination two ping-pong lists of boundary elements, each as long as its source
    size_t total;
};

struct SelCtrl {
    uint32_t want;        // K_j: ranked elements that are candidates
    uint32_t share;       // B_j
    uint32_t before;      // window: elements before and after the centre
    uint32_t after;
    uint32_t bin1;        // level-1 bin (key bits 31..21) holding the K_j-th largest key
    uint32_t above1;      // keys in bins above it
    uint32_t need1;       // still needed from inside it
    uint32_t bin2;        // level-2 bin (key bits 20..10) inside bin1
    uint32_t above2;      // keys of bin1 in level-2 bins above bin2
    uint32_t need2;       // still needed from inside (bin1, bin2)
    uint32_t cand_n;      // filled length of cand[j] after collect
    uint32_t tie_n;       // filled length of the first boundary list
    uint32_t total_n;     // candidates (elements) after refine
    uint32_t len;         // elements in the source array
    uint32_t cell;        // tokens an element stands for (m; 1 in the window-max form)
    uint32_t op;          // SelMode of the value function
    uint64_t src_off;     // source array: floats from the base pointer the pooling kernels are given
    uint64_t tie_off;     // boundary lists: uint64 words from the base of the tie region
    uint32_t exact;       // 1: refine cuts the candidates to exactly `want`
    uint32_t pad[3];
};

// Workspace carving for a job (only mode, L, counts and the max kernels are read).
SelectLayout make_select_layout(const SelectJob &job);

// Scores that still lie as per-unit partial vectors (the whole path): the selection reduces them into
// `scores` (all L positions, sink part included) itself, in its first pass where it can.
struct FusedScores {
    const float *partial;  // [nunits][L]
    int nunits;
    int rmax;              // 0 sum, 1 max over the units
    float *scores;         // L floats
    int64_t L;
};

// `scores` points at the body (the first token after the sink part).
hipError_t launch_select(const float *scores, const SelectJob &job, int32_t *out_idx, int32_t *out_count,
                         void *workspace, const SelectLayout &lay, hipStream_t s, const FusedScores *fused = nullptr);

hipError_t launch_gather_ids(const int32_t *ids, int64_t L, const int32_t *idx, int n, int32_t *out, hipStream_t s);

// ---------------------------------------------------------------- DCA re-RoPE of the key cache

struct RopeArgs {
    const unsigned char *in;
    unsigned char *out;
    int64_t L;
    int Hkv;
    int64_t stride_head, stride_token;  // in elements, the same for in and out
    int chunk, first_extra, nchunks;
    double inv_freq[ILRE_HEAD_DIM / 2];
};

hipError_t launch_rerope(const RopeArgs &a, int dtype, int pairing, hipStream_t s);

// ---------------------------------------------------------------- measurement aid: MFMA ceiling probes

int probe_variants();
const char *probe_describe(int variant);
hipError_t launch_probe(int variant, int iters, const void *operands, float *out, unsigned long long *clocks, double *flops,
                        hipStream_t s);

}  // namespace ilre
