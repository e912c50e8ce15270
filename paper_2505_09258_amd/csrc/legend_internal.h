// Internal declarations shared by the host runtime and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "legend.h"

namespace legend {

// Coalescing of gradient rows: table rows with more than kLongLen gradient rows are summed in units of
// kUnit rows (two levels, fixed order); batches of at most kSmallSortMax gradient rows are sorted, cut
// into segments and planned by one workgroup.
constexpr int kLongLen = 32;
constexpr int kUnit = 256;      // 8 groups x 32 rows
constexpr int kSmallSortMax = 4096;

// ---- kernel classes for per-kernel event timing --------------------------------------------
enum KernelClass : int {
    KC_PREPARE = 0,   // negative ids + sort keys of a batch
    KC_SORT,          // radix sort passes (histogram, scan, scatter) + segment heads
    KC_CHUNK,         // fused gather + scores + loss + backward per chunk (MFMA)
    KC_UPDATE,        // segmented gradient reduce + Adagrad (table rows with few gradient rows)
    KC_CHUNK_REDO,    // two-sweep kernel over the chunks the single-sweep kernel handed back
    KC_MISC,          // loss reduction, validation, scoring
    KC_UPDATE_LONG,   // the same for table rows with many gradient rows (two-level sums), on a stream of its own
    KC_COUNT
};

// ---- geometry of one batch --------------------------------------------------------------------
// Occurrence list: every gradient row a batch produces has a fixed position.
//   per side slot (dst side first, then src side):
//     [0, P)            gradient rows of the source embeddings of the P positives
//     [P, 2P)           gradient rows of the destination embeddings
//     [2P, 3P)          gradient rows of the relation embeddings (only if the score uses them)
//     then, chunk-major: for chunk c, row tile t, negative k:  ((c * T + t) * N + k)
struct BatchGeom {
    int32_t P;            // positives in this batch
    int32_t C;            // chunk size
    int32_t N;            // negatives per chunk and side
    int32_t T;            // row tiles per chunk (workgroups per chunk and side)
    int32_t rows_tile;    // positives handled by one workgroup (<= 64)
    int32_t nchunks;
    int32_t sides;        // 1 or 2
    int32_t side_id[2];   // 0 = dst corrupted, 1 = src corrupted
    int32_t roles;        // 2 or 3 (with relation rows)
    int64_t per_side;     // occurrences per side
    int64_t n_occ;        // total occurrences
};

// Everything the per-batch kernels need to know about the bucket and the model.
struct BucketParams {
    const int32_t* edges;      // device, [m][3]
    int64_t m;                 // edges in the bucket
    int64_t batch_lo;          // first edge of the batch
    float* E_src; float* S_src;   // slot of partition i
    float* E_dst; float* S_dst;   // slot of partition j
    float* E_rel; float* S_rel;   // relation table
    float* G_src; float* G_dst; float* G_rel;   // atomic mode: dense gradient accumulators (zero between batches)
    int32_t atomic_mode;
    int32_t rows_valid_src;    // valid rows of partition i
    int32_t rows_valid_dst;
    int32_t num_relations;
    int32_t dim;
    int32_t score, loss;       // loss: LEGEND_LOSS_SOFTMAX, _LOGISTIC or _MARGIN (kernel template parameter)
    int32_t softmax_with_pos;  // Eq. 1 variant: the positive score is a term of the log-sum-exp
    int32_t same_part;         // i == j
    uint32_t key_base_dst;     // key offset of table slot 1 (0 when same_part)
    uint32_t key_base_rel;     // key offset of the relation table
    int32_t num_degree_negs;
    float lr, eps, neg_weight;
    float margin;              // margin loss: a negative should score this much below its positive
    uint64_t hash_prefix;      // hash state after (seed, epoch, i, j, b)
};

// Per-batch device workspace.
struct Workspace {
    int32_t*  neg_ids;        // [sides][nchunks][N]
    uint32_t* keys[2];        // sort double buffer
    uint32_t* vals[2];
    uint32_t* ghist;          // [256][nblocks] radix histogram
    uint32_t* scan_tmp;       // block sums of the generic scan
    uint32_t* uniq_keys;      // [n_occ]
    uint32_t* seg_start;      // [n_occ + 1]
    uint32_t* counters;       // [8]: [0] unique rows of the batch, [1] error flag, [2] long rows, [3] units of long rows
    uint32_t* long_list;      // unique-row indices of rows with many gradient rows
    uint32_t* unit_start;     // first unit of each long row (+ total)
    double*   long_partial;   // [units][dim] fp64 partial sums
    unsigned long long* uniq_total;  // running sum of unique rows
    float*    grad;           // [n_occ][dim] staged gradient rows
    double*   loss_partial;   // one per chunk workgroup
    uint32_t* redo;           // per chunk workgroup: 1 = the single-sweep kernel left it to the general kernel
    unsigned long long* redo_total;  // running count of such workgroups
    // dim > 128 only: operands and intermediate results of the chain of contractions
    float*    gemm_Q;         // [sides][P][dim] composed rows
    float*    gemm_f;         // [sides][P] positive scores
    float*    gemm_S;         // [row tiles][rows_tile][N rounded up to 64] negative scores, then the weights dL/dS
    float*    gemm_a;         // [sides][P] dL/df
    float*    gemm_G;         // [sides][P][dim] G_Q
    int32_t   no_fast_path;   // LEGEND_NO_FAST_CHUNK=1: always use the general two-sweep kernel
    int32_t   fast_no_rescale;  // LEGEND_FAST_CHUNK_NO_RESCALE=1: a chunk that would raise its softmax reference goes to the two-sweep kernel instead
    float     fast_limit;     // how far above its row's current reference a score may lie before the single-sweep kernel raises the reference (LEGEND_FAST_CHUNK_LIMIT, default 110)
    double*   loss_sum;       // running bucket loss
    int64_t   cap_occ;
    int64_t   cap_wg;
};

// A kernel attribute (hipFuncSetAttribute) belongs to the device that is current when it is set:
// "already set" is remembered per device, not per process.
struct PerDeviceFlag {
    bool done[64] = {};
    int dev = 0;
    bool pending() {
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { dev = -1; return true; }
        return !done[dev];
    }
    void set() { if (dev >= 0) done[dev] = true; }
};

// ---- launch wrappers (defined in the kernel translation units) --------------------------------
hipError_t launch_validate_edges(hipStream_t st, const int32_t* edges, int64_t m, int32_t rows_src,
                                 int32_t rows_dst, int32_t num_rel, int check_rel, uint32_t* err_flag);
// seeded fill of `rows` table rows starting at global row `row0` (table_tag: kInitTagNode / kInitTagRel)
constexpr uint64_t kInitTagNode = 0x6E6F6465ull, kInitTagRel = 0x72656C73ull;
hipError_t launch_init_fill(hipStream_t st, float* out, int64_t rows, int32_t dim, int64_t row0, uint64_t seed,
                            uint64_t table_tag, float init_std);
hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t n);
// index side of a batch: keys and negative ids (launch_prepare), then the stable sort, the segment heads
// and, with plan_long, the rows with many gradient rows and their units; the sorted occurrence
// indices end up in ws.vals[*out_buf].  Batches of at most kSmallSortMax gradient rows do all of it in
// the one launch of launch_sort_and_segments.
hipError_t launch_prepare(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_sort_and_segments(hipStream_t st, const BatchGeom& g, const BucketParams& bp, int key_bits,
                                    const Workspace& ws, int* out_buf, bool plan_long);
// long rows and their units from the segment bounds; nothing to do for n_occ <= kSmallSortMax
hipError_t launch_long_plan(hipStream_t st, int64_t n_occ, const Workspace& ws);
// redo = false: the batch computation; redo = true: second launch over the workgroups the single-sweep kernel flagged
bool chunks_use_single_sweep(const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_chunks(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws, bool redo);
hipError_t launch_update(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                         const uint32_t* sorted_vals, bool long_rows);
// batches of at most kSmallSortMax gradient rows: loss sum, short and long rows in one launch
bool update_is_small(const BatchGeom& g);
hipError_t launch_update_small(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                               const uint32_t* sorted_vals, int64_t loss_n);
hipError_t launch_update_atomic(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_loss_reduce(hipStream_t st, int64_t nwg, const Workspace& ws);
hipError_t launch_score(hipStream_t st, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m,
                        float* const* part_emb, int32_t rows_per_partition, int32_t num_partitions,
                        int64_t num_nodes, const float* E_rel, int32_t num_relations, int32_t dim,
                        int32_t score, float* out, uint32_t* err_flag);
// ranks of m triples against a candidate set: q rows, own scores, greater/equal counts, MRR and Hits@k
int64_t rank_rows_padded(int64_t m);
int rank_dim_padded(int d);
hipError_t launch_rank(hipStream_t st, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m,
                       int32_t side, const int64_t* cand, int64_t n_cand, float* const* part_emb,
                       int32_t rows_per_partition, int64_t num_nodes, const float* E_rel, int32_t num_relations,
                       int32_t dim, int32_t score, float* Q, float* f, int32_t* true_id, int32_t* greater,
                       int32_t* equal, double* metrics, uint32_t* err_flag);
hipError_t launch_gather_rows(hipStream_t st, const int64_t* ids, int64_t m, float* const* part_base,
                              int32_t rows_per_partition, int64_t num_rows, int32_t dim, float* out,
                              uint32_t* err_flag);

int64_t update_long_rows_capacity(int64_t n_occ);
int64_t update_long_units_capacity(int64_t n_occ);
int row_tiles_for(int chunk_size, int dim);          // T
int64_t gemm_npad(int N);                            // negatives per row of the score buffer (dim > 128)
int rows_per_tile_for(int chunk_size, int dim);      // ceil(C / T)
int max_dim_supported();
bool dim_supported(int dim);

}  // namespace legend
