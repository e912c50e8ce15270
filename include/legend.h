/*
 * legend.h - C ABI of the MI355X bucket-training library.
 *
 * One context trains partitioned graph embeddings the way Legend
 * (arXiv 2505.09258) does it: node embeddings and their Adagrad state are
 * split into n equal partitions stored as contiguous [E_p | S_p] blocks
 * (Sec. 3, storage arrangement), a few partitions at a time live in a buffer in
 * GPU memory (Sec. 4: capacity 3), relation embeddings and their state stay on
 * the GPU, and edges are grouped into buckets (i, j) by the partitions of their
 * endpoints (Sec. 2.1).  The host tier that the paper keeps on an NVMe SSD is
 * pinned host memory here; swaps are asynchronous copies on a side stream.
 *
 * Conventions
 *   - Every pointer is a HOST pointer unless the argument is documented as
 *     "host or device" and comes with a legend_mem selector.
 *   - The caller owns all buffers it passes; the library owns the context and
 *     everything it allocates, and frees it in legend_destroy().
 *   - Every function returns LEGEND_OK (0) or a negative legend_status.  The
 *     message of the last failure on the calling thread is available through
 *     legend_last_error().  No exception crosses this boundary.
 *   - A context may be used by one thread at a time.
 *   - After LEGEND_E_HIP the context is unusable except for legend_destroy().
 *     Any other error leaves embeddings and optimiser state unchanged.
 */
#ifndef LEGEND_H
#define LEGEND_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct legend_ctx legend_ctx;

typedef enum legend_status {
    LEGEND_OK = 0,
    LEGEND_E_INVAL = -1,        /* bad argument or unsupported configuration       */
    LEGEND_E_NOMEM = -2,        /* host or device allocation failed                */
    LEGEND_E_NOT_RESIDENT = -3, /* a partition the call needs is not in the buffer */
    LEGEND_E_RANGE = -4,        /* a node or relation id is out of range           */
    LEGEND_E_HIP = -5,          /* a HIP runtime call failed                       */
    LEGEND_E_STATE = -6         /* call not valid in the context's current state   */
} legend_status;

/* Score functions f(theta_s, theta_r, theta_d) = <theta_s (x) theta_r, theta_d>
 * (Sec. 2.1, Sec. 6).  ComplEx rows hold [real half | imaginary half].
 * LEGEND_SCORE_TRANSE_L1 is the translational score -|theta_s + theta_r - theta_d|_1
 * (one of the other models Sec. 8 says fit the same frame): (x) is an addition, its
 * result u = theta_s + theta_r (v = theta_d - theta_r on the source side) is the
 * fp32 sum, and the derivative of |.| at 0 is taken as 0.  dim <= 128. */
enum { LEGEND_SCORE_DOT = 0, LEGEND_SCORE_DISTMULT = 1, LEGEND_SCORE_COMPLEX = 2, LEGEND_SCORE_TRANSE_L1 = 3 };
/* Eq. 1 as printed (log-sum-exp over the sampled negatives only), logistic, the
 * variant of Eq. 1 whose log-sum-exp also holds the positive score (sampled
 * cross-entropy: -f + log(exp f + sum_k exp S_k)), or the margin-based ranking
 * loss sum_k max(0, margin - f + S_k) (Sec. 8: other objectives fit the same
 * frame; every score function, margin >= 0 or LEGEND_E_INVAL). */
enum { LEGEND_LOSS_SOFTMAX = 0, LEGEND_LOSS_LOGISTIC = 1, LEGEND_LOSS_SOFTMAX_POS = 2, LEGEND_LOSS_MARGIN = 3 };
/* Which endpoint of a positive edge is replaced by sampled nodes. */
enum { LEGEND_CORRUPT_DST = 0, LEGEND_CORRUPT_SRC = 1, LEGEND_CORRUPT_BOTH = 2 };
/* Embedding update (Sec. 2.1 stage 6): gradient rows of one table row are summed
 * in a fixed order (sorted by row, then by position in the batch) or with
 * floating-point atomics in whatever order the hardware takes them. */
enum { LEGEND_UPDATE_DETERMINISTIC = 0, LEGEND_UPDATE_ATOMIC = 1 };
enum { LEGEND_MEM_HOST = 0, LEGEND_MEM_DEVICE = 1 };
/* Tables legend_read_embeddings can read. */
enum { LEGEND_TABLE_NODE_EMB = 0, LEGEND_TABLE_NODE_STATE = 1,
       LEGEND_TABLE_REL_EMB = 2, LEGEND_TABLE_REL_STATE = 3 };

typedef struct legend_config {
    uint32_t struct_size;      /* sizeof(legend_config) of the caller               */
    int32_t  device;           /* HIP device ordinal                                */
    int64_t  num_nodes;        /* |V|                                               */
    int32_t  num_relations;    /* |R|; 0 for a graph without relation types         */
    int32_t  dim;              /* d (even for ComplEx)                              */
    int32_t  num_partitions;   /* n; rows per partition R_p = ceil(|V| / n)         */
    int32_t  buffer_capacity;  /* partitions resident at once: 3 (Sec. 4) .. n      */
    int32_t  score;            /* LEGEND_SCORE_*                                    */
    int32_t  loss;             /* LEGEND_LOSS_*                                     */
    int32_t  corrupt;          /* LEGEND_CORRUPT_*                                  */
    int32_t  update_mode;      /* LEGEND_UPDATE_*                                   */
    int32_t  batch_size;       /* B positive edges per batch                        */
    int32_t  chunk_size;       /* C positives sharing one set of negatives          */
    int32_t  num_negs;         /* N negatives per chunk and corrupted side          */
    int32_t  num_degree_negs;  /* the last num_degree_negs of them are endpoints of
                                  uniformly drawn edges of the bucket               */
    float    lr;               /* Adagrad learning rate                             */
    float    eps;              /* Adagrad epsilon (added to sqrt of the state)      */
    float    neg_weight;       /* logistic loss: weight of each negative term;
                                  < 0 selects 1 / num_negs                          */
    float    init_std;         /* standard deviation of the seeded initial embeddings
                                  (used only for a table whose init pointer is NULL) */
    float    margin;           /* LEGEND_LOSS_MARGIN: how far below its positive a
                                  negative must score to cost nothing (>= 0)        */
    uint64_t seed;             /* seed of the negative-sampling counter hash        */
    void*    compute_stream;   /* borrowed hipStream_t, or NULL: library creates    */
    void*    copy_stream;      /* borrowed hipStream_t, or NULL: library creates    */
} legend_config;

/* Optional partition swap to start while a bucket trains (Sec. 3 steps 6-8,
 * Sec. 4): write partition `evict` back to the host tier and bring `load` into
 * the slot it frees.  Either may be -1 (only load into a free slot / only evict). */
typedef struct legend_prefetch {
    int32_t evict;
    int32_t load;
} legend_prefetch;

typedef struct legend_bucket_stats {
    double  loss_sum;   /* sum over the bucket's edges and sides of the loss terms */
    int64_t batches;
    int64_t edges;
    double  ms;         /* device time of the bucket's batches (event-timed)       */
} legend_bucket_stats;

/*
 * Create a context (Sec. 3, storage arrangement).
 *   cfg            configuration; validated, copied.
 *   init_node_emb  [num_nodes][dim] fp32, row-major, global node order.  Node g
 *                  lives in partition g / R_p at local row g % R_p; the last
 *                  partition is zero-padded to R_p rows.  NULL: seeded fill (below).
 *   init_rel_emb   [max(num_relations,1)][dim] fp32, or NULL: seeded fill (zeros for
 *                  LEGEND_SCORE_DOT, which ignores relations).
 *   out            receives the context.
 * Seeded fill ("randomly initialized", Sec. 3 step 1; the paper prints no distribution):
 * element (row g, column k) of a table is an integer function of cfg->seed,
 *     h = fold(fold(fold(seed, tag), g), k),  fold(h, x) = mix64(h + 0x9E3779B97F4A7C15 + x),
 *     mix64 = the splitmix64 output function, tag = 0x6E6F6465 (nodes) / 0x72656C73 (relations),
 *     u = sum of the four 16-bit fields of h,
 *     value = (float)(u - 131070) * (float)((double)init_std * sqrt(3) / 65536)
 * (a sum of four uniform integers: mean 0, standard deviation init_std, the same on every
 * machine).  init_std must be > 0 when a fill is asked for (LEGEND_E_INVAL otherwise).
 * Optimiser state starts at zero.  Allocates n pinned host blocks of
 * 2*R_p*dim floats, buffer_capacity device slots of the same size (one more when
 * buffer_capacity < num_partitions: the slot a partition is loaded into while the
 * one it replaces is still being written back), the relation
 * table and its state on the device, and the per-batch workspace.  No partition
 * is resident after the call.
 */
int legend_init_partitions(const legend_config* cfg, const float* init_node_emb,
                           const float* init_rel_emb, legend_ctx** out);

/* Wait for all work of the context, write resident partitions back to the host
 * tier is NOT done (use legend_swap_partition / legend_read_embeddings first if
 * the values are needed), free everything.  NULL is accepted. */
int legend_destroy(legend_ctx* ctx);

/*
 * Buffer management (Sec. 3 "buffer state", Sec. 4).
 * legend_swap_partition enqueues, on the copy stream, the write-back of
 * partition `evict` (if >= 0) to its host block and the load of partition `load`
 * (if >= 0) into the freed (or a free) slot.  The copies wait for all bucket
 * work enqueued so far; later legend_train_bucket calls that need `load` wait
 * for the copy, calls that need neither run concurrently with it.  Training a
 * bucket that touches `evict` after this call returns LEGEND_E_NOT_RESIDENT.
 * Errors: LEGEND_E_NOT_RESIDENT (evict not resident), LEGEND_E_STATE (no free
 * slot, or load already resident), LEGEND_E_INVAL.
 */
int legend_swap_partition(legend_ctx* ctx, int32_t evict, int32_t load);

/* Buffer slot of a partition, or -1 when it is not resident (in *slot). */
int legend_partition_slot(legend_ctx* ctx, int32_t part, int32_t* slot);

/*
 * Train one edge bucket (Sec. 2.1 stages 1-6; Sec. 3 steps 1-5; Sec. 6).
 *   src_part, dst_part  bucket id (i, j); both partitions must be resident.
 *   edges      [m][3] int32 (src_local, rel, dst_local): rows local to partition
 *              i resp. j, rel in [0, num_relations) (ignored for Dot).  Host or
 *              device memory as said by edges_mem; device memory must stay
 *              valid until the call's work has finished (legend_sync).
 *   m          number of edges, >= 0.
 *   epoch      enters the negative-sampling hash.
 *   hint       optional swap to start once this bucket's work is enqueued if the
 *              bucket does not touch hint->evict, else after the bucket (NULL: none).
 *   stats      optional; when given the call waits for the bucket and fills it.
 * Batches are the consecutive groups of batch_size edges in stored order, the
 * last one partial; chunks likewise inside a batch.  Each batch reads the tables
 * as they are when it starts and updates them before the next one starts.
 * Without `stats` the call returns once the work is enqueued.
 * Errors: LEGEND_E_NOT_RESIDENT, LEGEND_E_RANGE (an id outside its table; nothing
 * is trained), LEGEND_E_INVAL, LEGEND_E_HIP.
 */
int legend_train_bucket(legend_ctx* ctx, int32_t src_part, int32_t dst_part,
                        const int32_t* edges, int64_t m, int32_t edges_mem, int32_t epoch,
                        const legend_prefetch* hint, legend_bucket_stats* stats);

/*
 * The same for batches [batch_begin, batch_end) of the bucket only (batch_end < 0:
 * up to the last batch).  Batch numbers, negatives and chunking are those of the
 * whole bucket, so training a bucket in several consecutive ranges gives exactly
 * the result of one legend_train_bucket call (Sec. 2.1: batches are independent
 * units of the iteration).  stats, when given, covers the range.
 */
int legend_train_bucket_range(legend_ctx* ctx, int32_t src_part, int32_t dst_part,
                              const int32_t* edges, int64_t m, int32_t edges_mem, int32_t epoch,
                              int64_t batch_begin, int64_t batch_end,
                              const legend_prefetch* hint, legend_bucket_stats* stats);

typedef struct legend_epoch_stats {
    double  loss_sum;       /* sum of the loss terms of the epoch                         */
    int64_t edges;
    int64_t batches;
    int64_t swaps;          /* partition loads and write-backs enqueued                   */
    int64_t buffer_states;  /* states of the loading order (1 when everything is resident) */
    int64_t bytes_per_swap; /* size of one [E_p | S_p] block                              */
    double  ms;             /* host wall time from the first call to the final sync       */
} legend_epoch_stats;

/*
 * One epoch over all n*n buckets (Sec. 3 steps 1-8, Sec. 4 Alg. 1 and Alg. 2).
 *   bucket_edges  [n*n] pointers, bucket (i, j) at index i*n + j, each [size][3] int32
 *                 as in legend_train_bucket (all host or all device, edges_mem);
 *   bucket_sizes  [n*n] edge counts (0 allowed, pointer then ignored);
 *   overlap       1: the write-back of the evicted partition is enqueued as soon as the
 *                 buckets of the state that involve it are trained and runs while the
 *                 rest of the state trains (prefetching, Sec. 4); the load of the next
 *                 partition goes into the extra device slot and starts with the state;
 *                 0: swaps run after the state's last bucket has finished (the paper's
 *                 "without prefetching" ablation).
 * With buffer_capacity == num_partitions every partition is made resident and no
 * swap happens during the epoch; otherwise buffer_capacity must be 3 (the paper's
 * setting) and the planner's loading order is followed.  Partitions resident on
 * return are those of the last buffer state; legend_read_embeddings sees all data.
 * The call returns after all work has finished.
 */
int legend_train_epoch(legend_ctx* ctx, const int32_t* const* bucket_edges,
                       const int64_t* bucket_sizes, int32_t edges_mem, int32_t epoch,
                       int32_t overlap, legend_epoch_stats* stats);

/*
 * f(theta_s, theta_r, theta_d) of m triples with the current embeddings
 * (Sec. 2.1).  src/dst are GLOBAL node ids; rel may be NULL for Dot.  Every
 * partition referenced must be resident.  out: [m] fp32 (host).
 */
int legend_score_edges(legend_ctx* ctx, const int64_t* src, const int32_t* rel,
                       const int64_t* dst, int64_t m, float* out);

/*
 * Copy rows of a table to the host after all enqueued work has finished.
 *   table  LEGEND_TABLE_*; ids: global node ids / relation ids, or NULL for rows
 *          0..m-1; out: [m][dim] fp32.
 * Node rows come from the buffer slot when the partition is resident, else from
 * its host block.
 */
int legend_read_embeddings(legend_ctx* ctx, int32_t table, const int64_t* ids, int64_t m,
                           float* out);

/*
 * Index side of one batch, for bit-exact checks (Sec. 2.1 stages 1-2).
 * For batch `batch` of the given bucket, without training anything:
 *   neg_ids   [sides][chunks][num_negs] int32 local row ids (sides in the order
 *             dst, src), capacity neg_capacity entries;
 *   touched   sorted unique keys table * 2^32 + row of the rows the batch would
 *             update (table 0: partition i, 1: partition j when j != i, 2:
 *             relations), capacity touched_capacity entries;
 *   touched_count receives the number of keys.
 * LEGEND_E_INVAL when a capacity is too small.
 */
int legend_debug_batch_indices(legend_ctx* ctx, int32_t src_part, int32_t dst_part,
                               const int32_t* edges, int64_t m, int32_t edges_mem,
                               int32_t epoch, int64_t batch,
                               int32_t* neg_ids, int64_t neg_capacity,
                               int64_t* touched, int64_t touched_capacity,
                               int64_t* touched_count);

/*
 * Partition loading order and bucket iteration order for n partitions and a
 * buffer of three (Sec. 4, Alg. 1 and Alg. 2).  Host-only; no context needed.
 *   states        [*num_states][3] partitions per buffer slot for each state;
 *   buckets       [n*n][2] all buckets in training order;
 *   state_begin   [*num_states + 1] first bucket of each state;
 *   state_overlap [*num_states] index of the first bucket of the state that may
 *                 run while the swap to the next state is in flight.
 * Capacities are in states / buckets; LEGEND_E_INVAL if too small or n < 1.
 */
int legend_plan_order(int32_t n, int32_t* states, int32_t state_capacity, int32_t* num_states,
                      int32_t* buckets, int32_t* state_begin, int32_t* state_overlap);

/* Wait until everything enqueued on the context's streams has finished. */
int legend_sync(legend_ctx* ctx);

/*
 * Per-kernel-class device timing with HIP events on the stream each class runs
 * on (the index side of a batch is built one batch ahead on a stream of its own,
 * the update of rows with many gradient rows next to the main update kernel on
 * another: spans of different classes overlap in time, and a span contains the
 * wait for compute units that other streams hold).
 * legend_profile_enable: mask bit k switches timing of kernel class k on
 * (0 switches all off).  legend_profile_read waits for the work, returns the
 * accumulated milliseconds and launch counts per class since the last read and
 * clears them; names of the classes come from legend_profile_name (NULL past the
 * last class).
 */
int legend_profile_enable(legend_ctx* ctx, uint32_t mask);
int legend_profile_read(legend_ctx* ctx, double* ms, int64_t* launches, int32_t capacity);
const char* legend_profile_name(int32_t kernel_class);

/* Sizes of one batch as the kernels see it (for roofline accounting). */
typedef struct legend_batch_shape {
    int64_t occurrences;   /* gradient rows produced per full batch                */
    int64_t neg_rows;      /* negative rows gathered per full batch                */
    int64_t workspace_bytes;
    int32_t key_bits;
    int32_t row_tiles;     /* workgroups per chunk and side                        */
} legend_batch_shape;
int legend_batch_shape_of(legend_ctx* ctx, legend_batch_shape* out);
/* Unique rows updated by the batches since the last call (sum), then cleared. */
int legend_unique_rows_read(legend_ctx* ctx, int64_t* unique_rows, int64_t* batches);

/* Workgroups (one row tile of one chunk) of the single-sweep batch kernel that met
 * a score too far above their softmax reference (the reference is then raised in
 * place and what was accumulated rescaled, or the chunk handed over to the
 * two-sweep kernel) since the last call, then cleared.  A tuning aid: 0 early in
 * training. */
int legend_fallback_chunks_read(legend_ctx* ctx, int64_t* chunks);

/*
 * Link-prediction ranks of m triples (Sec. 7, "Metrics": MRR and Hits@k are functions
 * of these ranks; the protocol itself is not printed, the textbook one is used).
 * The `side` endpoint of every triple (LEGEND_CORRUPT_DST or LEGEND_CORRUPT_SRC) is
 * replaced by each candidate node in turn and scored with f (Sec. 2.1):
 *   greater[e] = number of candidates other than the true endpoint whose score is
 *                strictly above the triple's own, equal[e] = those that tie with it
 *                (fp32 comparisons of fp32 scores; no filtering of true edges);
 *   rank = 1 + greater + equal / 2, MRR = mean 1/rank, Hits@k = mean [rank <= k].
 *   src/rel/dst   as in legend_score_edges (global ids, host);
 *   candidates    [num_candidates] global node ids (host), shared by all triples, a
 *                 node listed twice counts twice; NULL: every node 0..num_nodes-1
 *                 (num_candidates is then ignored);
 *   greater/equal [m] int32 (host), either may be NULL;
 *   metrics       may be NULL; ms = device time of the kernels.
 * Every partition that a triple or a candidate refers to must be resident
 * (LEGEND_E_NOT_RESIDENT); ids out of range give LEGEND_E_RANGE; num_nodes must be
 * below 2^31.  Embeddings are not modified.  Returns when the results are final.
 */
typedef struct legend_rank_metrics {
    double mrr, hits1, hits3, hits10;
    float ms;
} legend_rank_metrics;
int legend_rank_edges(legend_ctx* ctx, const int64_t* src, const int32_t* rel, const int64_t* dst,
                      int64_t m, int32_t side, const int64_t* candidates, int64_t num_candidates,
                      int32_t* greater, int32_t* equal, legend_rank_metrics* metrics);

/*
 * legend_rank_edges for callers that cannot allocate: code under HIP graph capture, tight
 * evaluation loops inside a serving process, harnesses that forbid hipMalloc.  The same kernels
 * as legend_rank_edges, but
 *   - every pointer is a DEVICE pointer (src, rel, dst [m]; candidates [num_candidates] or NULL
 *     for every node; outputs greater, equal [m] int32, metrics [4] double = MRR, Hits@1,
 *     Hits@3, Hits@10, status [1] uint32), all owned by the caller and all required except rel
 *     (Dot) and candidates;
 *   - the intermediate results (composed rows q_e, own scores, true endpoints) live in a static
 *     device buffer of 8 MiB inside the library instead of an allocation: one copy per GPU, held
 *     until the process ends.  The call is refused with LEGEND_E_INVAL when m exceeds
 *     legend_rank_edges_static_max_triples(dim) (18 368 triples at dim 100, 5 184 at dim 400);
 *   - it calls no hipMalloc / hipFree and no allocating routine, clears what must start at zero
 *     with a fill kernel, enqueues everything on the context's compute stream and returns without
 *     waiting: results are final after legend_sync (or a wait on the borrowed compute stream).
 *     Exception: if the buffer contents changed since the last scoring or ranking call, the
 *     partition table is re-sent first (one small copy and a stream synchronisation).
 * status: 0 = fine; bit 0: a node, relation or candidate id out of range; bit 1: a partition
 * that is not resident (the counts of the triples concerned are then meaningless).
 * Every call on a GPU shares that GPU's buffer, whatever the context or stream: calls that
 * overlap in time on one GPU race; serialise them.  Per-kernel profiling does not cover this call.
 */
int legend_rank_edges_static(legend_ctx* ctx, const int64_t* src, const int32_t* rel, const int64_t* dst,
                             int64_t m, int32_t side, const int64_t* candidates, int64_t num_candidates,
                             int32_t* greater, int32_t* equal, double* metrics, uint32_t* status);
/* Largest m legend_rank_edges_static accepts at embedding dimension dim (0: unsupported dim). */
int64_t legend_rank_edges_static_max_triples(int32_t dim);

/* Message of the last error on this thread ("" if none). */
const char* legend_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LEGEND_H */
