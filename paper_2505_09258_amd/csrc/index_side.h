// The key of one occurrence (gradient row) of a batch, and for the rows of negatives the sampled id
// (paper Sec. 2.1 stages 1-2, Sec. 3 step 3).  Index arithmetic only; no floating point.
#pragma once

#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

// Occurrence o of the batch (positions as laid out in BatchGeom): its sort key = table base + row.
// Negative k of chunk c and side s is drawn with the counter hash H(prefix, c, s, k); the first
// N - num_degree_negs of a chunk uniformly over the valid rows of the side's partition, the others as
// the endpoint of a uniformly drawn edge of the bucket.  The id is stored once per chunk (row tile 0).
__device__ inline uint32_t occurrence_key(const BatchGeom& g, const BucketParams& bp, int64_t o,
                                          int32_t* __restrict__ neg_ids) {
    const int si = (int)(o / g.per_side);
    const int64_t r = o - (int64_t)si * g.per_side;
    const int side = g.side_id[si];
    const int32_t* eb = bp.edges + bp.batch_lo * 3;
    if (r < g.P) return (uint32_t)eb[r * 3 + 0];
    if (r < 2 * (int64_t)g.P) return bp.key_base_dst + (uint32_t)eb[(r - g.P) * 3 + 2];
    if (g.roles == 3 && r < 3 * (int64_t)g.P) return bp.key_base_rel + (uint32_t)eb[(r - 2 * (int64_t)g.P) * 3 + 1];
    const int64_t q = r - (int64_t)g.roles * g.P;
    const int k = (int)(q % g.N);
    const int64_t ct = q / g.N;
    const int t = (int)(ct % g.T);
    const int c = (int)(ct / g.T);
    const uint64_t h = hash_fold(hash_fold(hash_fold(bp.hash_prefix, (uint64_t)c), (uint64_t)side), (uint64_t)k);
    int32_t id;
    if (k < g.N - bp.num_degree_negs) {
        const uint64_t rows = (uint64_t)(side == 0 ? bp.rows_valid_dst : bp.rows_valid_src);
        id = (int32_t)__umul64hi(h, rows);
    } else {
        const uint64_t e = __umul64hi(h, (uint64_t)bp.m);
        id = bp.edges[e * 3 + (side == 0 ? 2 : 0)];
    }
    if (t == 0) neg_ids[((int64_t)si * g.nchunks + c) * g.N + k] = id;
    return (side == 0 ? bp.key_base_dst : 0u) + (uint32_t)id;
}

}  // namespace legend
