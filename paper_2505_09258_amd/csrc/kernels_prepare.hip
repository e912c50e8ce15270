// Small helpers around a bucket call: validation of a bucket's edge ids, plain fills, and the seeded
// initial embeddings (paper Sec. 3 steps 1-3).
#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

__global__ void __launch_bounds__(256)
k_validate_edges(const int32_t* __restrict__ edges, int64_t m, int32_t rows_src, int32_t rows_dst,
                 int32_t num_rel, int check_rel, uint32_t* __restrict__ err_flag) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (; e < m; e += stride) {
        int32_t s = edges[e * 3 + 0], r = edges[e * 3 + 1], d = edges[e * 3 + 2];
        bad |= (s < 0) | (s >= rows_src) | (d < 0) | (d >= rows_dst);
        if (check_rel) bad |= (r < 0) | (r >= num_rel);
    }
    if (bad) atomicOr(err_flag, 1u);
}

hipError_t launch_validate_edges(hipStream_t st, const int32_t* edges, int64_t m, int32_t rows_src,
                                 int32_t rows_dst, int32_t num_rel, int check_rel, uint32_t* err_flag) {
    if (m <= 0) return hipSuccess;
    int64_t blocks = (m + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_validate_edges, dim3((unsigned)blocks), dim3(256), 0, st, edges, m, rows_src, rows_dst,
                       num_rel, check_rel, err_flag);
    return hipGetLastError();
}

// Plain fill of 32-bit words: clears counters and flags where a memset node must not be recorded.
__global__ void __launch_bounds__(256) k_fill_u32(uint32_t* __restrict__ p, uint32_t v, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t n) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, st, p, v, n);
    return hipGetLastError();
}

// Seeded initial embeddings ("randomly initialized", Sec. 3 step 1; the distribution is not printed):
// element (row g, column k) of a table is a pure integer function of (seed, table tag, g, k),
//     h = fold(fold(fold(seed, tag), g), k),   u = sum of the four 16-bit fields of h  (0 .. 262140),
//     value = float(int(u) - 131070) * scale,  scale = float(init_std * sqrt(3) / 65536),
// a sum of four uniform integers: mean 0, standard deviation init_std, no transcendental function.
__global__ void __launch_bounds__(256)
k_init_fill(float* __restrict__ out, int64_t rows, int32_t dim, int64_t row0, uint64_t table_hash, float scale) {
    const int64_t total = rows * dim;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / dim;
        const int k = (int)(idx - r * dim);
        const uint64_t h = hash_fold(hash_fold(table_hash, (uint64_t)(row0 + r)), (uint64_t)k);
        const int32_t u = (int32_t)((h & 0xFFFFu) + ((h >> 16) & 0xFFFFu) + ((h >> 32) & 0xFFFFu) + (h >> 48));
        out[idx] = (float)(u - 131070) * scale;
    }
}

hipError_t launch_init_fill(hipStream_t st, float* out, int64_t rows, int32_t dim, int64_t row0, uint64_t seed,
                            uint64_t table_tag, float init_std) {
    if (rows <= 0) return hipSuccess;
    const float scale = (float)((double)init_std * 1.7320508075688772 / 65536.0);
    int64_t blocks = (rows * dim + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_init_fill, dim3((unsigned)blocks), dim3(256), 0, st, out, rows, dim, row0,
                       hash_fold(seed, table_tag), scale);
    return hipGetLastError();
}

}  // namespace legend
