// Stand-alone measurement, not part of the library: the fp32 MFMA rate this device sustains when
// nothing but matrix instructions is issued (independent accumulators, operands in registers), for
// the two block shapes the kernels use and for one to eight waves per SIMD.  It gives the chunk
// kernels' roofline a second reference next to the published peak.
//   hipcc --offload-arch=gfx950 -O3 paper_2505_09258_amd/csrc/bench_mfma_peak.hip -o /tmp/mfma_peak && /tmp/mfma_peak
#include <hip/hip_runtime.h>

#include <cstdio>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int SHAPE>
__global__ void __launch_bounds__(256) k_mfma_only(float* out, int iters) {
    const float a = threadIdx.x * 1e-3f, b = blockIdx.x * 1e-3f;
    float s = 0.f;
    if (SHAPE == 16) {
        f32x4 acc[8];
        for (int i = 0; i < 8; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
        }
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    } else {
        f32x16 acc[4];
        for (int i = 0; i < 4; ++i)
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
        }
        for (int i = 0; i < 4; ++i)
            for (int v = 0; v < 16; ++v) s += acc[i][v];
    }
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            std::printf("%s failed: %s\n", #x, hipGetErrorString(e_));            \
            return 1;                                                             \
        }                                                                         \
    } while (0)

int main() {
    float* out = nullptr;
    CHECK(hipMalloc(&out, 2048 * 256 * sizeof(float)));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int iters = 20000;
    for (int wgs : {256, 512, 1024, 2048}) {          // 256 compute units: 1, 2, 4, 8 waves per SIMD
        for (int shape : {16, 32}) {
            float ms = 0.f;
            for (int rep = 0; rep < 2; ++rep) {       // the first launch warms up
                CHECK(hipEventRecord(e0));
                if (shape == 16) hipLaunchKernelGGL(k_mfma_only<16>, dim3(wgs), dim3(256), 0, 0, out, iters);
                else hipLaunchKernelGGL(k_mfma_only<32>, dim3(wgs), dim3(256), 0, 0, out, iters);
                CHECK(hipGetLastError());
                CHECK(hipEventRecord(e1));
                CHECK(hipEventSynchronize(e1));
                CHECK(hipEventElapsedTime(&ms, e0, e1));
            }
            const double flops = shape == 16 ? (double)wgs * 4 * iters * 8 * 2048.0 : (double)wgs * 4 * iters * 4 * 4096.0;
            std::printf("%d waves per SIMD, %s: %.3f ms, %.1f TFLOP/s\n", wgs / 256, shape == 16 ? "16x16x4" : "32x32x2", ms,
                        flops / ms / 1e9);
        }
    }
    CHECK(hipFree(out));
    return 0;
}
