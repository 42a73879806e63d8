// Measured peaks of the GPU the library runs on, for the benchmark's roofline fractions: a loop of nothing but
// bf16 MFMAs on registers (no memory, no LDS) and a plain streaming copy.  Benchmark aids; not on the compute path.
#include "mfma_common.h"

namespace llsa {

// Every wave keeps 8 independent accumulators busy: 8 x iters MFMAs of 16 x 16 x 32 (16384 FLOP each).
__global__ void __launch_bounds__(256) peak_mfma_kernel(float *out, int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.5f + 0.001f * (float)(threadIdx.x & 7)); b[i] = (__bf16)(1.0f / (float)(i + 1)); }
    f32x4 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = mfma16(a, b, acc[k]);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    if (s == 123.456f) out[0] = s;                     // never true: keeps the loop alive
}

__global__ void __launch_bounds__(256) peak_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_peak_mfma(float *out, int iters, int workgroups, hipStream_t s) {
    peak_mfma_kernel<<<dim3((unsigned)workgroups), 256, 0, s>>>(out, iters);
    return hipGetLastError();
}

hipError_t launch_peak_copy(const void *src, void *dst, int64_t bytes, hipStream_t s) {
    const int64_t n16 = bytes / 16;
    const int64_t wgs = (n16 + 255) / 256;
    peak_copy_kernel<<<dim3((unsigned)(wgs < 65536 ? wgs : 65536)), 256, 0, s>>>(static_cast<const uint4 *>(src),
                                                                                  static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

}  // namespace llsa
