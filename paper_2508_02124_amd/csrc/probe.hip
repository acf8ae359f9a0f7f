// Measurement aids for the roofline report (no part of the method, and a library of their own:
// libdma_probe.so, include/dma_probe.h): the rate the matrix cores reach from registers alone with the
// instruction the attention kernels use, and a plain streaming copy.
#include "common.h"
#include "../../include/dma_probe.h"

namespace dma {

// Every wave runs `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 chains on constant
// operands (2 * 32 * 32 * 16 flops each); the sums are stored so that nothing is optimised away.
__global__ __launch_bounds__(512) void probe_mfma_kernel(float* sink, int iters) {
  const int l = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; e++) {
    a[e] = (__bf16)(0.001f * (float)(l + e));
    b[e] = (__bf16)(0.002f * (float)(l - e));
  }
  f32x16 acc[8];
#pragma unroll
  for (int c = 0; c < 8; c++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[c][v] = 0.f;
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int c = 0; c < 8; c++) acc[c] = mfma32(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < 8; c++)
#pragma unroll
    for (int v = 0; v < 16; v++) s += acc[c][v];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += st) dst[i] = src[i];
}

}  // namespace dma

extern "C" {

int dma_probe_mfma(float* sink, int n_workgroups, int iters, void* stream) {
  if (!sink || n_workgroups <= 0 || iters <= 0) return DMA_EINVAL;
  dma::probe_mfma_kernel<<<n_workgroups, 512, 0, (hipStream_t)stream>>>(sink, iters);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int dma_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  const bool aligned = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0;
  if (!src || !dst || bytes == 0 || bytes % 16 || !aligned) return DMA_EINVAL;
  dma::probe_copy_kernel<<<8192, 256, 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, bytes / 16);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // extern "C"
