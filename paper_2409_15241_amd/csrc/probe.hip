// MFMA-only probe: what the matrix pipes of this chip sustain on the layer's kind of data when nothing else
// competes (no LDS, no memory traffic).  Under matrix load the clock is power-limited and depends on how many
// operand bits toggle, so the figure is measured on caller-provided fragments, not taken from the data sheet.
#include "probe.h"
#include "common.h"

namespace {

// Every wave keeps 8 independent 32x32x16 accumulators and issues iters x 8 MFMAs back to back on one A and one
// B fragment per lane, read once from memory.
__global__ __launch_bounds__(256)
void mfma_probe_kernel(const bf16x8* __restrict__ a, const bf16x8* __restrict__ b, float* __restrict__ out, int iters) {
  const bf16x8 fa = a[threadIdx.x], fb = b[threadIdx.x];
  f32x16 c[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[j][v] = 0.0f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, c[j], 0, 0, 0);
  float t = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) t += c[j][v];
  out[(long)blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace

hipError_t mfma_probe_launch(const void* a, const void* b, float* out, int blocks, int iters, hipStream_t st) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const bf16x8*>(a),
                     static_cast<const bf16x8*>(b), out, iters);
  return hipGetLastError();
}
