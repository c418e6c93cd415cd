// Small HBM-bound element-wise kernels: rotary embedding and the block's final residual sum.
#include "eltwise.h"
#include "common.h"

namespace {

// One thread per (row, group of 8 pair indices i < d/2): the 8 angles pos * base^(-2i/d) are computed once and
// the rotation applied to the pairs (i, i + d/2) of every head of every column block with 16-byte accesses.
// The head dimension is a multiple of 16 here (64, 80, 128), so a group never straddles the half.
__global__ __launch_bounds__(256)
void rope_kernel(bf16_t* __restrict__ m, long ld, int rows, int seq, int col0, int nblocks, int heads, int d,
                 float log2_base, int inverse) {
  const int half = d >> 1, groups = half >> 3;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)rows * groups) return;
  const int row = (int)(idx / groups), i0 = (int)(idx % groups) * 8;
  const float pos = (float)(row % seq);
  float sn[8], cs[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sincosf(pos * rope_freq(i0 + e, d, log2_base), &sn[e], &cs[e]);
    if (inverse) sn[e] = -sn[e];
  }
  bf16_t* r = m + (long)row * ld + col0 + i0;
  for (int blk = 0; blk < nblocks; ++blk)
    for (int hh = 0; hh < heads; ++hh) {
      u32x4* plo = reinterpret_cast<u32x4*>(r + (blk * heads + hh) * d);
      u32x4* phi = reinterpret_cast<u32x4*>(r + (blk * heads + hh) * d + half);
      const u32x4 lo = *plo, hi = *phi;
      u32x4 olo, ohi;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float a0 = bf16_lo(lo[w]), a1 = bf16_hi(lo[w]), b0 = bf16_lo(hi[w]), b1 = bf16_hi(hi[w]);
        olo[w] = pack_bf16(a0 * cs[2 * w] - b0 * sn[2 * w], a1 * cs[2 * w + 1] - b1 * sn[2 * w + 1]);
        ohi[w] = pack_bf16(b0 * cs[2 * w] + a0 * sn[2 * w], b1 * cs[2 * w + 1] + a1 * sn[2 * w + 1]);
      }
      *plo = olo;
      *phi = ohi;
    }
}

__global__ __launch_bounds__(256)
void residual_out_kernel(const u32x4* __restrict__ x1, const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                         const u32x4* __restrict__ vec, u32x4* __restrict__ y, long nchunks, int hch) {
  const long c = (long)blockIdx.x * 256 + threadIdx.x;
  if (c >= nchunks) return;
  // all four loads are issued before the first use: absent operands read x1 again and are dropped
  const u32x4 vx = x1[c], va = a[c];
  const u32x4 vb = (b ? b : x1)[c];
  const u32x4 vv = (vec ? vec : x1)[vec ? c % hch : c];
  // same association as the fused norm kernel, ((x1 + a) + b) + vec with absent operands as +0, so that a
  // caller may fold this sum into the next block's Norm1 without changing a bit
  float f[8];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = ((bf16_lo(vx[e]) + bf16_lo(va[e])) + (b ? bf16_lo(vb[e]) : 0.0f)) + (vec ? bf16_lo(vv[e]) : 0.0f);
    f[2 * e + 1] = ((bf16_hi(vx[e]) + bf16_hi(va[e])) + (b ? bf16_hi(vb[e]) : 0.0f)) + (vec ? bf16_hi(vv[e]) : 0.0f);
  }
  u32x4 o = {pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7])};
  y[c] = o;
}

}  // namespace

hipError_t rope_launch(void* m, long ld, int rows, int seq, int col0, int nblocks, int heads, int d,
                       float base, int inverse, hipStream_t st) {
  const long n = (long)rows * (d / 16);
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     static_cast<bf16_t*>(m), ld, rows, seq, col0, nblocks, heads, d, log2f(base), inverse);
  return hipGetLastError();
}

hipError_t residual_out_launch(const void* x1, const void* a, const void* b, const void* vec, void* y,
                               long n_elems, int h, hipStream_t st) {
  const long nch = n_elems / 8;
  hipLaunchKernelGGL(residual_out_kernel, dim3((unsigned)((nch + 255) / 256)), dim3(256), 0, st,
                     static_cast<const u32x4*>(x1), static_cast<const u32x4*>(a), static_cast<const u32x4*>(b),
                     static_cast<const u32x4*>(vec), static_cast<u32x4*>(y), nch, h / 8);
  return hipGetLastError();
}
