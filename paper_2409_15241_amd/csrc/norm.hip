// LayerNorm / RMSNorm forward and backward with the surrounding residual traffic fused in
// (the "dropout, residual, LayerNorm" group of Sec. 4.1.1, dropout-free; RMSNorm per Sec. 5.4).
// HBM-bound: one wave owns a whole row in registers, every access is a 16-byte chunk and a wave's
// 64 lanes cover 1 KiB contiguous bytes per instruction.  Statistics are fp32; a wave reduction
// gives the row sums.
#include "norm.h"
#include "common.h"

namespace {

constexpr int MAXC = 16;   // 16-byte chunks per lane: hidden <= 8 * 64 * 16 = 8192

DEV void unpack8(const u32x4 v, float* f) {
  f[0] = bf16_lo(v[0]); f[1] = bf16_hi(v[0]); f[2] = bf16_lo(v[1]); f[3] = bf16_hi(v[1]);
  f[4] = bf16_lo(v[2]); f[5] = bf16_hi(v[2]); f[6] = bf16_lo(v[3]); f[7] = bf16_hi(v[3]);
}
DEV u32x4 pack8(const float* f) {
  u32x4 v = {pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7])};
  return v;
}

// y = Norm(x + add1 + add2 + vec) * gamma + beta; optionally writes the pre-norm sum (bf16) too.
// The statistics are taken from the bf16-rounded sum, i.e. from exactly what the backward re-reads.
template <int NC, bool RMS>
__global__ __launch_bounds__(256)
void norm_fwd_kernel(const NormFwdArgs p) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= p.rows) return;
  const int nch = p.h >> 3;
  const long ro = (long)row * p.h;
  const u32x4* x = reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.x) + ro);
  const u32x4* a1 = p.add1 ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.add1) + ro) : nullptr;
  const u32x4* a2 = p.add2 ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.add2) + ro) : nullptr;
  const u32x4* vec = reinterpret_cast<const u32x4*>(p.vec);
  const bool fused = a1 || a2 || vec;

  u32x4 xs[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    u32x4 z = {0u, 0u, 0u, 0u};
    xs[i] = c < nch ? x[c] : z;
  }
  if (fused) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float f[8], g[8];
        unpack8(xs[i], f);
        if (a1) { unpack8(a1[c], g);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] += g[e]; }
        if (a2) { unpack8(a2[c], g);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] += g[e]; }
        if (vec) { unpack8(vec[c], g);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] += g[e]; }
        xs[i] = pack8(f);
      }
    }
    if (p.xsum) {
      u32x4* o = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.xsum) + ro);
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) o[c] = xs[i];
      }
    }
  }

  const float inv_h = 1.0f / (float)p.h;
  float mean = 0.0f;
  if (!RMS) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      float f[8]; unpack8(xs[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += f[e];
    }
    mean = wave_sum(s) * inv_h;
  }
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      float f[8]; unpack8(xs[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = f[e] - mean; ss += d * d; }
    }
  }
  const float rstd = rsqrtf(wave_sum(ss) * inv_h + p.eps);
  if (lane == 0) {
    if (p.mean) p.mean[row] = mean;
    p.rstd[row] = rstd;
  }
  const u32x4* gam = reinterpret_cast<const u32x4*>(p.gamma);
  const u32x4* bet = reinterpret_cast<const u32x4*>(p.beta);
  u32x4* y = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.y) + ro);
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      float f[8], g[8];
      unpack8(xs[i], f);
      unpack8(gam[c], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = (f[e] - mean) * rstd * g[e];
      if (bet) {
        unpack8(bet[c], g);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] += g[e];
      }
      y[c] = pack8(f);
    }
  }
}

// dx = dres + NormBwd(ga + gb); per-workgroup partial sums of d gamma / d beta.
// A wave walks rows wave_id, wave_id + total_waves, ... and keeps the column sums of its lanes'
// columns in registers; the 4 waves of a workgroup then combine through LDS in a fixed order.
template <int NC, bool RMS>
__global__ __launch_bounds__(256)
void norm_bwd_kernel(const NormBwdArgs p) {
  extern __shared__ float red[];      // [2][h]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nch = p.h >> 3;
  const float inv_h = 1.0f / (float)p.h;
  const u32x4* gam = reinterpret_cast<const u32x4*>(p.gamma);

  float dg[NC][8], db[RMS ? 1 : NC][8];
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) { dg[i][e] = 0.0f; if (!RMS) db[i][e] = 0.0f; }

  for (int row = blockIdx.x * 4 + wave; row < p.rows; row += gridDim.x * 4) {
    const long ro = (long)row * p.h;
    const u32x4* x = reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.x) + ro);
    const u32x4* ga = reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.ga) + ro);
    const u32x4* gb = p.gb ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.gb) + ro) : nullptr;
    const u32x4* dres = p.dres ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.dres) + ro) : nullptr;
    u32x4* dx = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.dx) + ro);
    const float mean = RMS ? 0.0f : p.mean[row];
    const float rstd = p.rstd[row];

    u32x4 xs[NC], gs[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      u32x4 z = {0u, 0u, 0u, 0u};
      xs[i] = c < nch ? x[c] : z;
      gs[i] = c < nch ? ga[c] : z;
    }
    if (gb) {
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
          float f[8], g[8];
          unpack8(gs[i], f); unpack8(gb[c], g);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] += g[e];
          gs[i] = pack8(f);
        }
      }
    }
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float xv[8], gv[8], gm[8];
        unpack8(xs[i], xv); unpack8(gs[i], gv); unpack8(gam[c], gm);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (xv[e] - mean) * rstd;
          const float dxh = gv[e] * gm[e];
          s1 += dxh;
          s2 += dxh * xh;
          dg[i][e] += gv[e] * xh;
          if (!RMS) db[i][e] += gv[e];
        }
      }
    }
    const float c1 = RMS ? 0.0f : wave_sum(s1) * inv_h;
    const float c2 = wave_sum(s2) * inv_h;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float xv[8], gv[8], gm[8], o[8];
        unpack8(xs[i], xv); unpack8(gs[i], gv); unpack8(gam[c], gm);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (xv[e] - mean) * rstd;
          o[e] = rstd * (gv[e] * gm[e] - c1 - xh * c2);
        }
        if (dres) {
          float r[8]; unpack8(dres[c], r);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += r[e];
        }
        dx[c] = pack8(o);
      }
    }
  }

  // combine the 4 waves in order 0,1,2,3 and write this workgroup's partial row
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int col = c * 8 + e;
            if (w == 0) { red[col] = dg[i][e]; if (!RMS) red[p.h + col] = db[i][e]; }
            else { red[col] += dg[i][e]; if (!RMS) red[p.h + col] += db[i][e]; }
          }
        }
      }
    }
    __syncthreads();
  }
  float* pg = p.part_g + (long)blockIdx.x * p.h;
  float* pb = RMS ? nullptr : p.part_b + (long)blockIdx.x * p.h;
  for (int col = threadIdx.x; col < p.h; col += 256) {
    pg[col] = red[col];
    if (!RMS) pb[col] = red[p.h + col];
  }
}

// out[col] (+)= sum_k part[k][col]: the second stage of every column reduction.  A workgroup owns 32
// columns; its 8 row groups each sum every 8th partial row, then the 8 group sums are added in
// group order (a fixed summation tree: results do not depend on scheduling).
__global__ __launch_bounds__(256)
void colsum_finish_kernel(const float* __restrict__ part, int nparts, long stride, int n, float* __restrict__ out, int accumulate) {
  __shared__ float red[8][32];
  const int c = threadIdx.x & 31, kg = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + c;
  float s = 0.0f;
  if (col < n) {
#pragma unroll 4
    for (int k = kg; k < nparts; k += 8) s += part[(long)k * stride + col];
  }
  red[kg][c] = s;
  __syncthreads();
  if (kg == 0 && col < n) {
    float t = red[0][c];
#pragma unroll
    for (int g = 1; g < 8; ++g) t += red[g][c];
    out[col] = accumulate ? out[col] + t : t;
  }
}

// part[blockIdx.y][col] = sum over this block's row range of g[row][col] (bf16 in, fp32 out).
__global__ __launch_bounds__(64)
void colsum_partial_kernel(const bf16_t* __restrict__ g, long ld, int rows, int n, float* __restrict__ part) {
  const int chunk = blockIdx.x * 64 + threadIdx.x;      // 8 columns
  if (chunk * 8 >= n) return;
  const int per = (rows + gridDim.y - 1) / gridDim.y;
  const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
  for (int r = r0; r < r1; ++r) {
    float f[8];
    unpack8(*reinterpret_cast<const u32x4*>(g + (long)r * ld + chunk * 8), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += f[e];
  }
  float* o = part + (long)blockIdx.y * n + chunk * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = acc[e];
}

template <bool RMS>
hipError_t fwd_dispatch(const NormFwdArgs& a, hipStream_t st) {
  const int nc = ((a.h >> 3) + 63) / 64;
  dim3 grid((a.rows + 3) / 4), block(256);
  if (nc <= 4) hipLaunchKernelGGL((norm_fwd_kernel<4, RMS>), grid, block, 0, st, a);
  else if (nc <= 8) hipLaunchKernelGGL((norm_fwd_kernel<8, RMS>), grid, block, 0, st, a);
  else if (nc <= 10) hipLaunchKernelGGL((norm_fwd_kernel<10, RMS>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((norm_fwd_kernel<MAXC, RMS>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <int NC, bool RMS>
hipError_t bwd_launch(const NormBwdArgs& a, int nblocks, hipStream_t st) {
  auto kern = norm_bwd_kernel<NC, RMS>;
  const int lds = 2 * a.h * (int)sizeof(float);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(nblocks), dim3(256), lds, st, a);
  return hipGetLastError();
}

template <bool RMS>
hipError_t bwd_dispatch(const NormBwdArgs& a, int nblocks, hipStream_t st) {
  const int nc = ((a.h >> 3) + 63) / 64;
  if (nc <= 4) return bwd_launch<4, RMS>(a, nblocks, st);
  if (nc <= 8) return bwd_launch<8, RMS>(a, nblocks, st);
  if (nc <= 10) return bwd_launch<10, RMS>(a, nblocks, st);
  return bwd_launch<MAXC, RMS>(a, nblocks, st);
}

}  // namespace

int norm_bwd_blocks(int rows) {
  const int want = (rows + 3) / 4;
  return want < NORM_BWD_MAX_BLOCKS ? want : NORM_BWD_MAX_BLOCKS;
}

hipError_t norm_fwd_launch(const NormFwdArgs& a, hipStream_t st) {
  return a.rms ? fwd_dispatch<true>(a, st) : fwd_dispatch<false>(a, st);
}

hipError_t norm_bwd_launch(const NormBwdArgs& a, hipStream_t st) {
  const int nb = norm_bwd_blocks(a.rows);
  return a.rms ? bwd_dispatch<true>(a, nb, st) : bwd_dispatch<false>(a, nb, st);
}

hipError_t colsum_finish_launch(const float* part, int nparts, int n, float* out, int accumulate, hipStream_t st) {
  return colsum_finish_strided_launch(part, nparts, n, n, out, accumulate, st);
}

hipError_t colsum_finish_strided_launch(const float* part, int nparts, long stride, int n, float* out, int accumulate, hipStream_t st) {
  hipLaunchKernelGGL(colsum_finish_kernel, dim3((n + 31) / 32), dim3(256), 0, st, part, nparts, stride, n, out, accumulate);
  return hipGetLastError();
}

hipError_t colsum_partial_launch(const void* g, long ld, int rows, int n, float* part, hipStream_t st) {
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((n / 8 + 63) / 64, COLSUM_PARTS), dim3(64), 0, st,
                     static_cast<const bf16_t*>(g), ld, rows, n, part);
  return hipGetLastError();
}
