// LayerNorm / RMSNorm forward and backward with the surrounding residual traffic fused in
// (the "dropout, residual, LayerNorm" group of Sec. 4.1.1, dropout-free; RMSNorm per Sec. 5.4).
// HBM-bound: every access is a 16-byte chunk and a wave's 64 lanes cover 1 KiB contiguous bytes per
// instruction.  Statistics are fp32; wave reductions combined through LDS give the row sums.
#include "norm.h"
#include "common.h"

namespace {

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
// A workgroup of four waves owns one row, thread t the 16-byte chunks t, t+256, ... (at most 4: hidden <= 8192);
// every load of a phase is issued before the first is used (chunks past the row end read the last chunk instead
// of branching, and are masked out of the sums and stores); the two row sums cross the waves through LDS in wave
// order.  Under 96 registers a lane: such waves fit beside the two 192-register waves that a 256x256 product
// tile keeps on every SIMD.
template <int NC, bool RMS>
__global__ __launch_bounds__(256, 5)
void norm_fwd_kernel(const NormFwdArgs p) {
  __shared__ float red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int nch = p.h >> 3;
  const long ro = (long)row * p.h;
  const u32x4* x = reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.x) + ro);
  const u32x4* a1 = p.add1 ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.add1) + ro) : nullptr;
  const u32x4* a2 = p.add2 ? reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.add2) + ro) : nullptr;
  const u32x4* vec = reinterpret_cast<const u32x4*>(p.vec);
  const bool fused = a1 || a2 || vec;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  int cc[NC];
  bool live[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = tid + 256 * i;
    live[i] = c < nch;
    cc[i] = live[i] ? c : nch - 1;
  }
  u32x4 xs[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) xs[i] = x[cc[i]];
  if (fused) {
    u32x4 t1[NC], t2[NC], t3[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) t1[i] = a1 ? a1[cc[i]] : zero4;
#pragma unroll
    for (int i = 0; i < NC; ++i) t2[i] = a2 ? a2[cc[i]] : zero4;
#pragma unroll
    for (int i = 0; i < NC; ++i) t3[i] = vec ? vec[cc[i]] : zero4;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      float f[8], g[8];
      unpack8(xs[i], f);
      unpack8(t1[i], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] += g[e];
      unpack8(t2[i], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] += g[e];
      unpack8(t3[i], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] += g[e];
      xs[i] = pack8(f);
    }
    if (p.xsum) {
      u32x4* o = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.xsum) + ro);
#pragma unroll
      for (int i = 0; i < NC; ++i)
        if (live[i]) o[cc[i]] = xs[i];
    }
  }
  const u32x4* gam = reinterpret_cast<const u32x4*>(p.gamma);
  const u32x4* bet = reinterpret_cast<const u32x4*>(p.beta);
  u32x4 gs[NC], bs[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) gs[i] = gam[cc[i]];
  if (bet) {
#pragma unroll
    for (int i = 0; i < NC; ++i) bs[i] = bet[cc[i]];
  }

  const float inv_h = 1.0f / (float)p.h;
  float mean = 0.0f;
  if (!RMS) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      float f[8]; unpack8(xs[i], f);
      float t = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) t += f[e];
      s += live[i] ? t : 0.0f;
    }
    s = wave_sum(s);
    if (lane == 0) red[0][wave] = s;
    __syncthreads();
    mean = (((red[0][0] + red[0][1]) + red[0][2]) + red[0][3]) * inv_h;
  }
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    float f[8]; unpack8(xs[i], f);
    float t = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float d = f[e] - mean; t += d * d; }
    ss += live[i] ? t : 0.0f;
  }
  ss = wave_sum(ss);
  if (lane == 0) red[1][wave] = ss;
  __syncthreads();
  const float rstd = rsqrtf((((red[1][0] + red[1][1]) + red[1][2]) + red[1][3]) * inv_h + p.eps);
  if (tid == 0) {
    if (p.mean) p.mean[row] = mean;
    p.rstd[row] = rstd;
  }
  u32x4* y = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.y) + ro);
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    float f[8], g[8];
    unpack8(xs[i], f);
    unpack8(gs[i], g);
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (f[e] - mean) * rstd * g[e];
    if (bet) {
      unpack8(bs[i], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] += g[e];
    }
    if (live[i]) y[cc[i]] = pack8(f);
  }
}

// dx = dres + NormBwd(ga + gb); per-workgroup partial sums of d gamma / d beta.
// A workgroup owns a contiguous range of rows and walks it R rows at a time; thread t owns the 8
// columns of 16-byte chunk t in every row, so its share of the column sums (d gamma, d beta) is 16
// registers and every load of an iteration (R rows x up to 4 tensors) is in flight at once.  The two
// row sums cross the waves through LDS: wave sums in a double-buffered table, one barrier per
// iteration, added in wave order (fixed summation order).
template <int NT, int R, bool RMS, bool SUMS>
__global__ __launch_bounds__(NT)
void norm_bwd_kernel(const NormBwdArgs p, int rows_per_block) {
  constexpr int NW = NT / 64;
  constexpr int RW = 2 * R < 4 ? 4 : 2 * R;     // row sums per wave and iteration, padded to whole 16-byte reads
  __shared__ __align__(16) float red[2][NW][RW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nw = blockDim.x >> 6;
  const int nch = p.h >> 3;
  const bool live = tid < nch;
  const float inv_h = 1.0f / (float)p.h;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  float gm[8];
  unpack8(live ? reinterpret_cast<const u32x4*>(p.gamma)[tid] : zero4, gm);
  float dg[8], db[8], sres[8], sdx[8];     // sres / sdx: column sums of dres and of dx (SUMS only)
#pragma unroll
  for (int e = 0; e < 8; ++e) { dg[e] = 0.0f; db[e] = 0.0f; sres[e] = 0.0f; sdx[e] = 0.0f; }

  const int r0 = blockIdx.x * rows_per_block, r1 = min(p.rows, r0 + rows_per_block);
  // the rows of iteration k+1 are requested before iteration k is worked on, so the memory pipeline stays
  // busy across the barrier and the arithmetic of an iteration
  struct Rows { u32x4 xs[R], gs[R], bs[R], ds[R]; float mean[R], rstd[R]; };
  auto load_rows = [&](int rb, Rows& w) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int row = rb + j;
      const bool ok = live && row < r1;
      const long at = (long)row * p.h + tid * 8;
      w.xs[j] = ok ? *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.x) + at) : zero4;
      w.gs[j] = ok ? *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.ga) + at) : zero4;
      w.bs[j] = (ok && p.gb) ? *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.gb) + at) : zero4;
      w.ds[j] = (ok && p.dres) ? *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.dres) + at) : zero4;
      w.mean[j] = (!RMS && row < r1) ? p.mean[row] : 0.0f;
      w.rstd[j] = row < r1 ? p.rstd[row] : 0.0f;
    }
  };
  Rows cur, nxt;
  load_rows(r0, cur);
  int buf = 0;
  for (int rb = r0; rb < r1; rb += R, buf ^= 1) {
    load_rows(rb + R, nxt);                     // rows past r1 load nothing
    const u32x4 (&xs)[R] = cur.xs;
    const u32x4 (&gs)[R] = cur.gs;
    const u32x4 (&bs)[R] = cur.bs;
    const u32x4 (&ds)[R] = cur.ds;
    const float (&mean)[R] = cur.mean;
    const float (&rstd)[R] = cur.rstd;
    float sums[2 * R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      float xv[8], gv[8], bv[8];
      unpack8(xs[j], xv); unpack8(gs[j], gv); unpack8(bs[j], bv);
      float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        gv[e] += bv[e];
        const float xh = (xv[e] - mean[j]) * rstd[j];
        const float dxh = gv[e] * gm[e];
        s1 += dxh;
        s2 += dxh * xh;
        dg[e] += gv[e] * xh;
        if (!RMS) db[e] += gv[e];
      }
      sums[2 * j] = RMS ? 0.0f : wave_sum(s1);
      sums[2 * j + 1] = wave_sum(s2);
    }
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < RW; ++k) red[buf][wave][k] = k < 2 * R ? sums[k] : 0.0f;
    }
    __syncthreads();
    float tot[RW];
#pragma unroll
    for (int k = 0; k < RW; ++k) tot[k] = 0.0f;
    for (int w = 0; w < nw; ++w) {
#pragma unroll
      for (int k4 = 0; k4 < RW; k4 += 4) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(&red[buf][w][k4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) tot[k4 + e] += t[e];
      }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int row = rb + j;
      if (live && row < r1) {
        const float c1 = tot[2 * j] * inv_h, c2 = tot[2 * j + 1] * inv_h;
        float o[8], rv[8], xv[8], gv[8], bv[8];     // the incoming gradient is unpacked again rather than kept
        unpack8(ds[j], rv); unpack8(xs[j], xv); unpack8(gs[j], gv); unpack8(bs[j], bv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          o[e] = rstd[j] * ((gv[e] + bv[e]) * gm[e] - c1 - (xv[e] - mean[j]) * rstd[j] * c2) + rv[e];
          if (SUMS) { sres[e] += rv[e]; sdx[e] += o[e]; }
        }
        *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.dx) + (long)row * p.h + tid * 8) = pack8(o);
      }
    }
    cur = nxt;
  }
  if (live) {
    f32x4* pg = reinterpret_cast<f32x4*>(p.part_g + (long)blockIdx.x * p.h + tid * 8);
    pg[0] = f32x4{dg[0], dg[1], dg[2], dg[3]};
    pg[1] = f32x4{dg[4], dg[5], dg[6], dg[7]};
    if (!RMS) {
      f32x4* pb = reinterpret_cast<f32x4*>(p.part_b + (long)blockIdx.x * p.h + tid * 8);
      pb[0] = f32x4{db[0], db[1], db[2], db[3]};
      pb[1] = f32x4{db[4], db[5], db[6], db[7]};
    }
    if (SUMS) {
      f32x4* pr = reinterpret_cast<f32x4*>(p.part_dres + (long)blockIdx.x * p.h + tid * 8);
      pr[0] = f32x4{sres[0], sres[1], sres[2], sres[3]};
      pr[1] = f32x4{sres[4], sres[5], sres[6], sres[7]};
      f32x4* px = reinterpret_cast<f32x4*>(p.part_dx + (long)blockIdx.x * p.h + tid * 8);
      px[0] = f32x4{sdx[0], sdx[1], sdx[2], sdx[3]};
      px[1] = f32x4{sdx[4], sdx[5], sdx[6], sdx[7]};
    }
  }
}

// out[col] (+)= sum_k part[k][col]: the second stage of every column reduction, for up to
// COLSUM_MAX_JOBS independent reductions in one launch (blockIdx.y = job).  A workgroup owns 32
// columns; its 8 row groups each sum every 8th partial row, then the 8 group sums are added in
// group order (a fixed summation tree: results do not depend on scheduling).
__global__ __launch_bounds__(256)
void colsum_finish_kernel(const ColsumJobs jobs, int accumulate) {
  __shared__ float red[8][32];
  const ColsumJob job = jobs.job[blockIdx.y];
  if ((int)blockIdx.x * 32 >= job.n) return;
  const int c = threadIdx.x & 31, kg = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + c;
  float s = 0.0f;
  if (col < job.n) {
    for (int g = 0; g < job.nouter; ++g) {
      const float* part = job.part + (long)g * job.ostride + col;
#pragma unroll 4
      for (int k = kg; k < job.nparts; k += 8) s += part[(long)k * job.stride];
    }
  }
  red[kg][c] = s;
  __syncthreads();
  if (kg == 0 && col < job.n) {
    float t = red[0][c];
#pragma unroll
    for (int g = 1; g < 8; ++g) t += red[g][c];
    job.out[col] = accumulate ? job.out[col] + t : t;
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
  const int nq = ((a.h >> 3) + 255) / 256;               // 16-byte chunks per thread
  const dim3 grid(a.rows), block(256);
  if (nq <= 1) hipLaunchKernelGGL((norm_fwd_kernel<1, RMS>), grid, block, 0, st, a);
  else if (nq <= 2) hipLaunchKernelGGL((norm_fwd_kernel<2, RMS>), grid, block, 0, st, a);
  else if (nq <= 3) hipLaunchKernelGGL((norm_fwd_kernel<3, RMS>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((norm_fwd_kernel<4, RMS>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <bool RMS, bool SUMS>
hipError_t bwd_dispatch(const NormBwdArgs& a, int nblocks, hipStream_t st) {
  const int nt = (((a.h >> 3) + 63) / 64) * 64;           // one thread per 16-byte chunk of a row
  const int rpb = (a.rows + nblocks - 1) / nblocks;
  const dim3 grid(nblocks), block(nt);
  // rows per iteration: two iterations' loads are held at once, within the registers the block size leaves
  constexpr int RS = SUMS ? 2 : 4;
  if (nt <= 256) hipLaunchKernelGGL((norm_bwd_kernel<256, RS, RMS, SUMS>), grid, block, 0, st, a, rpb);
  else if (nt <= 512) hipLaunchKernelGGL((norm_bwd_kernel<512, RS, RMS, SUMS>), grid, block, 0, st, a, rpb);
  else if (nt <= 768) hipLaunchKernelGGL((norm_bwd_kernel<768, 2, RMS, SUMS>), grid, block, 0, st, a, rpb);
  else hipLaunchKernelGGL((norm_bwd_kernel<1024, 1, RMS, SUMS>), grid, block, 0, st, a, rpb);
  return hipGetLastError();
}

}  // namespace

int norm_bwd_blocks(int rows) {
  const int want = (rows + NORM_BWD_ROWS - 1) / NORM_BWD_ROWS;
  return want < NORM_BWD_MAX_BLOCKS ? want : NORM_BWD_MAX_BLOCKS;
}

hipError_t norm_fwd_launch(const NormFwdArgs& a, hipStream_t st) {
  return a.rms ? fwd_dispatch<true>(a, st) : fwd_dispatch<false>(a, st);
}

hipError_t norm_bwd_launch(const NormBwdArgs& a, hipStream_t st) {
  const int nb = norm_bwd_blocks(a.rows);
  const bool sums = a.part_dres && a.part_dx && a.dres;
  if (a.rms) return sums ? bwd_dispatch<true, true>(a, nb, st) : bwd_dispatch<true, false>(a, nb, st);
  return sums ? bwd_dispatch<false, true>(a, nb, st) : bwd_dispatch<false, false>(a, nb, st);
}

hipError_t colsum_finish_launch(const float* part, int nparts, int n, float* out, int accumulate, hipStream_t st) {
  ColsumJobs jobs{};
  jobs.job[0] = {part, out, nparts, n, (long)n, 1, 0};
  return colsum_finish_jobs_launch(jobs, 1, accumulate, st);
}

hipError_t colsum_finish_jobs_launch(const ColsumJobs& jobs, int njobs, int accumulate, hipStream_t st) {
  if (njobs <= 0) return hipSuccess;
  if (njobs > COLSUM_MAX_JOBS) return hipErrorInvalidValue;
  int widest = 0;
  for (int k = 0; k < njobs; ++k) widest = jobs.job[k].n > widest ? jobs.job[k].n : widest;
  hipLaunchKernelGGL(colsum_finish_kernel, dim3((widest + 31) / 32, njobs), dim3(256), 0, st, jobs, accumulate);
  return hipGetLastError();
}

hipError_t colsum_partial_launch(const void* g, long ld, int rows, int n, float* part, hipStream_t st) {
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((n / 8 + 63) / 64, COLSUM_PARTS), dim3(64), 0, st,
                     static_cast<const bf16_t*>(g), ld, rows, n, part);
  return hipGetLastError();
}
