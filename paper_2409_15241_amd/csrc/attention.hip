// Causal flash-style attention for one head shard on gfx950 MFMA (Eq. 2, first case:
// softmax(Q K^T / sqrt(d_k)) V; kept as one fused kernel because the first weight group is never
// sliced, Sec. 3.1), forward and backward.
//
// All products are computed transposed so that the query (forward, dQ pass) or key (dK/dV pass)
// index of an MFMA accumulator is the LANE and the other index lives in the lane's 16 registers:
//   S^T[kv, q] = K Q^T          row statistics of a query are then a reduction over one lane's
//   O^T[d, q]  = V^T P^T        registers plus one exchange between the two lane halves, and the
// probabilities never leave registers: an accumulator converted to bf16 is directly the second
// operand of the next product, provided the first operand's contraction index is gathered in the
// accumulator's row order (MoverKS<.., PERM=true>).
//
// Backward is two passes without atomics (run-to-run identical results):
//   dQ pass, one workgroup per 128 queries: recompute P^T from the saved log-sum-exp,
//     dP^T = V dO^T, dS^T = P^T (dP^T - D), dQ^T += K^T dS^T.
//   dK/dV pass, one workgroup per 128 keys: P = exp(S - lse), dV^T += dO^T P, dP = dO V^T,
//     dS = P (dP - D), dK^T += Q^T dS.
// D[q] = sum_d dO[q,d] O[q,d] comes from a small pre-pass.
#include "attention.h"
#include "lds_tile.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

template <int D>
struct Dims {
  static constexpr int DK = (D + 63) / 64;            // 64-wide contraction sub-tiles along d
  static constexpr int DPAD = ((D + 31) / 32) * 32;   // rows of a transposed ([d][pos]) tile
  static constexpr int DT = DPAD / 32;
  static constexpr int KSTEPS = D / 16;               // MFMA steps of a contraction over d
  static constexpr int KC_BYTES = DK * 64 * TILE_ROW_BYTES;   // [DK][64 pos][64 d]
  static constexpr int KS_BYTES = DPAD * TILE_ROW_BYTES;      // [DPAD d][64 pos]
};

// B-operand fragments straight from HBM: lane (pos = row0 + lane%32, half) takes 8 consecutive d.
template <int D>
DEV void load_row_frags(const bf16_t* __restrict__ base, long ld, int pos, int seq, int fh,
                        bf16x8 (&f)[Dims<D>::KSTEPS]) {
#pragma unroll
  for (int ks = 0; ks < Dims<D>::KSTEPS; ++ks) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (pos < seq) v = *reinterpret_cast<const u32x4*>(base + (long)pos * ld + ks * 16 + fh * 8);
    f[ks] = __builtin_bit_cast(bf16x8, v);
  }
}

// acc[t] (t = 0,1: two 32-row groups of the 64-position LDS tile) += Tile[32t.., d] * frag[d, lane]
template <int D>
DEV void mma_tile_rows(const uint8_t* kc_tile, const bf16x8 (&f)[Dims<D>::KSTEPS], int fr, int fh, f32x16 (&acc)[2]) {
#pragma unroll
  for (int ks = 0; ks < Dims<D>::KSTEPS; ++ks) {
    const uint8_t* sub = kc_tile + (ks >> 2) * (64 * TILE_ROW_BYTES);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16x8 a = lds_read_frag<false>(sub, 32 * t + fr, 2 * (ks & 3) + fh);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, f[ks], acc[t], 0, 0, 0);
    }
  }
}

// out[dt] += TileT[32dt.., pos] * bf16(vals)[pos, lane]; vals = two accumulators covering 64 positions
template <int D>
DEV void mma_tile_cols(const uint8_t* ks_tile, const f32x16 (&vals)[2], int fr, int fh, f32x16 (&out)[Dims<D>::DT]) {
  bf16x8 pf[4];
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    const int t = s4 >> 1, u = s4 & 1;
    u32x4 w = {pack_bf16(vals[t][8 * u + 0], vals[t][8 * u + 1]), pack_bf16(vals[t][8 * u + 2], vals[t][8 * u + 3]),
               pack_bf16(vals[t][8 * u + 4], vals[t][8 * u + 5]), pack_bf16(vals[t][8 * u + 6], vals[t][8 * u + 7])};
    pf[s4] = __builtin_bit_cast(bf16x8, w);
  }
#pragma unroll
  for (int dt = 0; dt < Dims<D>::DT; ++dt)
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const bf16x8 a = lds_read_frag<true>(ks_tile, 32 * dt + fr, 2 * s4 + fh);
      out[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[s4], out[dt], 0, 0, 0);
    }
}

// accumulator register v of the lane half fh holds tile row 8 (v/4) + 4 fh + v%4
DEV int acc_row(int v, int fh) { return 8 * (v >> 2) + 4 * fh + (v & 3); }

// store out^T[d, pos] (one lane = one position) as bf16 rows of a [pos][..] matrix, scaled
template <int D>
DEV void store_transposed(const f32x16 (&o)[Dims<D>::DT], float scale, bf16_t* __restrict__ row_ptr, int fh) {
#pragma unroll
  for (int dt = 0; dt < Dims<D>::DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int dd = 32 * dt + 8 * g + 4 * fh;
      if (dd < D) {
        u32x2 w = {pack_bf16(o[dt][4 * g] * scale, o[dt][4 * g + 1] * scale),
                   pack_bf16(o[dt][4 * g + 2] * scale, o[dt][4 * g + 3] * scale)};
        *reinterpret_cast<u32x2*>(row_ptr + dd) = w;
      }
    }
}

// ------------------------------------------------------------------------------------- forward
template <int D>
__global__ __launch_bounds__(256)
void attn_fwd_kernel(const AttnArgs p) {
  using X = Dims<D>;
  constexpr int STAGE = X::KC_BYTES + X::KS_BYTES;      // K tile [kv][d] and V tile [d][kv]
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int fr = lane & 31, fh = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;            // longest rows first
  const int hh = blockIdx.y, bi = blockIdx.z;
  const int s = p.seq;
  const int qw0 = qb * 128 + wave * 32, qpos = qw0 + fr;
  const long ld = p.ld;
  const bf16_t* tok0 = static_cast<const bf16_t*>(p.qkv) + (long)bi * s * ld;
  const int hl = p.heads * D;
  const long view_bytes = ((long)(s - 1) * ld + D) * 2;
  const buf_rsrc rsK = make_rsrc(tok0 + hl + hh * D, view_bytes);
  const buf_rsrc rsV = make_rsrc(tok0 + 2 * hl + hh * D, view_bytes);

  bf16x8 qf[X::KSTEPS];
  load_row_frags<D>(tok0 + hh * D, ld, qpos, s, fh, qf);

  MoverKC<64, 256> mvK[X::DK];
  MoverKS<X::DPAD, 256, true> mvV;
#pragma unroll
  for (int c = 0; c < X::DK; ++c) mvK[c].init((int)ld, 0, 1 << 30, tid);
  mvV.init((int)ld, IdentityCols{0, D}, tid);
  auto load_tiles = [&](int kv0) {
#pragma unroll
    for (int c = 0; c < X::DK; ++c) mvK[c].load(rsK, c * 64, D, (uint32_t)kv0 * (uint32_t)ld * 2u);
    mvV.load(rsV, kv0, 0);
  };
  auto store_tiles = [&](uint8_t* st) {
#pragma unroll
    for (int c = 0; c < X::DK; ++c) mvK[c].store(st + c * 64 * TILE_ROW_BYTES, tid);
    mvV.store(st + X::KC_BYTES, tid);
  };

  const int q_end = min(qb * 128 + 128, s);
  const int ntiles = (q_end + 63) / 64;
  f32x16 o[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.0f;
  float m = -INFINITY, l = 0.0f;
  const float sc = p.scale * LOG2E;

  load_tiles(0);
  store_tiles(smem);
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const uint8_t* st = smem + (j & 1) * STAGE;
    const int kv0 = j * 64;
    if (j + 1 < ntiles) load_tiles(kv0 + 64);
    if (kv0 <= qw0 + 31) {                               // this wave has unmasked keys in the tile
      f32x16 sT[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) sT[t][v] = 0.0f;
      mma_tile_rows<D>(st, qf, fr, fh, sT);
      const bool diag = kv0 + 63 > qw0;
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = sT[t][v] * sc;
          if (diag && kv0 + 32 * t + acc_row(v, fh) > qpos) x = -INFINITY;
          sT[t][v] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);                  // finite: key 0 is visible to every query
      const float alpha = exp2f(m - m_new);
      float rs = 0.0f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float e = exp2f(sT[t][v] - m_new);
          sT[t][v] = e;
          rs += e;
        }
      l = l * alpha + rs;
      m = m_new;
#pragma unroll
      for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
      mma_tile_cols<D>(st + X::KC_BYTES, sT, fr, fh, o);
    }
    if (j + 1 < ntiles) store_tiles(smem + ((j + 1) & 1) * STAGE);
    __syncthreads();
  }
  l += __shfl_xor(l, 32, 64);
  if (qpos < s) {
    bf16_t* out = static_cast<bf16_t*>(p.ctx) + ((long)bi * s + qpos) * p.ld_ctx + hh * D;
    store_transposed<D>(o, 1.0f / l, out, fh);
    if (fh == 0) p.lse[((long)bi * p.heads + hh) * s + qpos] = (m + log2f(l)) * LN2;
  }
}

// ------------------------------------------------------------------------------------- D = rowsum(dO * O)
__global__ __launch_bounds__(256)
void attn_dot_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dO, long ld, int rows, int seq,
                     int heads, int d, float* __restrict__ dot) {
  // one thread per (row, head): heads*d contiguous bf16 per row, d/8 16-byte chunks per head
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)rows * heads) return;
  const int row = (int)(idx / heads), hh = (int)(idx % heads);
  const u32x4* a = reinterpret_cast<const u32x4*>(o + (long)row * ld + hh * d);
  const u32x4* b = reinterpret_cast<const u32x4*>(dO + (long)row * ld + hh * d);
  float acc = 0.0f;
  for (int c = 0; c < d / 8; ++c) {
    const u32x4 x = a[c], y = b[c];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc += bf16_lo(x[e]) * bf16_lo(y[e]) + bf16_hi(x[e]) * bf16_hi(y[e]);
  }
  const int bi = row / seq, pos = row % seq;
  dot[((long)bi * heads + hh) * seq + pos] = acc;
}

// ------------------------------------------------------------------------------------- dQ pass
template <int D>
__global__ __launch_bounds__(256)
void attn_bwd_dq_kernel(const AttnArgs p) {
  using X = Dims<D>;
  constexpr int STAGE = 2 * X::KC_BYTES + X::KS_BYTES;  // K [kv][d], V [kv][d], K^T [d][kv]
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int fr = lane & 31, fh = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int hh = blockIdx.y, bi = blockIdx.z;
  const int s = p.seq;
  const int qw0 = qb * 128 + wave * 32, qpos = qw0 + fr;
  const long ld = p.ld;
  const bf16_t* tok0 = static_cast<const bf16_t*>(p.qkv) + (long)bi * s * ld;
  const int hl = p.heads * D;
  const long view_bytes = ((long)(s - 1) * ld + D) * 2;
  const buf_rsrc rsK = make_rsrc(tok0 + hl + hh * D, view_bytes);
  const buf_rsrc rsV = make_rsrc(tok0 + 2 * hl + hh * D, view_bytes);

  bf16x8 qf[X::KSTEPS], dof[X::KSTEPS];
  load_row_frags<D>(tok0 + hh * D, ld, qpos, s, fh, qf);
  load_row_frags<D>(static_cast<const bf16_t*>(p.dctx) + (long)bi * s * p.ld_ctx + hh * D, p.ld_ctx, qpos, s, fh, dof);
  const long stat = ((long)bi * p.heads + hh) * s + qpos;
  const float lse2 = qpos < s ? p.lse[stat] * LOG2E : INFINITY;
  const float dq_dot = qpos < s ? p.dot[stat] : 0.0f;

  MoverKC<64, 256> mvK[X::DK], mvV[X::DK];
  MoverKS<X::DPAD, 256, true> mvKt;
#pragma unroll
  for (int c = 0; c < X::DK; ++c) { mvK[c].init((int)ld, 0, 1 << 30, tid); mvV[c].init((int)ld, 0, 1 << 30, tid); }
  mvKt.init((int)ld, IdentityCols{0, D}, tid);
  auto load_tiles = [&](int kv0) {
    const uint32_t ro = (uint32_t)kv0 * (uint32_t)ld * 2u;
#pragma unroll
    for (int c = 0; c < X::DK; ++c) { mvK[c].load(rsK, c * 64, D, ro); mvV[c].load(rsV, c * 64, D, ro); }
    mvKt.load(rsK, kv0, 0);
  };
  auto store_tiles = [&](uint8_t* st) {
#pragma unroll
    for (int c = 0; c < X::DK; ++c) {
      mvK[c].store(st + c * 64 * TILE_ROW_BYTES, tid);
      mvV[c].store(st + X::KC_BYTES + c * 64 * TILE_ROW_BYTES, tid);
    }
    mvKt.store(st + 2 * X::KC_BYTES, tid);
  };

  const int q_end = min(qb * 128 + 128, s);
  const int ntiles = (q_end + 63) / 64;
  f32x16 dq[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[dt][v] = 0.0f;
  const float sc = p.scale * LOG2E;

  load_tiles(0);
  store_tiles(smem);
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const uint8_t* st = smem + (j & 1) * STAGE;
    const int kv0 = j * 64;
    if (j + 1 < ntiles) load_tiles(kv0 + 64);
    if (kv0 <= qw0 + 31) {
      f32x16 sT[2], dpT[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) { sT[t][v] = 0.0f; dpT[t][v] = 0.0f; }
      mma_tile_rows<D>(st, qf, fr, fh, sT);
      mma_tile_rows<D>(st + X::KC_BYTES, dof, fr, fh, dpT);
      const bool diag = kv0 + 63 > qw0;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float pr = exp2f(sT[t][v] * sc - lse2);
          if (diag && kv0 + 32 * t + acc_row(v, fh) > qpos) pr = 0.0f;
          sT[t][v] = pr * (dpT[t][v] - dq_dot);
        }
      mma_tile_cols<D>(st + 2 * X::KC_BYTES, sT, fr, fh, dq);
    }
    if (j + 1 < ntiles) store_tiles(smem + ((j + 1) & 1) * STAGE);
    __syncthreads();
  }
  if (qpos < s) {
    bf16_t* out = static_cast<bf16_t*>(p.dqkv) + ((long)bi * s + qpos) * ld + hh * D;
    store_transposed<D>(dq, p.scale, out, fh);
  }
}

// ------------------------------------------------------------------------------------- dK / dV pass
template <int D>
__global__ __launch_bounds__(256)
void attn_bwd_dkv_kernel(const AttnArgs p) {
  using X = Dims<D>;
  constexpr int TILES = 2 * X::KC_BYTES + 2 * X::KS_BYTES;   // Q, dO [q][d]; Q^T, dO^T [d][q]
  constexpr int STAGE = TILES + 2 * 64 * 4;                   // + lse2[64], dot[64]
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int fr = lane & 31, fh = lane >> 5;
  const int kb = blockIdx.x;                                  // 128 keys per workgroup
  const int hh = blockIdx.y, bi = blockIdx.z;
  const int s = p.seq;
  const int kw0 = kb * 128 + wave * 32, kpos = kw0 + fr;
  const long ld = p.ld, ldc = p.ld_ctx;
  const bf16_t* tok0 = static_cast<const bf16_t*>(p.qkv) + (long)bi * s * ld;
  const bf16_t* do0 = static_cast<const bf16_t*>(p.dctx) + (long)bi * s * ldc + hh * D;
  const int hl = p.heads * D;
  const buf_rsrc rsQ = make_rsrc(tok0 + hh * D, ((long)(s - 1) * ld + D) * 2);
  const buf_rsrc rsO = make_rsrc(do0, ((long)(s - 1) * ldc + D) * 2);
  const float* lse = p.lse + ((long)bi * p.heads + hh) * s;
  const float* dot = p.dot + ((long)bi * p.heads + hh) * s;

  bf16x8 kf[X::KSTEPS], vf[X::KSTEPS];
  load_row_frags<D>(tok0 + hl + hh * D, ld, kpos, s, fh, kf);
  load_row_frags<D>(tok0 + 2 * hl + hh * D, ld, kpos, s, fh, vf);

  MoverKC<64, 256> mvQ[X::DK], mvO[X::DK];
  MoverKS<X::DPAD, 256, true> mvQt, mvOt;
#pragma unroll
  for (int c = 0; c < X::DK; ++c) { mvQ[c].init((int)ld, 0, 1 << 30, tid); mvO[c].init((int)ldc, 0, 1 << 30, tid); }
  mvQt.init((int)ld, IdentityCols{0, D}, tid);
  mvOt.init((int)ldc, IdentityCols{0, D}, tid);
  float st_lse = 0.0f, st_dot = 0.0f;
  auto load_tiles = [&](int q0) {
#pragma unroll
    for (int c = 0; c < X::DK; ++c) {
      mvQ[c].load(rsQ, c * 64, D, (uint32_t)q0 * (uint32_t)ld * 2u);
      mvO[c].load(rsO, c * 64, D, (uint32_t)q0 * (uint32_t)ldc * 2u);
    }
    mvQt.load(rsQ, q0, 0);
    mvOt.load(rsO, q0, 0);
    if (tid < 64) {
      const int q = q0 + tid;
      st_lse = q < s ? lse[q] * LOG2E : INFINITY;     // exp2(x - inf) = 0 for rows past the end
      st_dot = q < s ? dot[q] : 0.0f;
    }
  };
  auto store_tiles = [&](uint8_t* st) {
#pragma unroll
    for (int c = 0; c < X::DK; ++c) {
      mvQ[c].store(st + c * 64 * TILE_ROW_BYTES, tid);
      mvO[c].store(st + X::KC_BYTES + c * 64 * TILE_ROW_BYTES, tid);
    }
    mvQt.store(st + 2 * X::KC_BYTES, tid);
    mvOt.store(st + 2 * X::KC_BYTES + X::KS_BYTES, tid);
    if (tid < 64) {
      float* f = reinterpret_cast<float*>(st + TILES);
      f[tid] = st_lse;
      f[64 + tid] = st_dot;
    }
  };

  const int nq = (s + 63) / 64;
  const int j0 = (kb * 128) / 64;                       // first query tile that sees these keys
  f32x16 dk[X::DT], dv[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.0f; dv[dt][v] = 0.0f; }
  const float sc = p.scale * LOG2E;

  load_tiles(j0 * 64);
  store_tiles(smem);
  __syncthreads();
  for (int j = j0; j < nq; ++j) {
    const uint8_t* st = smem + ((j - j0) & 1) * STAGE;
    const int q0 = j * 64;
    if (j + 1 < nq) load_tiles(q0 + 64);
    if (q0 + 63 >= kw0) {                                // some query of the tile sees this wave's keys
      f32x16 sm[2], dpm[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) { sm[t][v] = 0.0f; dpm[t][v] = 0.0f; }
      mma_tile_rows<D>(st, kf, fr, fh, sm);                        // S[q, kv]
      mma_tile_rows<D>(st + X::KC_BYTES, vf, fr, fh, dpm);         // dP[q, kv]
      const float* f_lse = reinterpret_cast<const float*>(st + TILES);
      const bool diag = q0 < kw0 + 31;
      f32x16 pm[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int r0 = 32 * t + 8 * g + 4 * fh;                  // 4 consecutive query rows
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(f_lse + r0);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(f_lse + 64 + r0);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int v = 4 * g + e;
            float pr = exp2f(sm[t][v] * sc - l4[e]);
            if (diag && q0 + r0 + e < kpos) pr = 0.0f;
            pm[t][v] = pr;
            sm[t][v] = pr * (dpm[t][v] - d4[e]);
          }
        }
      mma_tile_cols<D>(st + 2 * X::KC_BYTES + X::KS_BYTES, pm, fr, fh, dv);   // dV^T += dO^T P
      mma_tile_cols<D>(st + 2 * X::KC_BYTES, sm, fr, fh, dk);                 // dK^T += Q^T dS
    }
    if (j + 1 < nq) store_tiles(smem + ((j + 1 - j0) & 1) * STAGE);
    __syncthreads();
  }
  if (kpos < s) {
    bf16_t* out = static_cast<bf16_t*>(p.dqkv) + ((long)bi * s + kpos) * ld + hh * D;
    store_transposed<D>(dk, p.scale, out + hl, fh);
    store_transposed<D>(dv, 1.0f, out + 2 * hl, fh);
  }
}

template <class K>
hipError_t set_lds(K kern, int bytes, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done = true;
  return e;
}

template <int D>
hipError_t fwd_launch(const AttnArgs& a, hipStream_t st) {
  using X = Dims<D>;
  constexpr int LDS = 2 * (X::KC_BYTES + X::KS_BYTES);
  static bool done = false;
  hipError_t e = set_lds(attn_fwd_kernel<D>, LDS, done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_fwd_kernel<D>, dim3((a.seq + 127) / 128, a.heads, a.batch), dim3(256), LDS, st, a);
  return hipGetLastError();
}

template <int D>
hipError_t bwd_launch(const AttnArgs& a, hipStream_t st) {
  using X = Dims<D>;
  const long rows = (long)a.batch * a.seq;
  hipLaunchKernelGGL(attn_dot_kernel, dim3((unsigned)((rows * a.heads + 255) / 256)), dim3(256), 0, st,
                     static_cast<const bf16_t*>(a.ctx), static_cast<const bf16_t*>(a.dctx), a.ld_ctx, (int)rows, a.seq,
                     a.heads, D, a.dot);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr int LDS_Q = 2 * (2 * X::KC_BYTES + X::KS_BYTES);
  constexpr int LDS_KV = 2 * (2 * X::KC_BYTES + 2 * X::KS_BYTES + 512);
  static bool done_q = false, done_kv = false;
  if ((e = set_lds(attn_bwd_dq_kernel<D>, LDS_Q, done_q)) != hipSuccess) return e;
  if ((e = set_lds(attn_bwd_dkv_kernel<D>, LDS_KV, done_kv)) != hipSuccess) return e;
  const dim3 grid((a.seq + 127) / 128, a.heads, a.batch);
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<D>, grid, dim3(256), LDS_KV, st, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_kernel<D>, grid, dim3(256), LDS_Q, st, a);
  return hipGetLastError();
}

}  // namespace

hipError_t attention_fwd_launch(const AttnArgs& a, hipStream_t st) {
  switch (a.head_dim) {
    case 64: return fwd_launch<64>(a, st);
    case 80: return fwd_launch<80>(a, st);
    case 128: return fwd_launch<128>(a, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t attention_bwd_launch(const AttnArgs& a, hipStream_t st) {
  switch (a.head_dim) {
    case 64: return bwd_launch<64>(a, st);
    case 80: return bwd_launch<80>(a, st);
    case 128: return bwd_launch<128>(a, st);
    default: return hipErrorInvalidValue;
  }
}
