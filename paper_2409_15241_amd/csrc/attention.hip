// Causal flash-style attention for one head shard on gfx950 MFMA (Eq. 2, first case:
// softmax(Q K^T / sqrt(d_k)) V; kept as one fused kernel because the first weight group is never
// sliced, Sec. 3.1), forward and backward.
//
// All products are computed transposed so that the query (forward, dQ pass) or key (dK/dV pass)
// index of an MFMA accumulator is the LANE and the other index lives in the lane's 16 registers:
//   S^T[kv, q] = K Q^T          row statistics of a query are then a reduction over one lane's
//   O^T[d, q]  = V^T P^T        registers plus one exchange between the two lane halves, and the
// probabilities never leave registers: an accumulator converted to bf16 is directly the second
// operand of the next product, provided the first operand's contraction index is read in the
// accumulator's row order (the transposing LDS reads below take their rows in that order).
// Operand tiles travel HBM/L2 -> LDS with buffer_load ... lds, double buffered; see lds_dma.h.
//
// Backward is two passes without atomics (run-to-run identical results):
//   dQ pass, one workgroup per 128 queries: recompute P^T from the saved log-sum-exp,
//     dP^T = V dO^T, dS^T = P^T (dP^T - D), dQ^T += K^T dS^T.
//   dK/dV pass, one workgroup per 128 keys: P = exp(S - lse), dV^T += dO^T P, dP = dO V^T,
//     dS = P (dP - D), dK^T += Q^T dS.
// D[q] = sum_d dO[q,d] O[q,d] comes from a small pre-pass.
#include "attention.h"
#include "host_once.h"
#include "lds_dma.h"
#include <type_traits>

namespace {

// 2^x as the bare hardware instruction: the arguments here are differences to a running maximum or to the
// log-sum-exp (at most about 0; -inf for masked scores gives 0), where results below 2^-126 may flush to zero,
// so the range fix-up that the library's exp2f wraps around it (a compare, two selects and an ldexp per value)
// is dead weight on the vector ALUs that bound these kernels.
DEV float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

template <int D>
struct Dims {
  static constexpr int DT = (D + 31) / 32;             // 32-row d tiles of a transposed (d x position) product
  static constexpr int KSTEPS = D / 16;               // MFMA steps of a contraction over d
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

// The rotary embedding's transpose on out^T[d, pos]: the gradient with respect to a rotated q or k, taken back to
// the vector before the rotation.  The pair (i, i + D/2) of a position sits in one lane (accumulator rows 32 dt + 8 g
// + 4 fh + e: adding D/2 = 32, 40 or 64 changes dt and g only), so nothing crosses lanes.
template <int D>
DEV void rope_back(f32x16 (&o)[Dims<D>::DT], int pos, int fh, float log2_base) {
  constexpr int H = D / 2;
  const float fpos = (float)pos;
#pragma unroll
  for (int dt = 0; dt < Dims<D>::DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int dd0 = 32 * dt + 8 * g;               // this lane's rows of the group: dd0 + 4 fh + e
      if (dd0 < H) {
        const int dt2 = (dd0 + H) / 32, g2 = ((dd0 + H) % 32) / 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float sn, cs;
          rope_sincos(fpos, rope_freq(dd0 + 4 * fh + e, D, log2_base), &sn, &cs);
          const float lo = o[dt][4 * g + e], hi = o[dt2][4 * g2 + e];
          o[dt][4 * g + e] = lo * cs + hi * sn;
          o[dt2][4 * g2 + e] = hi * cs - lo * sn;
        }
      }
    }
}

// ------------------------------------------------------------------------------------- forward
// compile-time loop: f(std::integral_constant<int, I>) for I in [0, N)
template <int I, int N, class F>
DEV void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Work order.  Workgroups differ in length by the causal mask (2 to 2 s/64 tiles), and the hardware deals
// consecutive workgroup ids round-robin over the 8 XCDs: with a plain (block, head, batch) grid the workgroups
// whose block index is a multiple of 8 (the longest of every head) all land on one XCD, which then carries
// 2.4 times the work of the last one.  So the launch is a 1-D grid and the work items are ranked instead: rank
// = (position of the item inside its (batch, head) group, longest first) * groups + group, dealt over the XCDs
// in snake order (0..7, 7..0, ...): every XCD gets the same mix, longest items first.  Returns the item's
// position inside its group and the group, or false for the padding workgroups of the last round.
DEV bool ranked_item(int per_group, int groups, int& pos, int& group) {
  const int id = __builtin_amdgcn_readfirstlane(blockIdx.x);
  const int xcd = id & 7, round = id >> 3;
  const int rank = round * 8 + ((round & 1) ? 7 - xcd : xcd);
  if (rank >= per_group * groups) return false;
  pos = rank / groups;
  group = rank % groups;
  return true;
}
inline int ranked_grid(int per_group, int groups) { return ((per_group * groups + 7) / 8) * 8; }

// One workgroup = 128 queries of one (batch element, head): 4 waves x 32 queries.  K and V tiles of 64
// keys travel HBM/L2 -> LDS with buffer_load ... lds (double buffered, no VGPR staging): K as
// contraction-contiguous [kv][32 d] sub-tiles, V as row-major [32 kv][d] sub-tiles read back with the
// transposing LDS read in accumulator-row order, so P feeds P V straight from registers.
template <int D>
__global__ __launch_bounds__(256, 2)
void attn_fwd_kernel(const AttnArgs p) {
  using X = Dims<D>;
  constexpr int DS = (D + 31) / 32;                 // 32-wide d sub-tiles of K
  constexpr int K_BYTES = DS * 4096;                // [DS][64 kv][32 d]
  constexpr int V_BYTES = 2 * 8192;                 // [2][32 kv][128 d]
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int NB = (X::KSTEPS + 3) / 4;           // batches of up to 4 contraction steps over d
  extern __shared__ __align__(1024) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  const int s = p.seq;
  const int nqb = (s + 127) / 128;
  int pos, group;
  if (!ranked_item(nqb, p.heads * p.batch, pos, group)) return;
  const int qb = nqb - 1 - pos;                     // longest rows first
  const int hh = group % p.heads, bi = group / p.heads;
  const int qw0 = qb * 128 + wave * 32, qpos = qw0 + fr;
  const long ld = p.ld;
  const bf16_t* tok0 = static_cast<const bf16_t*>(p.qkv) + (long)bi * s * ld;
  const int hl = p.heads * D;
  const long view_bytes = ((long)(s - 1) * ld + D) * 2;
  const buf_rsrc rsK = make_rsrc(tok0 + hl + hh * D, view_bytes);
  const buf_rsrc rsV = make_rsrc(tok0 + 2 * hl + hh * D, view_bytes);

  bf16x8 qf[X::KSTEPS];
  load_row_frags<D>(tok0 + hh * D, ld, qpos, s, fh, qf);

  DmaLoader<64, 4, false> ldK;
  DmaLoader<128, 4, true> ldV;
  ldK.init_kc((int)ld, 0, 1 << 30, wave, lane);       // rows past the sequence end fall outside the extent
  ldV.init_ks((int)ld, IdentityCols{0, D}, wave, lane);
  auto issue_tile = [&](int j) {
    uint8_t* st = smem + (j & 1) * STAGE;
    const int kv0 = j * 64;
#pragma unroll
    for (int c = 0; c < DS; ++c) ldK.issue(rsK, st + c * 4096, c * 32, D, wave, (uint32_t)kv0 * (uint32_t)ld * 2u);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) ldV.issue(rsV, st + K_BYTES + h2 * 8192, kv0 + 32 * h2, 0, wave);
  };

  // per-lane LDS offsets: K fragment (row lane%32, chunk 2*step + lane/32) and V^T fragment rows d
  const uint32_t offK0 = kc_frag_off(lane, 0), offK1 = kc_frag_off(lane, 1);
  uint32_t offV[X::DT];
  {
    const int sl = lane & 15, nh = (lane >> 4) & 1;
    const int kr = 4 * fh + (sl >> 2);
#pragma unroll
    for (int dt = 0; dt < X::DT; ++dt)
      offV[dt] = (uint32_t)(kr * 256 + ((dt ^ (kr & 3)) << 6) + (16 * nh + 4 * (sl & 3)) * 2 + K_BYTES);
  }

  const int q_end = min(qb * 128 + 128, s);
  const int ntiles = (q_end + 63) / 64;
  f32x16 o[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.0f;
  float m = -INFINITY, l = 0.0f;
  const float sc = p.scale * LOG2E;
  const uint32_t smem_base = lds_addr(smem);

  issue_tile(0);
  for (int j = 0; j < ntiles; ++j) {
    wait_vmcnt<0>();                                  // tile j has landed (this wave's part)
    __builtin_amdgcn_s_barrier();                     // ... everybody's part; the other stage is free
    if (j + 1 < ntiles) issue_tile(j + 1);
    const int kv0 = j * 64;
    if (kv0 > qw0 + 31) continue;                     // every key of the tile is masked for this wave
    const uint32_t st = smem_base + (j & 1) * STAGE;

    // ---- S^T[kv, q] = K Q^T: batches of 4 contraction steps, next batch's reads in flight
    f32x16 sT[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) sT[t][v] = 0.0f;
    u32x4 kf[2][4][2];
    auto read_batch = [&](auto bb) {
      constexpr int B = decltype(bb)::value;
      static_for<0, 4>([&](auto kk) {
        constexpr int KS = B * 4 + decltype(kk)::value;
        if constexpr (KS < X::KSTEPS) {
          const uint32_t a = st + ((KS & 1) ? offK1 : offK0);
          kf[B & 1][decltype(kk)::value][0] = ds_read_b128_at<(KS >> 1) * 4096>(a);
          kf[B & 1][decltype(kk)::value][1] = ds_read_b128_at<(KS >> 1) * 4096 + 2048>(a);
        }
      });
    };
    read_batch(std::integral_constant<int, 0>{});
    static_for<0, NB>([&](auto bb) {
      constexpr int B = decltype(bb)::value;
      constexpr int NEXT = (B + 1 < NB) ? ((X::KSTEPS - 4 * (B + 1)) < 4 ? (X::KSTEPS - 4 * (B + 1)) : 4) * 2 : 0;
      if constexpr (B + 1 < NB) read_batch(std::integral_constant<int, B + 1>{});
      lds_wait<NEXT>();
      static_for<0, 4>([&](auto kk) {
        constexpr int KS = B * 4 + decltype(kk)::value;
        if constexpr (KS < X::KSTEPS) {
          tie(kf[B & 1][decltype(kk)::value][0]);
          tie(kf[B & 1][decltype(kk)::value][1]);
#pragma unroll
          for (int t = 0; t < 2; ++t)
            sT[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[B & 1][decltype(kk)::value][t]),
                                                            qf[KS], sT[t], 0, 0, 0);
        }
      });
    });

    // ---- online softmax; a lane owns one query (both lane halves: the two key halves of each 8)
    float mx = -INFINITY;
    if (kv0 + 63 > qw0) {                             // tile touches the diagonal: mask keys after the query
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          if (kv0 + 32 * t + acc_row(v, fh) > qpos) sT[t][v] = -INFINITY;
          mx = fmaxf(mx, sT[t][v]);
        }
    } else {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sT[t][v]);
    }
    mx = fmaxf(mx, other_half(mx)) * sc;       // scores scaled to the log2 domain (sc > 0)
    const float m_new = fmaxf(m, mx);                  // finite: key 0 is visible to every query
    if (__builtin_amdgcn_ballot_w64(m_new != m) != 0) {   // rescale only when some query's maximum moved
      const float alpha = exp2_raw(m - m_new);
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
      m = m_new;
    }
    float rs = 0.0f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float e = exp2_raw(sT[t][v] * sc - m);
        sT[t][v] = e;
        rs += e;
      }
    l += rs;
    bf16x8 pf[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const int t = s4 >> 1, u = s4 & 1;
      u32x4 w = {pack_bf16(sT[t][8 * u + 0], sT[t][8 * u + 1]), pack_bf16(sT[t][8 * u + 2], sT[t][8 * u + 3]),
                 pack_bf16(sT[t][8 * u + 4], sT[t][8 * u + 5]), pack_bf16(sT[t][8 * u + 6], sT[t][8 * u + 7])};
      pf[s4] = __builtin_bit_cast(bf16x8, w);
    }

    // ---- O^T[d, q] += V^T P^T, one 32-row d tile at a time, next tile's reads in flight
    u32x2 vf[2][4][2];
    auto read_v = [&](auto dd) {
      constexpr int DTI = decltype(dd)::value;
      static_for<0, 4>([&](auto ss) {
        constexpr int S4 = decltype(ss)::value;
        constexpr int OFF = (S4 >> 1) * 8192 + (S4 & 1) * 4096;
        vf[DTI & 1][S4][0] = ds_read_tr_at<OFF>(st + offV[DTI]);
        vf[DTI & 1][S4][1] = ds_read_tr_at<OFF + 2048>(st + offV[DTI]);
      });
    };
    read_v(std::integral_constant<int, 0>{});
    static_for<0, X::DT>([&](auto dd) {
      constexpr int DTI = decltype(dd)::value;
      if constexpr (DTI + 1 < X::DT) read_v(std::integral_constant<int, DTI + 1>{});
      lds_wait<(DTI + 1 < X::DT) ? 8 : 0>();
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        tie(vf[DTI & 1][s4][0]);
        tie(vf[DTI & 1][s4][1]);
        const u32x4 a = {vf[DTI & 1][s4][0][0], vf[DTI & 1][s4][0][1], vf[DTI & 1][s4][1][0], vf[DTI & 1][s4][1][1]};
        o[DTI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pf[s4], o[DTI], 0, 0, 0);
      }
    });
  }
  l += other_half(l);
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

// ------------------------------------------------------------------------------------- backward tiles
// Row-major LDS tile [64 positions][128 d] (16 KiB) filled by buffer_load ... lds, serving BOTH fragment
// kinds of one operand: the plain fragment (row = position, 8 consecutive d: ds_read_b128) and the
// transposed fragment (row = d, contraction over positions in accumulator-row order: two
// ds_read_b64_tr_b16).  16-byte chunk c of row r lives at r*256 + ((c ^ rm_swz(r)) << 4): the 16 rows of a
// plain read hit 16 distinct chunk positions, and the 4 rows x 2 column groups of a transposing
// read hit 8 distinct 32-byte pairs.
DEV int rm_swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

struct RmLoader {            // 4 waves x 4 one-KiB pieces (4 rows each)
  uint32_t base[4];
  DEV void init(int ld, int d_valid, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 4 * (wave * 4 + i) + (lane >> 4);
      const int d = ((lane & 15) ^ rm_swz(row)) * 8;
      base[i] = d < d_valid ? (uint32_t)(row * ld + d) * 2u : BUF_OOB;
    }
  }
  DEV void issue(buf_rsrc rs, uint8_t* tile, uint32_t row_byte_off, int wave) const {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, LDS_PTR(tile + (wave * 4 + i) * 1024), 16, base[i] + row_byte_off, 0, 0, 0);
  }
};
// per-lane byte offset of the plain fragment (row lane%32, chunk lane/32) at contraction step 0; step ks
// is reached by XOR (ks << 5), the second 32-row group by + 8192
DEV uint32_t rm_plain_off(int lane) {
  const int fr = lane & 31, fh = lane >> 5;
  return (uint32_t)(fr * 256 + ((fh ^ rm_swz(fr)) << 4));
}
// per-lane byte offset of the first transposing read of the transposed fragment (d tile 0); d tile dt and
// the second read are reached by XOR ((4 dt) ^ (2 second)) << 4; + 4096 u + 8192 sub + 2048 second
DEV uint32_t rm_trans_off(int lane) {
  const int sl = lane & 15, nh = (lane >> 4) & 1, fh = lane >> 5;
  const int posl = 4 * fh + (sl >> 2);
  const int h = (2 * nh + ((sl & 3) >> 1)) ^ rm_swz(posl);
  return (uint32_t)(posl * 256 + (h << 4) + 8 * (sl & 1));
}

// acc[t] += Tile[32 t + lane%32, d] * frag[d, lane] over all d, batches of 4 steps with the next batch's
// reads in flight.  tile_addr = LDS byte address of the row-major tile, off = rm_plain_off(lane).
template <int D>
DEV void rm_mma_rows(uint32_t tile_addr, uint32_t off, const bf16x8 (&f)[Dims<D>::KSTEPS], f32x16 (&acc)[2]) {
  using X = Dims<D>;
  constexpr int NB = (X::KSTEPS + 3) / 4;
  u32x4 fr[2][4][2];
  auto read_batch = [&](auto bb) {
    constexpr int B = decltype(bb)::value;
    static_for<0, 4>([&](auto kk) {
      constexpr int KS = B * 4 + decltype(kk)::value;
      if constexpr (KS < X::KSTEPS) {
        const uint32_t a = tile_addr + (off ^ (KS << 5));
        fr[B & 1][decltype(kk)::value][0] = ds_read_b128_at<0>(a);
        fr[B & 1][decltype(kk)::value][1] = ds_read_b128_at<8192>(a);
      }
    });
  };
  read_batch(std::integral_constant<int, 0>{});
  static_for<0, NB>([&](auto bb) {
    constexpr int B = decltype(bb)::value;
    constexpr int LEFT = X::KSTEPS - 4 * (B + 1);
    constexpr int NEXT = (B + 1 < NB) ? (LEFT < 4 ? LEFT : 4) * 2 : 0;
    if constexpr (B + 1 < NB) read_batch(std::integral_constant<int, B + 1>{});
    lds_wait<NEXT>();
    static_for<0, 4>([&](auto kk) {
      constexpr int KS = B * 4 + decltype(kk)::value;
      if constexpr (KS < X::KSTEPS) {
        tie(fr[B & 1][decltype(kk)::value][0]);
        tie(fr[B & 1][decltype(kk)::value][1]);
#pragma unroll
        for (int t = 0; t < 2; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr[B & 1][decltype(kk)::value][t]),
                                                          f[KS], acc[t], 0, 0, 0);
      }
    });
  });
}

// States that the running sums sit in the accumulation registers at this point.  Placed at the top of a pass's
// loop it keeps them there across the back edge; without it the register allocator carried all of them in
// vector registers at the loop head and copied them to the accumulation registers and back around every tile.
template <int N>
DEV void pin_acc(f32x16 (&acc)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+a"(acc[i]));
}

// Two accumulators covering a tile's 64 positions, rounded to bf16 as the second operand of rm_mma_cols:
// fragment s4 = 2 t + u holds accumulator t's values 8 u .. 8 u + 7.
DEV void pack_acc_pair(const f32x16 (&vals)[2], bf16x8 (&pf)[4]) {
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    const int t = s4 >> 1, u = s4 & 1;
    u32x4 w = {pack_bf16(vals[t][8 * u + 0], vals[t][8 * u + 1]), pack_bf16(vals[t][8 * u + 2], vals[t][8 * u + 3]),
               pack_bf16(vals[t][8 * u + 4], vals[t][8 * u + 5]), pack_bf16(vals[t][8 * u + 6], vals[t][8 * u + 7])};
    pf[s4] = __builtin_bit_cast(bf16x8, w);
  }
}

// out[dt] += TileT[32 dt + lane%32, pos] * pf[pos, lane]: pf = packed values covering the tile's 64
// positions (see pack_acc_pair); off = rm_trans_off(lane).
template <int D>
DEV void rm_mma_cols(uint32_t tile_addr, uint32_t off, const bf16x8 (&pf)[4], f32x16 (&out)[Dims<D>::DT]) {
  using X = Dims<D>;
  u32x2 vf[2][4][2];
  auto read_v = [&](auto dd) {
    constexpr int DTI = decltype(dd)::value;
    static_for<0, 4>([&](auto ss) {
      constexpr int S4 = decltype(ss)::value;
      constexpr int OFF = (S4 >> 1) * 8192 + (S4 & 1) * 4096;
      vf[DTI & 1][S4][0] = ds_read_tr_at<OFF>(tile_addr + (off ^ ((4 * DTI) << 4)));
      vf[DTI & 1][S4][1] = ds_read_tr_at<OFF + 2048>(tile_addr + (off ^ (((4 * DTI) ^ 2) << 4)));
    });
  };
  read_v(std::integral_constant<int, 0>{});
  static_for<0, X::DT>([&](auto dd) {
    constexpr int DTI = decltype(dd)::value;
    if constexpr (DTI + 1 < X::DT) read_v(std::integral_constant<int, DTI + 1>{});
    lds_wait<(DTI + 1 < X::DT) ? 8 : 0>();
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      tie(vf[DTI & 1][s4][0]);
      tie(vf[DTI & 1][s4][1]);
      const u32x4 a = {vf[DTI & 1][s4][0][0], vf[DTI & 1][s4][0][1], vf[DTI & 1][s4][1][0], vf[DTI & 1][s4][1][1]};
      out[DTI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pf[s4], out[DTI], 0, 0, 0);
    }
  });
}

constexpr int RM_TILE = 16384;

// ------------------------------------------------------------------------------------- dQ pass
template <int D>
DEV void attn_bwd_dq_body(const AttnArgs& p, uint8_t* smem, int qb, int hh, int bi) {
  using X = Dims<D>;
  constexpr int STAGE = 2 * RM_TILE;                      // K tile, V tile (64 keys each)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
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

  RmLoader ldr;
  ldr.init((int)ld, D, wave, lane);
  auto issue_tile = [&](int j) {
    uint8_t* st = smem + (j & 1) * STAGE;
    const uint32_t ro = (uint32_t)(j * 64) * (uint32_t)ld * 2u;
    ldr.issue(rsK, st, ro, wave);
    ldr.issue(rsV, st + RM_TILE, ro, wave);
  };
  const uint32_t offP = rm_plain_off(lane), offT = rm_trans_off(lane);

  const int q_end = min(qb * 128 + 128, s);
  const int ntiles = (q_end + 63) / 64;
  f32x16 dq[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[dt][v] = 0.0f;
  const float sc = p.scale * LOG2E;
  const uint32_t smem_base = lds_addr(smem);

  issue_tile(0);
  for (int j = 0; j < ntiles; ++j) {
    pin_acc(dq);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (j + 1 < ntiles) issue_tile(j + 1);
    const int kv0 = j * 64;
    if (kv0 > qw0 + 31) continue;
    const uint32_t st = smem_base + (j & 1) * STAGE;
    f32x16 sT[2], dpT[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) { sT[t][v] = 0.0f; dpT[t][v] = 0.0f; }
    rm_mma_rows<D>(st, offP, qf, sT);                    // S^T  = K Q^T
    rm_mma_rows<D>(st + RM_TILE, offP, dof, dpT);        // dP^T = V dO^T
    auto probs = [&](auto masked) {                       // the mask arithmetic only where the tile meets the diagonal
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float pr = exp2_raw(sT[t][v] * sc - lse2);
          if (decltype(masked)::value && kv0 + 32 * t + acc_row(v, fh) > qpos) pr = 0.0f;
          sT[t][v] = pr * (dpT[t][v] - dq_dot);
        }
    };
    if (kv0 + 63 > qw0) probs(std::true_type{}); else probs(std::false_type{});
    bf16x8 dsf[4];
    pack_acc_pair(sT, dsf);
    rm_mma_cols<D>(st, offT, dsf, dq);                   // dQ^T += K^T dS^T
  }
  if (qpos < s) {
    bf16_t* out = static_cast<bf16_t*>(p.dqkv) + ((long)bi * s + qpos) * ld + hh * D;
    if (p.rope) rope_back<D>(dq, qpos, fh, p.rope_log2_base);
    store_transposed<D>(dq, p.scale, out, fh);
  }
}

// ------------------------------------------------------------------------------------- dK / dV pass
template <int D>
DEV void attn_bwd_dkv_body(const AttnArgs& p, uint8_t* smem, int kb, int hh, int bi) {
  using X = Dims<D>;
  constexpr int STAGE = 2 * RM_TILE + 512;                // Q tile, dO tile (64 queries), lse[64], dot[64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  const int s = p.seq;                            // 128 keys per workgroup
  const int kw0 = kb * 128 + wave * 32, kpos = kw0 + fr;
  const long ld = p.ld, ldc = p.ld_ctx;
  const bf16_t* tok0 = static_cast<const bf16_t*>(p.qkv) + (long)bi * s * ld;
  const bf16_t* do0 = static_cast<const bf16_t*>(p.dctx) + (long)bi * s * ldc + hh * D;
  const int hl = p.heads * D;
  const buf_rsrc rsQ = make_rsrc(tok0 + hh * D, ((long)(s - 1) * ld + D) * 2);
  const buf_rsrc rsO = make_rsrc(do0, ((long)(s - 1) * ldc + D) * 2);
  const long stat0 = ((long)bi * p.heads + hh) * s;
  const buf_rsrc rsL = make_rsrc(p.lse + stat0, (long)s * 4);   // rows past the end read as 0: harmless, their
  const buf_rsrc rsD = make_rsrc(p.dot + stat0, (long)s * 4);   // Q and dO rows are zero as well

  bf16x8 kf[X::KSTEPS], vf[X::KSTEPS];
  load_row_frags<D>(tok0 + hl + hh * D, ld, kpos, s, fh, kf);
  load_row_frags<D>(tok0 + 2 * hl + hh * D, ld, kpos, s, fh, vf);

  RmLoader ldq, ldo;
  ldq.init((int)ld, D, wave, lane);
  ldo.init((int)ldc, D, wave, lane);
  auto issue_tile = [&](int j, int slot) {
    uint8_t* st = smem + slot * STAGE;
    ldq.issue(rsQ, st, (uint32_t)(j * 64) * (uint32_t)ld * 2u, wave);
    ldo.issue(rsO, st + RM_TILE, (uint32_t)(j * 64) * (uint32_t)ldc * 2u, wave);
    if (wave == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsL, LDS_PTR(st + 2 * RM_TILE), 4, (uint32_t)(j * 64 + lane) * 4u, 0, 0, 0);
    if (wave == 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsD, LDS_PTR(st + 2 * RM_TILE + 256), 4, (uint32_t)(j * 64 + lane) * 4u, 0, 0, 0);
  };
  const uint32_t offP = rm_plain_off(lane), offT = rm_trans_off(lane);

  const int nq = (s + 63) / 64;
  const int j0 = (kb * 128) / 64;                         // first query tile that sees these keys
  f32x16 dk[X::DT], dv[X::DT];
#pragma unroll
  for (int dt = 0; dt < X::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.0f; dv[dt][v] = 0.0f; }
  const float sc = p.scale * LOG2E;
  const uint32_t smem_base = lds_addr(smem);

  issue_tile(j0, 0);
  for (int j = j0; j < nq; ++j) {
    pin_acc(dk);
    pin_acc(dv);
    const int slot = (j - j0) & 1;
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (j + 1 < nq) issue_tile(j + 1, slot ^ 1);
    const int q0 = j * 64;
    if (q0 + 63 < kw0) continue;                          // no query of the tile sees this wave's keys
    const uint32_t st = smem_base + slot * STAGE;
    f32x16 sm[2], dpm[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) { sm[t][v] = 0.0f; dpm[t][v] = 0.0f; }
    rm_mma_rows<D>(st, offP, kf, sm);                     // S[q, kv]  = Q K^T
    rm_mma_rows<D>(st + RM_TILE, offP, vf, dpm);          // dP[q, kv] = dO V^T
    u32x4 pw[4], dw[4];                                   // P and dS rounded to bf16 as they are formed
    auto probs = [&](auto masked) {                       // the mask arithmetic only where the tile meets the diagonal
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      u32x4 l4[4], d4[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {                       // 4 consecutive query rows 32 t + 8 g + 4 fh ..
        const uint32_t a = st + 2 * RM_TILE + (uint32_t)(32 * t + 8 * g + 4 * fh) * 4u;
        l4[g] = ds_read_b128_at<0>(a);
        d4[g] = ds_read_b128_at<256>(a);
      }
      lds_wait<0>();
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        tie(l4[g]);
        tie(d4[g]);
        const f32x4 lf = __builtin_bit_cast(f32x4, l4[g]), df = __builtin_bit_cast(f32x4, d4[g]);
        float pr[4], ds[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * g + e;
          pr[e] = exp2_raw(sm[t][v] * sc - lf[e] * LOG2E);
          if (decltype(masked)::value && q0 + 32 * t + 8 * g + 4 * fh + e < kpos) pr[e] = 0.0f;
          ds[e] = pr[e] * (dpm[t][v] - df[e]);
        }
        // values 4 g .. 4 g + 3 of accumulator t are words 2 (g & 1), 2 (g & 1) + 1 of fragment 2 t + (g >> 1)
        pw[2 * t + (g >> 1)][2 * (g & 1)] = pack_bf16(pr[0], pr[1]);
        pw[2 * t + (g >> 1)][2 * (g & 1) + 1] = pack_bf16(pr[2], pr[3]);
        dw[2 * t + (g >> 1)][2 * (g & 1)] = pack_bf16(ds[0], ds[1]);
        dw[2 * t + (g >> 1)][2 * (g & 1) + 1] = pack_bf16(ds[2], ds[3]);
      }
    }
    };
    if (q0 < kw0 + 31) probs(std::true_type{}); else probs(std::false_type{});
    bf16x8 pf[4], dsf[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) { pf[s4] = __builtin_bit_cast(bf16x8, pw[s4]); dsf[s4] = __builtin_bit_cast(bf16x8, dw[s4]); }
    rm_mma_cols<D>(st + RM_TILE, offT, pf, dv);           // dV^T += dO^T P
    rm_mma_cols<D>(st, offT, dsf, dk);                    // dK^T += Q^T dS
  }
  if (kpos < s) {
    bf16_t* out = static_cast<bf16_t*>(p.dqkv) + ((long)bi * s + kpos) * ld + hh * D;
    if (p.rope) rope_back<D>(dk, kpos, fh, p.rope_log2_base);
    store_transposed<D>(dk, p.scale, out + hl, fh);
    store_transposed<D>(dv, 1.0f, out + 2 * hl, fh);
  }
}


// Both backward passes in one launch (they are independent given D, so one launch puts twice as many
// workgroups on the chip and the attention backward leaves its slice's critical path sooner).  Inside a
// (batch, head) group the items alternate, longest first: dK/dV pass of key block 0, dQ pass of the last query
// block, dK/dV pass of key block 1, ...
template <int D>
__global__ __launch_bounds__(256)
void attn_bwd_kernel(const AttnArgs p) {
  extern __shared__ __align__(1024) uint8_t smem[];
  const int nxb = (p.seq + 127) / 128;
  int pos, group;
  if (!ranked_item(2 * nxb, p.heads * p.batch, pos, group)) return;
  const int hh = group % p.heads, bi = group / p.heads;
  if (pos & 1) attn_bwd_dq_body<D>(p, smem, nxb - 1 - (pos >> 1), hh, bi);
  else attn_bwd_dkv_body<D>(p, smem, pos >> 1, hh, bi);
}


template <int D>
hipError_t fwd_launch(const AttnArgs& a, hipStream_t st) {
  constexpr int LDS = 2 * (((D + 31) / 32) * 4096 + 2 * 8192);
  static LdsLimitOnce lds_limit;
  hipError_t e = lds_limit.ensure(reinterpret_cast<const void*>(attn_fwd_kernel<D>), LDS);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_fwd_kernel<D>, dim3(ranked_grid((a.seq + 127) / 128, a.heads * a.batch)), dim3(256), LDS, st, a);
  return hipGetLastError();
}

template <int D>
hipError_t bwd_launch(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.batch * a.seq;
  hipLaunchKernelGGL(attn_dot_kernel, dim3((unsigned)((rows * a.heads + 255) / 256)), dim3(256), 0, st,
                     static_cast<const bf16_t*>(a.ctx), static_cast<const bf16_t*>(a.dctx), a.ld_ctx, (int)rows, a.seq,
                     a.heads, D, a.dot);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr int LDS = 2 * (2 * RM_TILE + 512);             // the larger of the two passes' needs
  static LdsLimitOnce lds_limit;
  if ((e = lds_limit.ensure(reinterpret_cast<const void*>(attn_bwd_kernel<D>), LDS)) != hipSuccess) return e;
  const dim3 grid(ranked_grid(2 * ((a.seq + 127) / 128), a.heads * a.batch));
  hipLaunchKernelGGL(attn_bwd_kernel<D>, grid, dim3(256), LDS, st, a);
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
