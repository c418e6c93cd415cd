// bf16 MFMA GEMM for gfx950 with fused epilogues: the products of Eq. 1-4 (X*A, (XA)*B_j) and the
// two products of every "grad matmul" (Sec. 4.1.2: input gradient and weight gradient).
//
//   C[m][n] = epilogue( sum_k Aop(m,k) * Bop(k,n) ),  fp32 accumulation in MFMA 32x32x16.
//
// Each operand is either contraction-contiguous in memory (KC: [row][k]) or contraction-strided
// (KS: [k][row]); see lds_dma.h.  The three products of a linear layer map to
//   forward   X[M,K]   * W[K,N]            : A KC, B KS
//   dgrad     dY[M,N'] * W[K',N']^T        : A KC, B KC   (contraction over N')
//   wgrad     X[M',K']^T * dY[M',N]        : A KS, B KS   (contraction over the tokens M')
//
// Work decomposition: one workgroup per BM x BN tile of C, (BM/WM)*(BN/WN) waves, each owning a
// WM x WN sub-tile as (WN/32) x (WM/32) MFMA accumulators.  Operand tiles of 32 contraction elements
// travel HBM/L2 -> LDS with buffer_load ... lds through a ring of NST stages: while the MFMAs consume
// stage kt, the loads of tiles kt+1 .. kt+NST-1 are in flight.  One s_waitcnt vmcnt + one barrier per
// tile; no VGPR staging, no ds_write.
// The MFMA is issued with the roles swapped (first operand = B fragment) so that a lane ends up
// with 4 consecutive n for one m: 8-byte bf16 / 16-byte fp32 stores.
#include "gemm.h"
#include <cmath>
#include "host_once.h"
#include "lds_dma.h"
#include <type_traits>

namespace {

constexpr int NST = 4;   // LDS ring depth

template <int BM, int BN, int WM, int WN, bool AKS, bool BKS, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64)
void gemm_kernel(const GemmArgs p) {
  constexpr int NW = (BM / WM) * (BN / WN);
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_BYTES = BM * DMA_BK * 2, B_BYTES = BN * DMA_BK * 2;
  constexpr int STAGE = A_BYTES + B_BYTES;
  extern __shared__ __align__(1024) uint8_t smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave % (BM / WM)) * WM, wn0 = (wave / (BM / WM)) * WN;

  // Consecutive workgroup ids land on different XCDs (each with its own L2): with m fastest, the
  // tiles of one XCD share few A panels and walk the B panels in step.
  int tm, tn;
  if (p.group_m == 0) {
    const int tile = blockIdx.x;
    tm = tile % p.tiles_m; tn = tile / p.tiles_m;
  } else {
    // workgroup ids go round-robin over the 8 XCDs: give each XCD one contiguous chunk of a tile order
    // that walks bands of group_m tile rows, so the tiles sharing an L2 share operand panels
    const int T = p.tiles_m * p.tiles_n, chunk = (T + 7) >> 3;
    const int lin = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
    if (lin >= T) return;
    const int band = lin / (p.group_m * p.tiles_n), r = lin % (p.group_m * p.tiles_n);
    const int gm = min(p.group_m, p.tiles_m - band * p.group_m);
    tm = band * p.group_m + r % gm; tn = r / gm;
  }
  const int m0 = tm * BM, n0 = tn * BN;

  const buf_rsrc A = make_rsrc(p.A, p.a_bytes);
  const buf_rsrc B = make_rsrc(p.B, p.b_bytes);

  // SwiGLU forward: the tile's even 32-column groups are gate columns, the odd ones the matching
  // up columns, so one lane sees gate and up of the same ffn column.
  struct GluCols {
    int c0, n_split;
    DEV int operator()(int r) const {
      int col = c0 + ((r >> 6) << 5) + (r & 31);
      if (col >= n_split) return -1;
      return col + ((r >> 5) & 1) * n_split;
    }
  };

  // Rotary embedding: the partner columns (i, i + d/2) of a head must meet in one lane of the epilogue, which pairs
  // tile columns 32 apart inside a wave's 64 columns (as for SwiGLU).  Heads of 64 columns already lie that way; for
  // heads of 128 the tile's second and third group of 32 inside every 128 trade places.
  struct RopeCols {
    int n0, n_end, d;
    DEV int perm(int r) const {
      return d == 128 ? ((r & ~96) | (((r >> 5) & 1) << 6) | (((r >> 6) & 1) << 5)) : r;
    }
    DEV int operator()(int r) const { const int g = n0 + perm(r); return g < n_end ? g : -1; }
  };

  DmaLoader<BM, NW, AKS> ldA;
  DmaLoader<BN, NW, BKS> ldB;
  if constexpr (AKS) ldA.init_ks((int)p.lda, IdentityCols{m0, p.M}, wave, lane);
  else ldA.init_kc((int)p.lda, m0, p.M, wave, lane);
  if constexpr (BKS) {
    if constexpr (EPI == EPI_SWIGLU) ldB.init_ks((int)p.ldb, GluCols{tn * (BN / 2), p.n_split}, wave, lane);
    else if constexpr (EPI == EPI_ROPE) ldB.init_ks((int)p.ldb, RopeCols{n0, p.N, p.rope_d}, wave, lane);
    else ldB.init_ks((int)p.ldb, IdentityCols{n0, p.N}, wave, lane);
  } else {
    ldB.init_kc((int)p.ldb, n0, p.N, wave, lane);
  }
  auto issue_tile = [&](int t) {          // tiles past the end read out of bounds and store zeros
    uint8_t* st = smem + (t % NST) * STAGE;
    ldA.issue(A, st, t * DMA_BK, p.K, wave);
    ldB.issue(B, st + A_BYTES, t * DMA_BK, p.K, wave);
  };
  constexpr int LOADS_PER_TILE = DmaLoader<BM, NW, AKS>::IPW + DmaLoader<BN, NW, BKS>::IPW;

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // per-lane LDS byte offsets of the fragments inside a stage, for the two 16-deep MFMA steps of a tile
  uint32_t offA[2][AKS ? TM : 1], offB[2][BKS ? TN : 1];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    if constexpr (AKS) {
#pragma unroll
      for (int j = 0; j < TM; ++j) offA[ks][j] = ks_frag_off<BM>(lane, ks, (wm0 >> 5) + j);
    } else {
      offA[ks][0] = kc_frag_off(lane, ks) + wm0 * 64;
    }
    if constexpr (BKS) {
#pragma unroll
      for (int i = 0; i < TN; ++i) offB[ks][i] = ks_frag_off<BN>(lane, ks, (wn0 >> 5) + i) + A_BYTES;
    } else {
      offB[ks][0] = kc_frag_off(lane, ks) + wn0 * 64 + A_BYTES;
    }
  }

  const int nk = (p.K + DMA_BK - 1) / DMA_BK;
#pragma unroll
  for (int t = 0; t < NST - 1; ++t) issue_tile(t);

  const uint32_t smem_base = lds_addr(smem);
  const int fr = lane & 31, fh = lane >> 5;
  constexpr int STEP_READS = (AKS ? 2 * TM : TM) + (BKS ? 2 * TN : TN);
  static_assert(STEP_READS <= 15, "lgkmcnt is a 4-bit counter");
  u32x4 fa[2][TM], fb[2][TN];
  // fragments of MFMA step ks (16 contraction elements) of the stage at LDS address st
  auto read_step = [&](auto ks_c, uint32_t st) {
    constexpr int ks = decltype(ks_c)::value;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      if constexpr (AKS) {
        const u32x2 lo = ds_read_tr_at<0>(st + offA[ks][j]), hi = ds_read_tr_at<8 * BM>(st + offA[ks][j]);
        fa[ks][j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      } else {
        fa[ks][j] = (j == 0) ? ds_read_b128_at<0>(st + offA[ks][0]) : (j == 1) ? ds_read_b128_at<2048>(st + offA[ks][0])
                  : (j == 2) ? ds_read_b128_at<4096>(st + offA[ks][0]) : ds_read_b128_at<6144>(st + offA[ks][0]);
      }
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      if constexpr (BKS) {
        const u32x2 lo = ds_read_tr_at<0>(st + offB[ks][i]), hi = ds_read_tr_at<8 * BN>(st + offB[ks][i]);
        fb[ks][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      } else {
        fb[ks][i] = (i == 0) ? ds_read_b128_at<0>(st + offB[ks][0]) : (i == 1) ? ds_read_b128_at<2048>(st + offB[ks][0])
                  : (i == 2) ? ds_read_b128_at<4096>(st + offB[ks][0]) : ds_read_b128_at<6144>(st + offB[ks][0]);
      }
    }
  };
  // The MFMAs of step ks.  LDS returns in order, so after lgkmcnt(STEP_READS) only the younger step's
  // reads may be outstanding.  The empty asm statements "use and define" the fragments so that no MFMA
  // can be scheduled above the wait.
  auto mma_step = [&](auto ks_c) {
    constexpr int ks = decltype(ks_c)::value;
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(STEP_READS) : "memory");
#pragma unroll
    for (int j = 0; j < TM; ++j) asm volatile("" : "+v"(fa[ks][j]));
#pragma unroll
    for (int i = 0; i < TN; ++i) asm volatile("" : "+v"(fb[ks][i]));
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[ks][i]),
                                                            __builtin_bit_cast(bf16x8, fa[ks][j]), acc[i][j], 0, 0, 0);
  };
  using step0 = std::integral_constant<int, 0>;
  using step1 = std::integral_constant<int, 1>;

  // Software pipeline over the 16-deep MFMA steps: the LDS reads of a step are in flight while the
  // MFMAs of the step before run, across the tile boundary too (tile kt+1 must therefore have landed
  // by the middle of tile kt: one tile less of HBM/L2 prefetch distance than the ring depth).
  wait_vmcnt<(NST - 2) * LOADS_PER_TILE>();
  __builtin_amdgcn_s_barrier();
  read_step(step0{}, smem_base);
  for (int kt = 0; kt < nk; ++kt) {
    read_step(step1{}, smem_base + (kt % NST) * STAGE);
    mma_step(step0{});
    wait_vmcnt<(NST - 3) * LOADS_PER_TILE>();      // tile kt+1 has landed (this wave's share)
    __builtin_amdgcn_s_barrier();                  // ... everybody's; and nobody reads stage (kt-1)%NST any more
    issue_tile(kt + NST - 1);
    read_step(step0{}, smem_base + ((kt + 1) % NST) * STAGE);
    mma_step(step1{});
  }
  wait_vmcnt<0>();     // the zero-fill loads issued past the last tile must land before the LDS is released
  // The last iteration's look-ahead reads are still in flight: they must land in their registers
  // before the epilogue may reuse those registers.
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int j = 0; j < TM; ++j) asm volatile("" : "+v"(fa[0][j]));
#pragma unroll
  for (int i = 0; i < TN; ++i) asm volatile("" : "+v"(fb[0][i]));

  // ---- epilogue.  Accumulator (i, j) value v of a lane is C[m][n] with
  //      m = m0 + wm0 + 32 j + lane%32,  n = n0 + wn0 + 32 i + 8 (v/4) + 4 (lane/32) + v%4,
  // i.e. a lane owns one row: stored from there, every instruction would touch 32 rows with 16 bytes
  // each.  Each wave therefore turns its 32 x WN blocks through its own piece of the (now free) LDS:
  // written by row owner, read back with WN/4 consecutive lanes along a row, so that loads of the side
  // tensors and all stores cover whole 128-byte lines.
  __builtin_amdgcn_s_barrier();                  // every wave has finished reading the operand stages
  constexpr int ROWB = WN * 4 + 16;              // padded row: the 16 rows of a write phase hit distinct banks
  constexpr int LPR = WN / 4;                    // lanes per row when reading back
  constexpr int RPI = 64 / LPR;                  // rows per read instruction
  uint8_t* wbuf = smem + wave * (32 * ROWB);
  const int rrow = lane / LPR, rcol = (lane % LPR) * 4;
  const bool tanh_form = p.gelu_tanh != 0;
  constexpr int NT_ROWS = 32 / RPI;              // read-back instructions per 32-row block

  // what depends on the lane's 4 columns only
  const int nl = wn0 + rcol;                     // tile-local column of the first of this lane's 4
  int n, col = 0;                                // global column; SwiGLU: ffn column of the gate / up pair
  bool n_ok;
  if constexpr (EPI == EPI_SWIGLU) {
    col = tn * (BN / 2) + ((nl >> 6) << 5) + (nl & 31);
    n = col;
    n_ok = !((nl >> 5) & 1) && col < p.n_split;  // up groups are handled by the lane holding their gate group
  } else if constexpr (EPI == EPI_ROPE) {
    static_assert(EPI != EPI_ROPE || WN == 64, "the rotary epilogue pairs columns inside 64-column wave blocks");
    n = n0 + RopeCols{n0, p.N, p.rope_d}.perm(nl);            // memory column of the first element of the pair
    n_ok = !((nl >> 5) & 1) && n < p.N;                        // the partner groups are handled by the lane holding i
  } else {
    n = n0 + nl;
    n_ok = n < p.N;
  }
  // rotary embedding: the frequencies of this lane's 4 pair indices
  [[maybe_unused]] float rfreq[4];
  [[maybe_unused]] bool rot = false;
  if constexpr (EPI == EPI_ROPE) {
    rot = n_ok && n < p.rope_cols;
#pragma unroll
    for (int e = 0; e < 4; ++e) rfreq[e] = rot ? rope_freq(n % p.rope_d + e, p.rope_d, p.rope_log2_base) : 0.0f;
  }
  f32x4 bias4 = {0.0f, 0.0f, 0.0f, 0.0f};
  if constexpr (EPI == EPI_STORE || EPI == EPI_BIAS_GELU) {
    if (p.bias && n_ok) {
      const u32x2 bb = *reinterpret_cast<const u32x2*>(static_cast<const bf16_t*>(p.bias) + n);
      bias4 = f32x4{bf16_lo(bb[0]), bf16_hi(bb[0]), bf16_lo(bb[1]), bf16_hi(bb[1])};
    }
  }

#pragma unroll
  for (int j = 0; j < TM; ++j) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        *reinterpret_cast<f32x4*>(wbuf + fr * ROWB + (i * 32 + g * 8 + fh * 4) * 4) = v;
      }
    // phase 1: every load of the block (LDS read-back and side tensors) is issued before any is used; rows or
    // columns outside the matrix read a safe address instead of branching, their results are never stored
    f32x4 v[NT_ROWS], u[(EPI == EPI_SWIGLU || EPI == EPI_ROPE) ? NT_ROWS : 1], old[EPI == EPI_ACC_F32 ? NT_ROWS : 1];
    u32x2 sa[(EPI == EPI_DGELU || EPI == EPI_DSWIGLU) ? NT_ROWS : 1], sb[EPI == EPI_DSWIGLU ? NT_ROWS : 1];
    bool ok[NT_ROWS];
    long mrow[NT_ROWS];
#pragma unroll
    for (int t = 0; t < NT_ROWS; ++t) {
      const int row = t * RPI + rrow;
      const int m = m0 + wm0 + j * 32 + row;
      ok[t] = n_ok && m < p.M;
      mrow[t] = ok[t] ? (long)m : 0L;
      v[t] = *reinterpret_cast<const f32x4*>(wbuf + row * ROWB + rcol * 4);
      if constexpr (EPI == EPI_SWIGLU || EPI == EPI_ROPE) u[t] = *reinterpret_cast<const f32x4*>(wbuf + row * ROWB + ((rcol + 32) % WN) * 4);
      const int ns = ok[t] ? n : 0;
      if constexpr (EPI == EPI_ACC_F32) {
        if (p.beta) old[t] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.C) + mrow[t] * p.ldc + ns);
      } else if constexpr (EPI == EPI_DGELU) {
        sa[t] = *reinterpret_cast<const u32x2*>(static_cast<const bf16_t*>(p.aux) + mrow[t] * p.ldaux + ns);
      } else if constexpr (EPI == EPI_DSWIGLU) {
        const bf16_t* aux = static_cast<const bf16_t*>(p.aux) + mrow[t] * p.ldaux;
        sa[t] = *reinterpret_cast<const u32x2*>(aux + ns);
        sb[t] = *reinterpret_cast<const u32x2*>(aux + p.n_split + ns);
      }
    }
    // phase 2: arithmetic and stores
#pragma unroll
    for (int t = 0; t < NT_ROWS; ++t) {
      f32x4 w = v[t];
      if constexpr (EPI == EPI_SWIGLU) {
        if (ok[t]) {
          bf16_t* aux = static_cast<bf16_t*>(p.aux) + mrow[t] * p.ldaux;
          const u32x2 pg = {pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3])};
          const u32x2 pu = {pack_bf16(u[t][0], u[t][1]), pack_bf16(u[t][2], u[t][3])};
          *reinterpret_cast<u32x2*>(aux + col) = pg;
          *reinterpret_cast<u32x2*>(aux + p.n_split + col) = pu;
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = w[e] * sigmoid_f(w[e]) * u[t][e];
          const u32x2 po = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
          *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(p.C) + mrow[t] * p.ldc + col) = po;
        }
      } else if constexpr (EPI == EPI_ACC_F32) {
        if (p.beta) w += old[t];
        if (ok[t]) *reinterpret_cast<f32x4*>(static_cast<float*>(p.C) + mrow[t] * p.ldc + n) = w;
      } else if constexpr (EPI == EPI_ROPE) {
        f32x4 hi = u[t];
        if (rot) {
          const float pos = (float)(int)(mrow[t] % p.rope_seq);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float sn, cs;
            rope_sincos(pos, rfreq[e], &sn, &cs);
            const float a = w[e], b = hi[e];
            w[e] = a * cs - b * sn;
            hi[e] = b * cs + a * sn;
          }
        }
        if (ok[t]) {
          bf16_t* crow = static_cast<bf16_t*>(p.C) + mrow[t] * p.ldc + n;
          const u32x2 plo = {pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3])};
          const u32x2 phi = {pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])};
          *reinterpret_cast<u32x2*>(crow) = plo;
          *reinterpret_cast<u32x2*>(crow + (p.rope_d >> 1)) = phi;
        }
      } else {
        w += bias4;
        if constexpr (EPI == EPI_BIAS_GELU) {
          const u32x2 pp = {pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3])};
          if (ok[t]) *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(p.aux) + mrow[t] * p.ldaux + n) = pp;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = gelu_f(w[e], tanh_form);
        } else if constexpr (EPI == EPI_DGELU) {
          w[0] *= gelu_grad_f(bf16_lo(sa[t][0]), tanh_form); w[1] *= gelu_grad_f(bf16_hi(sa[t][0]), tanh_form);
          w[2] *= gelu_grad_f(bf16_lo(sa[t][1]), tanh_form); w[3] *= gelu_grad_f(bf16_hi(sa[t][1]), tanh_form);
        } else if constexpr (EPI == EPI_DSWIGLU) {
          const float gv[4] = {bf16_lo(sa[t][0]), bf16_hi(sa[t][0]), bf16_lo(sa[t][1]), bf16_hi(sa[t][1])};
          const float uv[4] = {bf16_lo(sb[t][0]), bf16_hi(sb[t][0]), bf16_lo(sb[t][1]), bf16_hi(sb[t][1])};
          f32x4 du;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float sg = sigmoid_f(gv[e]);
            du[e] = w[e] * gv[e] * sg;                                   // d_act * silu(g)
            w[e] = w[e] * uv[e] * sg * (1.0f + gv[e] * (1.0f - sg));     // d_act * u * silu'(g)
          }
          const u32x2 pdu = {pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3])};
          if (ok[t]) *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(p.C) + mrow[t] * p.ldc + p.n_split + n) = pdu;
        }
        const u32x2 po = {pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3])};
        if (ok[t]) *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(p.C) + mrow[t] * p.ldc + n) = po;
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, bool AKS, bool BKS, int EPI>
hipError_t launch_cfg(const GemmArgs& a0, hipStream_t stream) {
  GemmArgs a = a0;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int LDS = NST * (BM + BN) * DMA_BK * 2;
  const int n_logical = (EPI == EPI_SWIGLU) ? 2 * a.n_split : a.N;
  a.tiles_m = (a.M + BM - 1) / BM;
  a.a_bytes = AKS ? ((long)(a.K - 1) * a.lda + a.M) * 2 : ((long)(a.M - 1) * a.lda + a.K) * 2;
  a.b_bytes = BKS ? ((long)(a.K - 1) * a.ldb + n_logical) * 2 : ((long)(a.N - 1) * a.ldb + a.K) * 2;
  if (a.a_bytes >= (1L << 31) || a.b_bytes >= (1L << 31)) return hipErrorInvalidValue;
  a.tiles_n = (n_logical + BN - 1) / BN;
  auto kern = gemm_kernel<BM, BN, WM, WN, AKS, BKS, EPI>;
  static LdsLimitOnce lds_limit;      // one per instantiation
  if (hipError_t e = lds_limit.ensure(reinterpret_cast<const void*>(kern), LDS); e != hipSuccess) return e;
  const int T = a.tiles_m * a.tiles_n;
  a.group_m = (T >= 16 && a.tiles_m >= 2) ? 2 : 0;    // measured: a third fewer L2 misses, 1-2 % on the layer
  hipLaunchKernelGGL(kern, dim3(a.group_m ? 8 * ((T + 7) / 8) : T), dim3(NT), LDS, stream, a);
  return hipGetLastError();
}

template <bool AKS, bool BKS, int EPI>
hipError_t launch_layout(const GemmArgs& a, int tile_cfg, hipStream_t stream) {
  if constexpr (EPI == EPI_ROPE) {          // needs 64-column wave blocks: the 128x256 tile has 128
    if (tile_cfg == GEMM_TILE_128x256) tile_cfg = GEMM_TILE_256x256;
    switch (tile_cfg) {
      case GEMM_TILE_256x256: return launch_cfg<256, 256, 128, 64, AKS, BKS, EPI>(a, stream);
      case GEMM_TILE_256x128: return launch_cfg<256, 128, 128, 64, AKS, BKS, EPI>(a, stream);
      default:                return launch_cfg<128, 128, 64, 64, AKS, BKS, EPI>(a, stream);
    }
  } else {
    switch (tile_cfg) {
      case GEMM_TILE_256x256: return launch_cfg<256, 256, 128, 64, AKS, BKS, EPI>(a, stream);
      case GEMM_TILE_256x128: return launch_cfg<256, 128, 128, 64, AKS, BKS, EPI>(a, stream);
      case GEMM_TILE_128x256: return launch_cfg<128, 256, 64, 128, AKS, BKS, EPI>(a, stream);
      default:                return launch_cfg<128, 128, 64, 64, AKS, BKS, EPI>(a, stream);
    }
  }
}

}  // namespace

int gemm_pick_tile(int M, int N, int concurrency) {
  // The main loop is bound by the operand stream into LDS, so a workgroup's rate grows with the flops
  // per operand byte of its tile, BM*BN/(BM+BN); the relative per-CU rates below are measured.
  // Against that, one launch only fills the 256 CUs if it has enough tiles.  With three or more
  // launches of this size in flight on other streams the chip is kept full dynamically and only the
  // rate and the padding of ragged edges count; alone, whole rounds of tiles count.  128x128 tiles run
  // two to a CU (sharing its feed) and balance dynamically.
  if (concurrency < 1) concurrency = 1;
  struct Cand { int id, bm, bn; double rate; };
  static const Cand cands[] = {{GEMM_TILE_256x256, 256, 256, 6.3}, {GEMM_TILE_128x256, 128, 256, 4.5},
                               {GEMM_TILE_256x128, 256, 128, 4.5}, {GEMM_TILE_128x128, 128, 128, 3.4}};
  int best = GEMM_TILE_128x128;
  double best_cost = 1e30;
  for (const Cand& c : cands) {
    const double tiles = (double)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
    double rounds, rate = c.rate;
    if (concurrency >= 3) {
      // a launch of few tiles is a long serial kernel on its stream's critical path, and the other
      // launches in flight do not always fill the chip beside it: charge a tile shape for leaving more
      // than three eighths of its fair share of the chip (256 / concurrency CUs) unused.  Measured on
      // the 640-column input gradient of the 13B shard, four such launches side by side: 24 tiles of
      // 256x256 take 103 us, 40 tiles of 256x128 79 us (0.5 % of the step).  (While the slices' weight
      // gradients still ran between their input gradients, charging against a quarter of the share was
      // the better rule; charging against the whole share was 0.7 % slower then.)
      const double share = 160.0 / concurrency;
      rounds = tiles / 256.0 * (tiles < share ? share / tiles : 1.0);
    } else if (c.id == GEMM_TILE_128x128) {
      const double t = tiles * concurrency;
      if (t > 256) { rate = 2.1; rounds = t / 512 > 1.0 ? t / 512 : 1.0; }
      else rounds = 1.0;
    } else {
      const double t = tiles * concurrency;
      rounds = ceil(t / 256.0);
      if (rounds > 2) rounds = t / 256.0 + 0.5;
    }
    const double cost = rounds * c.bm * c.bn / rate;
    if (cost < best_cost * 0.999) { best_cost = cost; best = c.id; }
  }
  return best;
}

hipError_t gemm_launch(int layout, int epi, const GemmArgs& a, int tile_cfg, hipStream_t stream) {
  if (tile_cfg < 0) tile_cfg = gemm_pick_tile(a.M, epi == EPI_SWIGLU ? 2 * a.n_split : a.N, a.concurrency);
  if (layout == GEMM_NN) {
    switch (epi) {
      case EPI_STORE:     return launch_layout<false, true, EPI_STORE>(a, tile_cfg, stream);
      case EPI_BIAS_GELU: return launch_layout<false, true, EPI_BIAS_GELU>(a, tile_cfg, stream);
      case EPI_SWIGLU:    return launch_layout<false, true, EPI_SWIGLU>(a, tile_cfg, stream);
      case EPI_ROPE:      return launch_layout<false, true, EPI_ROPE>(a, tile_cfg, stream);
      default: return hipErrorInvalidValue;
    }
  } else if (layout == GEMM_NT) {
    switch (epi) {
      case EPI_STORE:   return launch_layout<false, false, EPI_STORE>(a, tile_cfg, stream);
      case EPI_DGELU:   return launch_layout<false, false, EPI_DGELU>(a, tile_cfg, stream);
      case EPI_DSWIGLU: return launch_layout<false, false, EPI_DSWIGLU>(a, tile_cfg, stream);
      default: return hipErrorInvalidValue;
    }
  } else if (layout == GEMM_TN) {
    if (epi == EPI_ACC_F32) return launch_layout<true, true, EPI_ACC_F32>(a, tile_cfg, stream);
    return hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}
