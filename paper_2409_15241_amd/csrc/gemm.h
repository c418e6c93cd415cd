// Internal launcher interface of the bf16 MFMA GEMM (see gemm.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

enum GemmLayout { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum GemmEpilogue {
  EPI_STORE = 0,      // C = bf16(acc + bias)                      bias optional
  EPI_BIAS_GELU = 1,  // aux = bf16(acc + bias); C = bf16(GeLU(acc + bias))
  EPI_SWIGLU = 2,     // aux[:, n] = gate, aux[:, n_split + n] = up; C[:, n] = silu(gate) * up
  EPI_DGELU = 3,      // C = bf16(acc * GeLU'(aux))
  EPI_DSWIGLU = 4,    // C[:, n] = acc * up * silu'(gate); C[:, n_split + n] = acc * silu(gate)
  EPI_ACC_F32 = 5,    // C(fp32) = acc (+ C if beta)
  EPI_ROPE = 6,       // C = bf16(acc) with the rotary embedding applied to columns below rope_cols (heads of rope_d columns)
};
enum GemmTile { GEMM_TILE_128x128 = 0, GEMM_TILE_256x128 = 1, GEMM_TILE_256x256 = 2, GEMM_TILE_128x256 = 3 };

struct GemmArgs {
  const void* A; const void* B; void* C;
  long lda, ldb, ldc;
  int M, N, K;
  const void* bias;      // bf16 [N] or null
  void* aux; long ldaux; // epilogue side tensor (read or written, see GemmEpilogue)
  int n_split;           // SwiGLU: number of gate (= up) columns
  int beta;              // EPI_ACC_F32: 1 = accumulate into C
  int rope_d, rope_seq, rope_cols;   // EPI_ROPE: head width (64 or 128), sequence length (position = row % seq), rotated columns
  float rope_log2_base;
  int gelu_tanh;
  int concurrency;       // launches of similar size expected in flight at once (other streams); 0 = 1
  int tiles_m, tiles_n;  // filled by the launcher
  int group_m;           // filled by the launcher: tile rows per band of the XCD-blocked order, 0 = linear
  long a_bytes, b_bytes; // extent of the A / B views in bytes, filled by the launcher
};

int gemm_pick_tile(int M, int N, int concurrency);
// tile_cfg < 0: pick by shape.  Enqueues on `stream`; returns the launch status.
hipError_t gemm_launch(int layout, int epi, const GemmArgs& a, int tile_cfg, hipStream_t stream);
