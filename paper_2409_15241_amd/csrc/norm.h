// Internal launcher interface of the normalisation and column-reduction kernels (see norm.hip).
#pragma once
#include <hip/hip_runtime.h>

constexpr int NORM_BWD_MAX_BLOCKS = 256;   // one partial row of d gamma / d beta per workgroup
constexpr int NORM_BWD_ROWS = 16;          // rows per workgroup until the block limit is reached
constexpr int COLSUM_PARTS = 64;           // row ranges of the first column-sum stage

struct NormFwdArgs {
  const void* x;          // bf16 [rows, h]
  const void* add1;       // bf16 [rows, h] or null   (a partial sum to add before normalising)
  const void* add2;       // bf16 [rows, h] or null   (the other ranks' sum)
  const void* vec;        // bf16 [h] or null          (a bias added to every row)
  const void* gamma;      // bf16 [h]
  const void* beta;       // bf16 [h] or null
  void* xsum;             // bf16 [rows, h] or null: x + add1 + add2 + vec
  void* y;                // bf16 [rows, h]
  float* mean;            // fp32 [rows] or null (unused for RMSNorm)
  float* rstd;            // fp32 [rows]
  int rows, h, rms;
  float eps;
};

struct NormBwdArgs {
  const void* ga;         // bf16 [rows, h]: gradient w.r.t. the norm output (this rank's partial)
  const void* gb;         // bf16 [rows, h] or null: the other ranks' sum, added to ga
  const void* x;          // bf16 [rows, h]: the norm input
  const void* gamma;      // bf16 [h]
  const float* mean;      // fp32 [rows] (LayerNorm only)
  const float* rstd;      // fp32 [rows]
  const void* dres;       // bf16 [rows, h] or null: gradient arriving over the residual branch
  void* dx;               // bf16 [rows, h] = dres + NormBwd(ga + gb)
  float* part_g;          // fp32 [norm_bwd_blocks(rows), h]
  float* part_b;          // fp32 [norm_bwd_blocks(rows), h] (LayerNorm only)
  float* part_dres;       // fp32 [norm_bwd_blocks(rows), h] or null: partial column sums of dres (a bias gradient)
  float* part_dx;         // fp32 [norm_bwd_blocks(rows), h] or null: partial column sums of dx (a bias gradient)
  int rows, h, rms;
};

int norm_bwd_blocks(int rows);
hipError_t norm_fwd_launch(const NormFwdArgs& a, hipStream_t st);
hipError_t norm_bwd_launch(const NormBwdArgs& a, hipStream_t st);
// out[n] (+)= sum over nparts rows of part[nparts][n], summed in index order
hipError_t colsum_finish_launch(const float* part, int nparts, int n, float* out, int accumulate, hipStream_t st);
// several such reductions in one launch; a job sums nouter groups (ostride floats apart) of nparts
// partial rows (stride floats apart), group by group
constexpr int COLSUM_MAX_JOBS = 8;
struct ColsumJob { const float* part; float* out; int nparts, n; long stride; int nouter; long ostride; };
struct ColsumJobs { ColsumJob job[COLSUM_MAX_JOBS]; };
hipError_t colsum_finish_jobs_launch(const ColsumJobs& jobs, int njobs, int accumulate, hipStream_t st);
// part[COLSUM_PARTS][n] = partial column sums of the bf16 matrix g[rows][ld]
hipError_t colsum_partial_launch(const void* g, long ld, int rows, int n, float* part, hipStream_t st);
