// Internal launcher interface of the small element-wise kernels (see eltwise.hip).
#pragma once
#include <hip/hip_runtime.h>

// Rotary embedding (Sec. 5.4 names it for Llama-2) applied in place to `nblocks` consecutive
// [heads*d]-wide column blocks of a token-major matrix m[rows][ld] starting at column col0;
// position of a row = row % seq.  inverse != 0 applies the transposed rotation (backward).
hipError_t rope_launch(void* m, long ld, int rows, int seq, int col0, int nblocks, int heads, int d,
                       float base, int inverse, hipStream_t st);

// y = x1 + a (+ b) (+ vec): the residual sum that ends the block (bf16, 16-byte chunks).
hipError_t residual_out_launch(const void* x1, const void* a, const void* b, const void* vec, void* y,
                               long n_elems, int h, hipStream_t st);
