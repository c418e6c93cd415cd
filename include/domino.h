/* domino.h - C ABI of the MI355X-native rank-local hot path of Domino tensor-parallel training.
 *
 * One tensor-parallel rank's share of a pre-norm transformer block, forward and backward, run the
 * Domino way: the batch is cut into p independent row slices (paper Sec. 3.2 / 4.1, Eq. 3) and the
 * second weight matrix of each sub-layer (attention out-projection, MLP down-projection) into q
 * column slices (Sec. 3.3 / 4.2, Eq. 4); the p x q pieces (Sec. 3.4) are enqueued on a fixed pool of
 * caller-provided HIP streams (Sec. 4.3.1).  The four all-reduces of a block (Sec. 2.3) are not
 * performed: the tensors they would sum are outputs ("*_partial"), and what they would add from
 * the other ranks are optional inputs ("*_others").
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers, 16-byte aligned, caller-owned; the library allocates
 *     no device memory.  Activations are bf16, row-major [tokens, features] with tokens = batch*seq
 *     (batch-major); weight matrices are bf16 row-major [in, out]; gradients of parameters are fp32.
 *   - Streams are hipStream_t handles passed as void*.  Calls only enqueue work and return; on
 *     return, everything is ordered before later work submitted to streams[0].  No host sync.
 *   - Return value: DOMINO_OK or a negative DOMINO_ERR_*; domino_last_error() gives the text.
 *     Arguments are validated before any GPU call, so invalid calls fail the same way on a host
 *     without a GPU.  The library never throws and never aborts.  DOMINO_ERR_HIP can come back in the
 *     middle of a call's launches: the streams may then hold part of the work, not joined to streams[0];
 *     synchronise the device before using the buffers or the pool again.
 *   - All streams of a call belong to the current device.  Calls are serialised by a lock inside the
 *     library; the events for the edges between streams are cached per device (domino_shutdown frees them).
 *   - Every single tensor must be smaller than 2 GiB (32-bit buffer offsets in the kernels).
 */
#ifndef DOMINO_H
#define DOMINO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DOMINO_OK = 0,
  DOMINO_ERR_INVALID_ARG = -1,         /* a scalar out of range */
  DOMINO_ERR_INDIVISIBLE = -2,         /* batch % p, hidden % q, heads % tp, ffn % tp, hidden % heads */
  DOMINO_ERR_NULL_POINTER = -3,
  DOMINO_ERR_WORKSPACE_TOO_SMALL = -4,
  DOMINO_ERR_UNSUPPORTED = -5,         /* head_dim not in {64, 80, 128}, dims not multiples of 8/32, ... */
  DOMINO_ERR_HIP = -6                  /* a HIP runtime call failed (text holds hipGetErrorString) */
};

enum { DOMINO_ARCH_GPT = 0,            /* LayerNorm, biases, GeLU (op list of Sec. 4.1.1) */
       DOMINO_ARCH_LLAMA = 1 };        /* RMSNorm, no biases, SwiGLU, rotary embedding (Sec. 5.4) */

typedef struct domino_cfg {
  int32_t hidden, heads, tp, rank;     /* h, n, tensor-parallel degree t, this rank r (Sec. 3.1) */
  int32_t p, q;                        /* row slices p1 (Sec. 4.1.1), column slices p2 (Sec. 4.2) */
  int32_t batch, seq, ffn;             /* b, s, FULL ffn width f (4h, 11008, ...) */
  int32_t arch;                        /* DOMINO_ARCH_* */
  int32_t gelu_tanh;                   /* 1 = tanh form (default), 0 = erf form */
  float norm_eps;                      /* inside the square root; 1e-5 */
  float rope_base;                     /* 10000 */
  int32_t wgrad_per_slice;             /* 0 (default): with p > 2 the weight gradients of a block are formed once over all
                                          rows after the last slice's input gradients (see domino_layer_bwd);
                                          1: always slice by slice behind each input gradient, as Sec. 4.1.2 orders them */
} domino_cfg;

/* Rank-local parameters.  h_l = hidden/tp, f_l = ffn/tp.
 *   norm1_g/b, norm2_g/b [h]; w_qkv [h, 3*h_l] with column blocks [Q | K | V], heads contiguous inside a
 *   block (rank r owns heads r*n/t .. (r+1)*n/t-1); b_qkv [3*h_l]; w_o [h_l, h]; b_o [h];
 *   w_up [h, f_l] (GPT) or [h, 2*f_l] = [gate | up] (Llama); b_up [f_l]; w_down [f_l, h]; b_down [h].
 * Llama: every *_b / b_* pointer must be NULL.  b_o and b_down belong to the reduced tensors: they are
 * added once where the sum is consumed, never to the partials. */
typedef struct domino_params {
  const void *norm1_g, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o,
             *norm2_g, *norm2_b, *w_up, *b_up, *w_down, *b_down;
} domino_params;

/* fp32 gradients, same shapes as domino_params (NULL where the parameter is NULL). */
typedef struct domino_grads {
  float *norm1_g, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o,
        *norm2_g, *norm2_b, *w_up, *b_up, *w_down, *b_down;
} domino_grads;

/* Host-only checks of a configuration (no GPU call): the cuts of Sec. 4.1.1 (batch into p1 parts) and Sec. 4.2
 * (hidden into p2 parts) and the tensor-parallel split of Sec. 3.1 must be exact.  Returns DOMINO_OK or the error. */
int domino_validate_cfg(const domino_cfg* cfg);

/* Bytes of the activation block carried from forward to backward, and of the scratch workspace
 * either call needs (0 on an invalid cfg).  Both are caller-allocated, 256-byte aligned: like the
 * pre-allocated full-width output buffer of Sec. 4.2 into which the column pieces are written, every
 * buffer of the path exists before the call and the library allocates none. */
size_t domino_saved_bytes(const domino_cfg* cfg);
size_t domino_workspace_bytes(const domino_cfg* cfg);

/* Byte offset and size of one named tensor inside the saved block (for inspection by tests):
 * "ln1","qkv","ctx","lse","x1","ln2","pre","act","mean1","rstd1","mean2","rstd2".  Returns DOMINO_OK
 * or DOMINO_ERR_INVALID_ARG for an unknown name. */
int domino_saved_slot(const domino_cfg* cfg, const char* name, size_t* offset, size_t* bytes);

/* Forward of the rank's block on x [b, s, h] (Sec. 3.1-3.4; schedule of Sec. 4.1.1 / 4.2).
 * For each row slice i: Norm1, QKV product (never column-sliced, Sec. 3.1), causal attention, then per
 * column slice j the out-projection piece written in place into attn_partial[rows_i, cols_j] (the
 * concatenation of Sec. 4.2 without a copy); after all q pieces of slice i (the column
 * synchronisation of Sec. 3.3): x1 = x + attn_partial + attn_others + b_o, Norm2, MLP-up with fused
 * activation, per column slice j the down-projection piece into mlp_partial[rows_i, cols_j]; finally
 * y = x1 + mlp_partial + mlp_others + b_down.
 *   attn_others, mlp_others: [b,s,h] or NULL (= zeros): sum of the other ranks' partials.
 *   attn_partial, mlp_partial: out [b,s,h]: what the two forward all-reduces would consume.
 *   y: out [b,s,h] or NULL.   saved: out, domino_saved_bytes().   workspace: scratch.
 *   streams[0..nstreams-1]: row slice i, with its q column pieces in index order, runs on
 *   streams[i % m], m = min(nstreams, p); the forward uses no other stream.  (The backward, when m <= 2 and
 *   nstreams >= 2 m and streams[0] is not being captured, puts slice i's weight gradients on streams[m + i % m],
 *   beside the input gradients that follow them: few slices alone do not fill the chip.)
 *   Slices overlap only if their streams sit on distinct hardware queues: create
 *   the pool once, and let the process have more hardware queues than the pool has streams (HIP's
 *   GPU_MAX_HW_QUEUES, read when the runtime starts; domino_last_warning() tells when it looks too small).
 *   streams[0] may be under HIP graph capture (the other streams join the capture through the call's own
 *   fork and leave it at its join) for the pools domino_capture_supported() accepts. */
int domino_layer_fwd(const domino_cfg* cfg, const domino_params* params,
                     const void* x, const void* attn_others, const void* mlp_others,
                     void* attn_partial, void* mlp_partial, void* y,
                     void* saved, void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams);

/* Backward for L = sum(y * dy) (Sec. 4.1.2: per row slice, the input gradient of each product is
 * formed before its weight gradient).  x and saved are those of the forward call.
 *   dln2_others, dln1_others: [b,s,h] or NULL: the other ranks' sums of the two backward all-reduces.
 *   dln2_partial, dln1_partial: out [b,s,h]: this rank's input gradients of MLP-up and QKV.
 *   dx: out [b,s,h]; must not overlap dy.   grads: fp32; accumulate != 0 adds to their contents, else overwrites.
 * Weight gradients: with p <= 2 (or cfg->wgrad_per_slice) each slice adds its share right behind its input gradient, in
 * slice order; with p > 2 one launch per matrix contracts over all rows of the block after the last slice's input gradients (every
 * further slice would otherwise read and rewrite the whole fp32 gradient; on one GPU that traffic is time), the four
 * launches spread over the slices' streams.  Either way the order of the sums is fixed: results are run-to-run
 * identical and do not depend on the stream pool. */
int domino_layer_bwd(const domino_cfg* cfg, const domino_params* params, const void* saved,
                     const void* x, const void* dy,
                     const void* dln2_others, const void* dln1_others,
                     void* dln2_partial, void* dln1_partial, void* dx,
                     const domino_grads* grads, int accumulate,
                     void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams);

/* ---- the block cut at its four all-reduce points (Sec. 2.3, Fig. 2: one all-reduce after self-attention and
 * one after the MLP in the forward, one before each in the backward).  A caller that performs the reductions
 * itself runs the parts in order and fills the *_others inputs of the next part from the partial outputs of
 * the part before.  Arguments as in domino_layer_fwd / domino_layer_bwd; `parts` is an OR of the flags below
 * and must form one of the listed runs; buffers that the chosen parts neither read nor write may be NULL.
 * saved and workspace carry state from part to part and must not be touched in between. */
enum { DOMINO_FWD_ATTN = 1,    /* Norm1, QKV, attention, out-projection pieces -> attn_partial          */
       DOMINO_FWD_MLP = 2,     /* x1 = x + attn_partial + attn_others + b_o, Norm2, MLP -> mlp_partial, y */
       DOMINO_FWD_ALL = 3 };
enum { DOMINO_BWD_MLP = 1,     /* gradients of MLP-down and MLP-up -> dln2_partial                        */
       DOMINO_BWD_ATTN = 2,    /* Norm2 backward (dln2_partial + dln2_others), out-projection, attention,
                                  QKV -> dln1_partial                                                    */
       DOMINO_BWD_NORM1 = 4,   /* Norm1 backward (dln1_partial + dln1_others) -> dx; vector gradients     */
       DOMINO_BWD_ALL = 7 };
int domino_layer_fwd_parts(const domino_cfg* cfg, const domino_params* params,
                           const void* x, const void* attn_others, const void* mlp_others,
                           void* attn_partial, void* mlp_partial, void* y,
                           void* saved, void* workspace, size_t workspace_bytes,
                           void* const* streams, int nstreams, int parts);
/* The gradient tensors of every matrix are complete after the part that owns the matrix; the eight vector
 * gradients (gains, shifts, biases) are written by DOMINO_BWD_NORM1, from partial sums that the earlier
 * parts left in the workspace.  accumulate must be the same in all parts of one backward. */
int domino_layer_bwd_parts(const domino_cfg* cfg, const domino_params* params, const void* saved,
                           const void* x, const void* dy,
                           const void* dln2_others, const void* dln1_others,
                           void* dln2_partial, void* dln1_partial, void* dx,
                           const domino_grads* grads, int accumulate,
                           void* workspace, size_t workspace_bytes,
                           void* const* streams, int nstreams, int parts);

/* ---- a stack of blocks (Sec. 2.3: N blocks one after the other; Sec. 3.2 and 4.1.1: the row slices stay
 * independent from block to block, so slice 0 of block l+1 starts while the other slices of block l still run) --- */

/* Buffers of one block of a stack in the forward: meanings as in domino_layer_fwd.  y is required (it is the
 * next block's input; the last block's y is the stack's output). */
typedef struct domino_stack_fwd_io {
  const void *attn_others, *mlp_others;     /* [b,s,h] or NULL */
  void *attn_partial, *mlp_partial, *y;     /* out [b,s,h] */
  void *saved;                              /* out, domino_saved_bytes() */
} domino_stack_fwd_io;

/* Buffers of one block of a stack in the backward: meanings as in domino_layer_bwd.  x is the block's forward
 * input (the stack's x for block 0, block l-1's y otherwise), saved the block's saved activations. */
typedef struct domino_stack_bwd_io {
  const void *x, *saved;
  const void *dln2_others, *dln1_others;    /* [b,s,h] or NULL */
  void *dln2_partial, *dln1_partial;        /* out [b,s,h] */
} domino_stack_bwd_io;

/* Workspace bytes of a stack of nlayers blocks (1..1024): one block's workspace, one area of partial
 * vector-gradient sums per further block, two [b,s,h] gradients handed from block to block in turn and, for
 * p > 2, a second set of the activation gradients that the weight gradients read.  0 on error. */
size_t domino_stack_workspace_bytes(const domino_cfg* cfg, int nlayers);

/* Forward of nlayers blocks of the same configuration, params[l] and io[l] being block l's (host arrays of
 * nlayers structs).  Row slice i of every block runs on the stream domino_layer_fwd would give it, and the
 * only joins are the column synchronisations inside a block and one join onto streams[0] after the last
 * block: no stream waits for another between blocks.  Between two blocks one pass over a slice's rows forms
 * the lower block's y and the upper block's Norm1 of it.  Results are bitwise those of nlayers calls of
 * domino_layer_fwd with y of one as x of the next. */
int domino_stack_fwd(const domino_cfg* cfg, int nlayers, const domino_params* params, const void* x,
                     const domino_stack_fwd_io* io, void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams);

/* Backward of the stack for L = sum(y_last * dy): blocks nlayers-1 .. 0, dx of one being dy of the one below
 * (kept in the workspace).  grads[l] are block l's gradients (host array of nlayers structs); accumulate as
 * in domino_layer_bwd.  Within a block the weight and vector gradients are summed as domino_layer_bwd sums them.
 * For p <= 2 a slice goes on from block to block without waiting for the others; for p > 2 the slices of a block
 * meet before its weight gradients (one launch per matrix over all rows), after which each stream goes on with
 * its slice of the block below while the other streams' launches still run (the tensors those read are kept
 * twice and used in turn).  Results are bitwise those of nlayers calls of domino_layer_bwd.
 * Under HIP graph capture (see domino_layer_fwd) a stack backward of more than one block with p > 2 returns
 * DOMINO_ERR_UNSUPPORTED before anything is enqueued: capture one domino_layer_bwd call per block instead. */
int domino_stack_bwd(const domino_cfg* cfg, int nlayers, const domino_params* params, const void* dy,
                     const domino_stack_bwd_io* io, void* dx, const domino_grads* grads, int accumulate,
                     void* workspace, size_t workspace_bytes, void* const* streams, int nstreams);

/* ---- single kernels (the steps above, exposed for unit parity tests and roofline runs) ---------- */

enum { DOMINO_GEMM_NN = 0,   /* C[M,N] = A[M,K] * B[K,N]        forward products (Eq. 1-4)            */
       DOMINO_GEMM_NT = 1,   /* C[M,N] = A[M,K] * B[N,K]^T      input gradient  (Sec. 4.1.2)          */
       DOMINO_GEMM_TN = 2 }; /* C[M,N] = A[K,M]^T * B[K,N]      weight gradient, C fp32 (Sec. 4.1.2)  */
enum { DOMINO_EPI_STORE = 0,      /* C = bf16(acc + bias)                                    NN, NT */
       DOMINO_EPI_BIAS_GELU = 1,  /* aux = bf16(acc + bias), C = GeLU(acc + bias)            NN     */
       DOMINO_EPI_SWIGLU = 2,     /* B = [gate | up] (n_split columns each), N = n_split;
                                     aux[M, 2*n_split] = [gate | up], C[M, n_split] = silu(gate)*up  NN */
       DOMINO_EPI_DGELU = 3,      /* C = acc * GeLU'(aux)                                    NT     */
       DOMINO_EPI_DSWIGLU = 4,    /* aux[M, 2*n_split] = saved [gate | up], N = n_split;
                                     C[M, 2*n_split] = [acc*up*silu'(gate) | acc*silu(gate)]  NT     */
       DOMINO_EPI_ACC_F32 = 5 };  /* C(fp32) = acc, or += acc if beta                        TN     */

/* bf16 MFMA product with fp32 accumulation.  M, N, K and all leading dimensions (in elements) must be
 * multiples of 8.  tile: -1 = choose by shape, 0 = 128x128, 1 = 256x128, 2 = 256x256, 3 = 128x256 workgroup tile.
 * bias: bf16 [N] or NULL.  Invalid layout/epilogue pairs return DOMINO_ERR_INVALID_ARG. */
int domino_gemm(int layout, int epilogue, int tile,
                const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                int M, int N, int K, const void* bias, void* aux, int64_t ldaux,
                int n_split, int beta, int gelu_tanh, void* stream);

/* The forward product C[M,N] = A[M,K] * B[K,N] (bf16, no bias) with the rotary embedding (Sec. 5.4 names it for the
 * Llama-2 models) applied in the epilogue: N is a row of heads of head_dim (64 or 128) columns; in the heads that
 * start below column rope_cols the pairs (i, i + head_dim/2) turn by pos * base^(-2i/head_dim), pos = row % seq;
 * the other heads are stored as they are.  This is how the block's QKV product hands q and k to the attention
 * (rope_cols = 2 * heads * head_dim).  tile as in domino_gemm. */
int domino_gemm_rope(int tile, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int M, int N, int K, int seq, int head_dim, int rope_cols, float base, void* stream);

/* y = Norm(x + add1 + add2 + vec): LayerNorm (rms = 0) or RMSNorm (rms = 1) over the last axis of
 * [rows, h]; add1, add2 [rows, h], vec [h], beta [h], xsum (out: the pre-norm sum), mean may be NULL.
 * mean, rstd: fp32 [rows].  h must be a multiple of 8 and at most 8192. */
int domino_norm_fwd(const void* x, const void* add1, const void* add2, const void* vec,
                    const void* gamma, const void* beta, void* xsum, void* y, float* mean, float* rstd,
                    int rows, int h, int rms, float eps, void* stream);

/* dx = dres + NormBwd(ga + gb) and the parameter gradients dgamma, dbeta (fp32 [h], overwritten;
 * dbeta NULL for RMSNorm).  gb, dres may be NULL.  scratch: fp32, domino_norm_bwd_scratch_floats(rows, h). */
size_t domino_norm_bwd_scratch_floats(int rows, int h);
int domino_norm_bwd(const void* ga, const void* gb, const void* x, const void* gamma,
                    const float* mean, const float* rstd, const void* dres, void* dx,
                    float* dgamma, float* dbeta, float* scratch,
                    int rows, int h, int rms, void* stream);

/* Causal softmax(q k^T / sqrt(d)) v (Eq. 2, first case) per (batch element, local head), flash
 * style (no seq x seq matrix in HBM).  qkv: bf16 [batch*seq, ld] with q of head hh at columns
 * hh*d, k at heads*d + hh*d, v at 2*heads*d + hh*d.  ctx: out bf16 [batch*seq, heads*d];
 * lse: out fp32 [batch, heads, seq], natural-log-sum-exp of the scaled masked scores.
 * head_dim in {64, 80, 128}. */
int domino_attention_fwd(const void* qkv, int64_t ld, int batch, int seq, int heads, int head_dim,
                         void* ctx, float* lse, void* stream);

/* Gradients of the above: dqkv (same layout as qkv) from dctx.  dot: fp32 scratch [batch, heads, seq]. */
int domino_attention_bwd(const void* qkv, int64_t ld, const void* ctx, const void* dctx, const float* lse,
                         void* dqkv, float* dot, int batch, int seq, int heads, int head_dim, void* stream);

/* domino_attention_bwd for q and k that carry the rotary embedding (as domino_gemm_rope or domino_rope leaves them):
 * the dq and dk columns of dqkv are the gradients with respect to q and k BEFORE the rotation (the transposed rotation
 * is applied where they are stored); dv as before.  head_dim in {64, 80, 128}. */
int domino_attention_bwd_rope(const void* qkv, int64_t ld, const void* ctx, const void* dctx, const float* lse,
                              void* dqkv, float* dot, int batch, int seq, int heads, int head_dim, float base, void* stream);

/* Rotary embedding in place on nblocks consecutive [heads*head_dim]-wide column blocks of
 * m[rows, ld] starting at column col0 (pairs (i, i + d/2), angle pos * base^(-2i/d), pos = row % seq);
 * inverse != 0 applies the transposed rotation.  head_dim must be a multiple of 16, col0 and ld multiples of 8
 * (16-byte accesses). */
int domino_rope(void* m, int64_t ld, int rows, int seq, int col0, int nblocks, int heads, int head_dim,
                float base, int inverse, void* stream);

/* out[n] (fp32) = column sums of the bf16 matrix g[rows, ld] (+= if accumulate).
 * scratch: fp32, 64 * n floats. */
int domino_colsum(const void* g, int64_t ld, int rows, int n, float* out, int accumulate,
                  float* scratch, void* stream);

/* domino_colsum for callers that cannot allocate device memory and have no scratch to pass (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same two kernels, with the first stage's
 * 64 x n partial sums in a 2 MiB array that is part of the library's device code (one copy on every GPU the library
 * runs on, held until the process ends).  Allocates nothing.  n is limited to 8192 columns (DOMINO_ERR_UNSUPPORTED
 * beyond); other arguments and errors as domino_colsum; results are bitwise those of domino_colsum.
 * All calls on one GPU share the array: two calls whose kernels can overlap (different streams without an
 * ordering between them, or different host threads' streams) race on it; calls on one stream are safe. */
int domino_colsum_noalloc(const void* g, int64_t ld, int rows, int n, float* out, int accumulate, void* stream);

/* MFMA-only probe for the "share of the measured matrix ceiling" figure that goes beside the share of the nominal
 * peak (the paper's metric is throughput, Sec. 5.2; a roofline needs the ceiling the chip really sustains): `blocks`
 * workgroups of 4 waves, every wave issuing iters x 8 independent 32x32x16 bf16 MFMAs back to back on one A and
 * one B fragment per lane taken from a and b (bf16 [2048] each, caller-filled with the data distribution to
 * probe).  out: fp32 [blocks * 256], receives accumulator sums.  *flops (may be NULL) = flops of the launch. */
int domino_mfma_probe(const void* a, const void* b, float* out, int blocks, int iters, double* flops, void* stream);

/* ---- instrumentation -------------------------------------------------------------------------- */

/* While enabled, every kernel launched by domino_layer_fwd/bwd is bracketed by a pair of timing
 * events on its own stream.  domino_profile_read() synchronises those events and returns, for step
 * class `cls` (0 .. domino_profile_classes()-1), the summed elapsed milliseconds and the launch count
 * since the last domino_profile_reset().  Costs two event records per launch: keep it off when
 * timing the whole layer. */
int domino_profile_enable(int on);
int domino_profile_classes(void);
const char* domino_profile_name(int cls);
int domino_profile_read(int cls, double* total_ms, int* launches);
int domino_profile_reset(void);
/* The single launches behind those sums, in the order they were enqueued since the last reset:
 * domino_profile_records() is their number; domino_profile_record() synchronises record `index`'s events and
 * returns its step class, the stream it ran on (the handle the caller passed in) and its start and stop in
 * milliseconds after the start of record 0 (negative if it began earlier on another stream).  Together they give
 * the timeline of a step across the pool.  Errors: INVALID_ARG for an index out of range, NULL_POINTER, HIP. */
int domino_profile_records(void);
int domino_profile_record(int index, int* cls, void** stream, double* start_ms, double* stop_ms);

const char* domino_last_error(void);   /* thread-local, static storage */

/* A note about a condition that costs time without changing results, or "" if there is none (process-wide,
 * static storage, written at most once per condition).  Today: a layer or stack call that puts 4 or more row
 * slices on streams of their own while GPU_MAX_HW_QUEUES, as found in the environment, is unset or below the
 * number of those streams + 1 (Sec. 4.3.1 keeps a fixed pool of streams; on this runtime two streams that share a
 * hardware queue run their slices one after the other: 3.7-4.0 ms instead of 2.6 ms per step on the 13B shard).
 * The runtime reads the variable when it starts, so the library can only report it. */
const char* domino_last_warning(void);

/* Whether layer and stack calls may be recorded into a HIP graph (Sec. 4.3.2) with a pool of nstreams streams
 * and p row slices: 1 or 0, host-only.  Replays are bitwise the eager step for pools of 1, 2 or 4 streams of
 * which 1, 2 or 4 carry slices.  A call whose streams[0] is being captured with any other pool returns
 * DOMINO_ERR_UNSUPPORTED before it enqueues anything (instantiating such a graph has aborted inside the runtime). */
int domino_capture_supported(int nstreams, int p);
const char* domino_version(void);
void domino_shutdown(void);            /* destroys cached events; the library stays usable */

#ifdef __cplusplus
}
#endif
#endif /* DOMINO_H */
