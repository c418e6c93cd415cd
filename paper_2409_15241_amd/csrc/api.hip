// Host side of the C ABI declared in include/domino.h: argument validation, memory layout of the
// saved / workspace blocks, the p x q piece schedule over the caller's stream pool (one block, one
// block cut at its all-reduce points, or a stack of blocks whose row slices run on without joining),
// and the single-kernel entry points.  No device memory is allocated here and no host synchronisation
// is performed by the layer calls.
#include "../../include/domino.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "attention.h"
#include "eltwise.h"
#include "gemm.h"
#include "norm.h"
#include "probe.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
int fail_hip(hipError_t e, const char* what) {
  return fail(DOMINO_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}
#define HIP_TRY(expr, what)                                  \
  do {                                                       \
    hipError_t e_ = (expr);                                  \
    if (e_ != hipSuccess) return fail_hip(e_, what);         \
  } while (0)

// One-time notes about conditions that do not change results but cost time (process-wide, see domino_last_warning).
std::mutex g_warn_mutex;
char g_warn[512] = "";
bool g_warned_queues = false;

// The pool's streams overlap only if each sits on a hardware queue of its own.  The HIP runtime reads
// GPU_MAX_HW_QUEUES once, when it starts (default 4, one of which serves the null stream), so all the library can do
// is look at the environment the process was started with and say what it sees.
void note_hw_queues(int nslice) {
  if (nslice < 4) return;
  std::lock_guard<std::mutex> lock(g_warn_mutex);
  if (g_warned_queues) return;
  const char* env = getenv("GPU_MAX_HW_QUEUES");
  const int have = env ? atoi(env) : 0;
  if (have >= nslice + 1) return;
  g_warned_queues = true;
  snprintf(g_warn, sizeof(g_warn),
           "%d row slices run on %d streams but GPU_MAX_HW_QUEUES is %s%s: with fewer hardware queues than streams + 1 "
           "two pool streams share a queue and their slices run one after the other (measured 3.7-4.0 ms instead of "
           "2.6 ms per step on the 13B shard); set GPU_MAX_HW_QUEUES >= %d before the HIP runtime starts",
           nslice, nslice, env ? "" : "unset (runtime default 4)", env ? env : "", nslice + 1);
}

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
constexpr long TWO_GIB = 1L << 31;

// ---------------------------------------------------------------------------------- layout
struct Layout {
  int h, n, t, r, p, q, b, s, f, d, nl, hl, fl, upc, M, Ms, hq;
  bool llama;
  bool merged;       // weight and vector gradients of a block in one launch each over all slices (see merged_wgrads)
  // saved block (bytes)
  size_t ln1, qkv, ctx, lse, x1, ln2, pre, act, mean1, rstd1, mean2, rstd2, saved_total;
  // workspace block (bytes)
  size_t d_pre, dx1, dctx, dqkv, dot, red, ws_total;
  // per-slice block of partial column sums: area k starts area_off[k] floats in and holds area_rows[k]
  // rows of area_n[k] floats; red_floats = size of one slice's block
  size_t red_floats, area_off[8];
  int area_rows[8], area_n[8];
};

enum { AREA_G1 = 0, AREA_B1, AREA_G2, AREA_B2, AREA_BQKV, AREA_BO, AREA_BUP, AREA_BDOWN, NAREAS };

int validate(const domino_cfg* c, Layout* L) {
  if (!c) return fail(DOMINO_ERR_NULL_POINTER, "cfg is NULL");
  if (c->hidden <= 0 || c->heads <= 0 || c->tp <= 0 || c->p <= 0 || c->q <= 0 || c->batch <= 0 ||
      c->seq <= 0 || c->ffn <= 0)
    return fail(DOMINO_ERR_INVALID_ARG, "hidden, heads, tp, p, q, batch, seq, ffn must be positive");
  if (c->rank < 0 || c->rank >= c->tp) return fail(DOMINO_ERR_INVALID_ARG, "rank %d outside [0, tp=%d)", c->rank, c->tp);
  if (c->arch != DOMINO_ARCH_GPT && c->arch != DOMINO_ARCH_LLAMA)
    return fail(DOMINO_ERR_INVALID_ARG, "arch %d is neither GPT (0) nor Llama (1)", c->arch);
  if (!(c->norm_eps > 0.0f) || !(c->norm_eps < 1.0f)) return fail(DOMINO_ERR_INVALID_ARG, "norm_eps must lie in (0, 1)");
  if (c->arch == DOMINO_ARCH_LLAMA && !(c->rope_base > 1.0f)) return fail(DOMINO_ERR_INVALID_ARG, "rope_base must exceed 1");
  if (c->hidden % c->heads) return fail(DOMINO_ERR_INDIVISIBLE, "hidden %d %% heads %d != 0", c->hidden, c->heads);
  if (c->heads % c->tp) return fail(DOMINO_ERR_INDIVISIBLE, "heads %d %% tp %d != 0", c->heads, c->tp);
  if (c->ffn % c->tp) return fail(DOMINO_ERR_INDIVISIBLE, "ffn %d %% tp %d != 0", c->ffn, c->tp);
  if (c->batch % c->p) return fail(DOMINO_ERR_INDIVISIBLE, "batch %d %% p %d != 0", c->batch, c->p);
  if (c->hidden % c->q) return fail(DOMINO_ERR_INDIVISIBLE, "hidden %d %% q %d != 0", c->hidden, c->q);
  Layout l{};
  l.h = c->hidden; l.n = c->heads; l.t = c->tp; l.r = c->rank; l.p = c->p; l.q = c->q;
  l.b = c->batch; l.s = c->seq; l.f = c->ffn;
  l.llama = c->arch == DOMINO_ARCH_LLAMA;
  if (c->wgrad_per_slice != 0 && c->wgrad_per_slice != 1) return fail(DOMINO_ERR_INVALID_ARG, "wgrad_per_slice must be 0 or 1");
  l.merged = c->p > 2 && !c->wgrad_per_slice;
  l.d = l.h / l.n; l.nl = l.n / l.t; l.hl = l.nl * l.d; l.fl = l.f / l.t;
  l.upc = l.fl * (l.llama ? 2 : 1);
  l.hq = l.h / l.q;
  if (l.d != 64 && l.d != 80 && l.d != 128) return fail(DOMINO_ERR_UNSUPPORTED, "head_dim %d not in {64, 80, 128}", l.d);
  if (l.h % 8 || l.hq % 8 || l.fl % 8) return fail(DOMINO_ERR_UNSUPPORTED, "hidden, hidden/q and ffn/tp must be multiples of 8");
  if (l.llama && l.fl % 32) return fail(DOMINO_ERR_UNSUPPORTED, "SwiGLU needs ffn/tp to be a multiple of 32");
  if (l.h > 8192) return fail(DOMINO_ERR_UNSUPPORTED, "hidden %d exceeds 8192", l.h);
  const long M = (long)l.b * l.s;
  long widest = l.h;
  if (3 * l.hl > widest) widest = 3 * l.hl;
  if (l.upc > widest) widest = l.upc;
  if (M * widest * 2 >= TWO_GIB) return fail(DOMINO_ERR_UNSUPPORTED, "an activation tensor would reach 2 GiB");
  if ((long)l.h * widest * 4 >= TWO_GIB) return fail(DOMINO_ERR_UNSUPPORTED, "a weight-gradient tensor would reach 2 GiB");
  l.M = (int)M;
  l.Ms = l.M / l.p;

  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
  const size_t Mz = (size_t)l.M;
  l.ln1 = take(Mz * l.h * 2);
  l.qkv = take(Mz * 3 * l.hl * 2);
  l.ctx = take(Mz * l.hl * 2);
  l.lse = take((size_t)l.b * l.nl * l.s * 4);
  l.x1 = take(Mz * l.h * 2);
  l.ln2 = take(Mz * l.h * 2);
  l.pre = take(Mz * l.upc * 2);
  l.act = take(Mz * l.fl * 2);
  l.mean1 = take(Mz * 4); l.rstd1 = take(Mz * 4); l.mean2 = take(Mz * 4); l.rstd2 = take(Mz * 4);
  l.saved_total = o;

  o = 0;
  l.d_pre = take(Mz * l.upc * 2);
  l.dx1 = take(Mz * l.h * 2);
  l.dctx = take(Mz * l.hl * 2);
  l.dqkv = take(Mz * 3 * l.hl * 2);
  l.dot = take((size_t)l.b * l.nl * l.s * 4);
  {
    const int nb = norm_bwd_blocks(l.Ms);
    // b_o and b_down come out of the Norm2 backward kernel (one partial row per workgroup), the others from column-sum passes
    const int rows[NAREAS] = {nb, nb, nb, nb, COLSUM_PARTS, nb, COLSUM_PARTS, nb};
    const int width[NAREAS] = {l.h, l.h, l.h, l.h, 3 * l.hl, l.h, l.fl, l.h};
    size_t fo = 0;
    for (int k = 0; k < NAREAS; ++k) {
      l.area_off[k] = fo; l.area_rows[k] = rows[k]; l.area_n[k] = width[k];
      fo += (size_t)rows[k] * width[k];
    }
    l.red_floats = (fo + 63) / 64 * 64;
  }
  l.red = take((size_t)l.p * l.red_floats * 4);
  l.ws_total = o;
  if (L) *L = l;
  return DOMINO_OK;
}

// ---------------------------------------------------------------------------------- events, profiling
std::mutex g_mutex;
// Events for the cross-stream edges of a call (timing disabled), kept per device and handed out again from the
// first by the next call on that device: an edge already enqueued keeps the record it was made with.
struct EventPool { std::vector<hipEvent_t> events; size_t used = 0; };
std::map<int, EventPool> g_pools;
EventPool* g_pool = nullptr;               // the current device's pool, set by begin_call()

// Pools under which a layer or stack call has been replayed from a HIP graph bit for bit: 1, 2 or 4 streams, with
// 1, 2 or 4 of them carrying slices.  Instantiating a graph captured with a pool of 3 or 8 streams has aborted
// inside the runtime; until the reason is known such captures are refused before anything is enqueued.
bool capture_pool_ok(int nstreams, int p) {
  const int nslice = p < nstreams ? p : nstreams;
  auto ok = [](int v) { return v == 1 || v == 2 || v == 4; };
  return ok(nstreams) && ok(nslice);
}

thread_local bool g_capturing = false;     // streams[0] of the call being enqueued is under HIP graph capture

int begin_call(void* const* streams, int nstreams, int p, bool backward = false) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  g_pool = &g_pools[dev];
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  HIP_TRY(hipStreamIsCapturing(static_cast<hipStream_t>(streams[0]), &cs), "hipStreamIsCapturing");
  g_capturing = cs != hipStreamCaptureStatusNone;
  if (g_capturing) {
    if (!capture_pool_ok(nstreams, p))
      return fail(DOMINO_ERR_UNSUPPORTED, "streams[0] is being captured into a HIP graph with a pool of %d streams for %d row "
                  "slices: capture is supported for pools of 1, 2 or 4 streams only (see domino_capture_supported)", nstreams, p);
    // every edge of one capture keeps an event of its own: the calls recorded into a capture (a forward and a
    // backward, say) never re-record an event that an earlier call of the same capture recorded
  } else {
    g_pool->used = 0;
  }
  const int nslice = p < nstreams ? p : nstreams;
  note_hw_queues((backward && !g_capturing && nslice <= 2 && nstreams >= 2 * nslice) ? 2 * nslice : nslice);     // streams with launches in flight
  return DOMINO_OK;
}

int next_sync_event(hipEvent_t* ev) {
  if (g_pool->used == g_pool->events.size()) {
    hipEvent_t e;
    HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming), "hipEventCreate");
    g_pool->events.push_back(e);
  }
  *ev = g_pool->events[g_pool->used++];
  return DOMINO_OK;
}

enum ProfClass {
  PC_NORM_FWD = 0, PC_GEMM_QKV, PC_ROPE, PC_ATTN_FWD, PC_GEMM_OUT, PC_GEMM_UP, PC_GEMM_DOWN, PC_RESID_OUT,
  PC_DGRAD_DOWN, PC_WGRAD_DOWN, PC_DGRAD_UP, PC_WGRAD_UP, PC_NORM_BWD, PC_DGRAD_OUT, PC_WGRAD_OUT,
  PC_ATTN_BWD, PC_DGRAD_QKV, PC_WGRAD_QKV, PC_COLSUM, PC_COUNT
};
const char* const PROF_NAMES[PC_COUNT] = {
  "norm_fwd", "gemm_qkv", "rope", "attn_fwd", "gemm_out", "gemm_up", "gemm_down", "residual_out",
  "dgrad_down", "wgrad_down", "dgrad_up", "wgrad_up", "norm_bwd", "dgrad_out", "wgrad_out",
  "attn_bwd", "dgrad_qkv", "wgrad_qkv", "colsum"};

struct ProfRec { int cls; hipStream_t stream; hipEvent_t start, stop; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_free;

int prof_event(hipEvent_t* ev) {
  if (!g_prof_free.empty()) { *ev = g_prof_free.back(); g_prof_free.pop_back(); return DOMINO_OK; }
  HIP_TRY(hipEventCreate(ev), "hipEventCreate");
  return DOMINO_OK;
}

// RAII bracket around the launches of one step on one stream
struct ProfScope {
  int cls; hipStream_t st; hipEvent_t start{}, stop{}; bool live = false;
  ProfScope(int c, hipStream_t s) : cls(c), st(s) {
    if (!g_prof_on) return;
    if (prof_event(&start) != DOMINO_OK || prof_event(&stop) != DOMINO_OK) return;
    if (hipEventRecord(start, st) != hipSuccess) return;
    live = true;
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(stop, st);
    g_prof_recs.push_back({cls, st, start, stop});
  }
};

// row slices in flight at once in the layer call being enqueued (tile choice of its GEMMs); 1 outside
thread_local int g_concurrency = 1;
struct ConcurrencyScope {
  explicit ConcurrencyScope(int c) { g_concurrency = c < 1 ? 1 : c; }
  ~ConcurrencyScope() { g_concurrency = 1; }
};

inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }
inline const char* at(const void* base, size_t off) { return static_cast<const char*>(base) + off; }
inline char* at(void* base, size_t off) { return static_cast<char*>(base) + off; }

GemmArgs gemm_args(const void* A, long lda, const void* B, long ldb, void* C, long ldc, int M, int N, int K) {
  GemmArgs a{};
  a.A = A; a.B = B; a.C = C; a.lda = lda; a.ldb = ldb; a.ldc = ldc; a.M = M; a.N = N; a.K = K;
  a.gelu_tanh = 1;
  a.concurrency = g_concurrency;
  return a;
}

// edge: work submitted later to `to` waits for everything submitted so far to `from`
int edge(hipStream_t from, hipStream_t to) {
  if (from == to) return DOMINO_OK;
  hipEvent_t ev;
  int rc = next_sync_event(&ev);
  if (rc != DOMINO_OK) return rc;
  HIP_TRY(hipEventRecord(ev, from), "hipEventRecord");
  HIP_TRY(hipStreamWaitEvent(to, ev, 0), "hipStreamWaitEvent");
  return DOMINO_OK;
}

#define TRY(expr)                      \
  do {                                 \
    int rc_ = (expr);                  \
    if (rc_ != DOMINO_OK) return rc_;  \
  } while (0)
#define LAUNCH(expr, what) HIP_TRY((expr), what)

int check_streams(void* const* streams, int nstreams) {
  if (!streams) return fail(DOMINO_ERR_NULL_POINTER, "streams is NULL");
  if (nstreams < 1 || nstreams > 64) return fail(DOMINO_ERR_INVALID_ARG, "nstreams %d outside [1, 64]", nstreams);
  return DOMINO_OK;
}

int check_params(const Layout& L, const domino_params* P) {
  if (!P) return fail(DOMINO_ERR_NULL_POINTER, "params is NULL");
  if (!P->norm1_g || !P->norm2_g || !P->w_qkv || !P->w_o || !P->w_up || !P->w_down)
    return fail(DOMINO_ERR_NULL_POINTER, "a weight matrix or norm gain pointer is NULL");
  if (L.llama) {
    if (P->norm1_b || P->norm2_b || P->b_qkv || P->b_o || P->b_up || P->b_down)
      return fail(DOMINO_ERR_INVALID_ARG, "the Llama architecture has no shifts or biases: those pointers must be NULL");
  } else if (!P->norm1_b || !P->norm2_b || !P->b_qkv || !P->b_o || !P->b_up || !P->b_down) {
    return fail(DOMINO_ERR_NULL_POINTER, "a GPT bias or norm shift pointer is NULL");
  }
  return DOMINO_OK;
}


// The QKV product applies the rotary embedding in its epilogue when a head's partner columns (i, i + d/2) can meet in
// one lane there: heads of 64 or 128 columns.  Other head sizes (80) take a separate in-place pass over q and k.
inline bool rope_fused(const Layout& L) { return L.llama && (L.d == 64 || L.d == 128); }

// ---------------------------------------------------------------------------------- the piece schedule
// One block's buffers as the forward / the backward sees them (all device pointers, caller-owned).
struct FwdLayer {
  const domino_params* P;
  const void *x, *attn_others, *mlp_others;
  void *attn_partial, *mlp_partial, *y, *saved;
};
struct BwdLayer {
  const domino_params* P;
  const domino_grads* G;
  const void *saved, *x, *dy, *dln2_others, *dln1_others;
  void *dln2_partial, *dln1_partial, *dx;
  float* red;        // this block's partial column sums: p slices of red_floats floats
  int accumulate;
};

// which stream of the pool carries which piece (Sec. 4.3.1: a fixed pool, picked by index)
// Row slice i runs on streams[i % nslice] with all its column pieces: on one GPU there is no all-reduce for a
// piece to overlap, and pieces on streams of their own were measured slower (the slices already fill the chip).
// With one or two slices in flight and at least twice as many streams in the pool, the backward puts a slice's weight
// gradients on a second stream of its own, streams[nslice + i % nslice]: the weight gradient of a product then runs
// beside the input gradients that follow it on the slice's stream (Sec. 4.1.2 runs it beside the all-reduce of the
// input gradient).  One or two launches have too few tiles for 256 compute units (11-12 % faster steps on the
// shards configured with p = 2); from four launches in flight on the chip is full and more only slow each other
// down (the 13B shard with 4 slices and 4 such extra streams: 630 instead of 790 TFLOP/s).
struct StreamPlan {
  void* const* streams;
  int ns, p, nslice;
  bool side;             // weight gradients on streams of their own
  // (not under graph capture: instantiating a graph captured with the weight gradients on streams of their own has
  // crashed inside the runtime, so a captured call keeps them on the slices' streams)
  StreamPlan(void* const* s, int n, int p_)
      : streams(s), ns(n), p(p_), nslice(p_ < n ? p_ : n), side(!g_capturing && (p_ < n ? p_ : n) <= 2 && n >= 2 * (p_ < n ? p_ : n)) {}
  hipStream_t slice(int i) const { return as_stream(streams[i % nslice]); }
  hipStream_t second(int i) const { return as_stream(streams[(side ? nslice : 0) + i % nslice]); }
  int in_flight(bool backward) const { return (backward && side) ? 2 * nslice : nslice; }
  // streams that a call touches: the first nslice, in the backward also the weight-gradient streams
  std::vector<char> used(bool backward = false) const {
    std::vector<char> u(ns, 0);
    for (int k = 0; k < in_flight(backward); ++k) u[k] = 1;
    return u;
  }
};

// fork: one event on streams[0]; every other stream marked in `used` waits for it
int fork_streams(const StreamPlan& S, const std::vector<char>& used) {
  hipEvent_t fork;
  TRY(next_sync_event(&fork));
  HIP_TRY(hipEventRecord(fork, as_stream(S.streams[0])), "hipEventRecord");
  for (int k = 1; k < S.ns; ++k)
    if (used[k]) HIP_TRY(hipStreamWaitEvent(as_stream(S.streams[k]), fork, 0), "hipStreamWaitEvent");
  return DOMINO_OK;
}
int join_streams(const StreamPlan& S, const std::vector<char>& used) {
  for (int k = 1; k < S.ns; ++k)
    if (used[k]) TRY(edge(as_stream(S.streams[k]), as_stream(S.streams[0])));
  return DOMINO_OK;
}

int check_fwd_layer(const Layout& L, const FwdLayer& B, int parts = DOMINO_FWD_ALL) {
  TRY(check_params(L, B.P));
  if (parts <= 0 || (parts & ~DOMINO_FWD_ALL)) return fail(DOMINO_ERR_INVALID_ARG, "forward parts %d outside [1, %d]", parts, (int)DOMINO_FWD_ALL);
  if (!B.x || !B.attn_partial || !B.saved) return fail(DOMINO_ERR_NULL_POINTER, "x, attn_partial or saved is NULL");
  if ((parts & DOMINO_FWD_MLP) && !B.mlp_partial) return fail(DOMINO_ERR_NULL_POINTER, "mlp_partial is NULL");
  return DOMINO_OK;
}

int check_bwd_layer(const Layout& L, const BwdLayer& B, int parts = DOMINO_BWD_ALL) {
  TRY(check_params(L, B.P));
  const domino_grads* G = B.G;
  if (parts <= 0 || (parts & ~DOMINO_BWD_ALL)) return fail(DOMINO_ERR_INVALID_ARG, "backward parts %d outside [1, %d]", parts, (int)DOMINO_BWD_ALL);
  if (!B.saved || !G) return fail(DOMINO_ERR_NULL_POINTER, "saved or grads is NULL");
  if ((parts & (DOMINO_BWD_MLP | DOMINO_BWD_ATTN)) && (!B.dy || !B.dln2_partial))
    return fail(DOMINO_ERR_NULL_POINTER, "dy or dln2_partial is NULL");
  if ((parts & (DOMINO_BWD_ATTN | DOMINO_BWD_NORM1)) && !B.dln1_partial) return fail(DOMINO_ERR_NULL_POINTER, "dln1_partial is NULL");
  if ((parts & DOMINO_BWD_NORM1) && (!B.x || !B.dx)) return fail(DOMINO_ERR_NULL_POINTER, "x or dx is NULL");
  if (!G->norm1_g || !G->norm2_g || !G->w_qkv || !G->w_o || !G->w_up || !G->w_down)
    return fail(DOMINO_ERR_NULL_POINTER, "a weight or norm-gain gradient pointer is NULL");
  if (!L.llama && (!G->norm1_b || !G->norm2_b || !G->b_qkv || !G->b_o || !G->b_up || !G->b_down))
    return fail(DOMINO_ERR_NULL_POINTER, "a GPT bias or norm-shift gradient pointer is NULL");
  if ((parts & DOMINO_BWD_MLP) && (parts & DOMINO_BWD_NORM1)) {      // the down-projection's weight gradient may read dy after dx is written
    const size_t bytes = (size_t)L.M * L.h * 2;
    const char *a = static_cast<const char*>(B.dy), *b = static_cast<const char*>(B.dx);
    if (a < b + bytes && b < a + bytes) return fail(DOMINO_ERR_INVALID_ARG, "dx overlaps dy");
  }
  return DOMINO_OK;
}

// Forward of row slice i of one block (Sec. 3.2, Eq. 3): every kernel of the slice on its own stream, the q
// column pieces of the two row-cut products (Sec. 3.3, Eq. 4) written in place into the full-width buffers.
// `norm1_done`: the block's Norm1 of this slice has already been written (by the block below, see `next`).
// `next`: the block above in a stack; its Norm1 is then taken in the same pass that forms this block's output.
int enqueue_fwd_slice(const Layout& L, const domino_cfg* cfg, const StreamPlan& S, const FwdLayer& B, int i,
                      int parts = DOMINO_FWD_ALL, bool norm1_done = false, const FwdLayer* next = nullptr) {
  const domino_params* P = B.P;
  const int Ms = L.Ms;
  const bool rms = L.llama;
  hipStream_t st = S.slice(i);
  const size_t r0 = (size_t)i * Ms;                       // first token row of the slice
  const size_t rh = r0 * L.h * 2;                         // byte offset into [M, h] bf16 tensors
  const char* xi = at(B.x, rh);
  void* saved = B.saved;
  char* ln1 = at(saved, L.ln1 + rh);
  char* qkv = at(saved, L.qkv + r0 * 3 * L.hl * 2);
  char* ctx = at(saved, L.ctx + r0 * L.hl * 2);
  float* lse = reinterpret_cast<float*>(at(saved, L.lse)) + (size_t)i * (L.b / L.p) * L.nl * L.s;
  char* x1 = at(saved, L.x1 + rh);
  char* ln2 = at(saved, L.ln2 + rh);
  char* pre = at(saved, L.pre + r0 * L.upc * 2);
  char* act = at(saved, L.act + r0 * L.fl * 2);
  float* mean1 = reinterpret_cast<float*>(at(saved, L.mean1)) + r0;
  float* rstd1 = reinterpret_cast<float*>(at(saved, L.rstd1)) + r0;
  float* mean2 = reinterpret_cast<float*>(at(saved, L.mean2)) + r0;
  float* rstd2 = reinterpret_cast<float*>(at(saved, L.rstd2)) + r0;

  if (parts & DOMINO_FWD_ATTN) {
  if (!norm1_done) {  // F1: Norm1
    ProfScope ps(PC_NORM_FWD, st);
    NormFwdArgs a{};
    a.x = xi; a.gamma = P->norm1_g; a.beta = P->norm1_b; a.y = ln1; a.mean = rms ? nullptr : mean1; a.rstd = rstd1;
    a.rows = Ms; a.h = L.h; a.rms = rms; a.eps = cfg->norm_eps;
    LAUNCH(norm_fwd_launch(a, st), "norm1 forward");
  }
  {  // F2: X * A (attention), column-parallel, never column-sliced
    ProfScope ps(PC_GEMM_QKV, st);
    GemmArgs a = gemm_args(ln1, L.h, P->w_qkv, 3 * L.hl, qkv, 3 * L.hl, Ms, 3 * L.hl, L.h);
    a.bias = P->b_qkv;
    if (rope_fused(L)) {     // q and k leave the product already rotated (the rotary embedding of Sec. 5.4)
      a.rope_d = L.d; a.rope_seq = L.s; a.rope_cols = 2 * L.hl; a.rope_log2_base = log2f(cfg->rope_base);
      LAUNCH(gemm_launch(GEMM_NN, EPI_ROPE, a, -1, st), "qkv product");
    } else {
      LAUNCH(gemm_launch(GEMM_NN, EPI_STORE, a, -1, st), "qkv product");
    }
  }
  if (L.llama && !rope_fused(L)) {
    ProfScope ps(PC_ROPE, st);
    LAUNCH(rope_launch(qkv, 3 * L.hl, Ms, L.s, 0, 2, L.nl, L.d, cfg->rope_base, 0, st), "rotary embedding");
  }
  {  // F3
    ProfScope ps(PC_ATTN_FWD, st);
    AttnArgs a{};
    a.qkv = qkv; a.ld = 3 * L.hl; a.ctx = ctx; a.ld_ctx = L.hl; a.lse = lse;
    a.batch = L.b / L.p; a.seq = L.s; a.heads = L.nl; a.head_dim = L.d; a.scale = 1.0f / sqrtf((float)L.d);
    LAUNCH(attention_fwd_launch(a, st), "attention forward");
  }
  // F4: (XA) * B_j, one piece per column slice, written in place into the full-width buffer
  for (int j = 0; j < L.q; ++j) {
    ProfScope ps(PC_GEMM_OUT, st);
    const size_t cj = (size_t)j * L.hq * 2;
    GemmArgs a = gemm_args(ctx, L.hl, at(P->w_o, cj), L.h, at(B.attn_partial, rh + cj), L.h, Ms, L.hq, L.hl);
    LAUNCH(gemm_launch(GEMM_NN, EPI_STORE, a, -1, st), "out-projection piece");
  }                                                       // column synchronisation before Norm2: stream order
  }
  if (!(parts & DOMINO_FWD_MLP)) return DOMINO_OK;
  {  // F5: residual + reduced attention output + Norm2
    ProfScope ps(PC_NORM_FWD, st);
    NormFwdArgs a{};
    a.x = xi; a.add1 = at(B.attn_partial, rh); a.add2 = B.attn_others ? at(B.attn_others, rh) : nullptr; a.vec = P->b_o;
    a.gamma = P->norm2_g; a.beta = P->norm2_b; a.xsum = x1; a.y = ln2; a.mean = rms ? nullptr : mean2; a.rstd = rstd2;
    a.rows = Ms; a.h = L.h; a.rms = rms; a.eps = cfg->norm_eps;
    LAUNCH(norm_fwd_launch(a, st), "norm2 forward");
  }
  {  // F6: X * A (MLP) with the activation fused
    ProfScope ps(PC_GEMM_UP, st);
    GemmArgs a = gemm_args(ln2, L.h, P->w_up, L.upc, act, L.fl, Ms, L.fl, L.h);
    a.aux = pre; a.ldaux = L.upc; a.gelu_tanh = cfg->gelu_tanh;
    if (L.llama) { a.n_split = L.fl; LAUNCH(gemm_launch(GEMM_NN, EPI_SWIGLU, a, -1, st), "mlp-up product"); }
    else { a.bias = P->b_up; LAUNCH(gemm_launch(GEMM_NN, EPI_BIAS_GELU, a, -1, st), "mlp-up product"); }
  }
  for (int j = 0; j < L.q; ++j) {  // F7
    ProfScope ps(PC_GEMM_DOWN, st);
    const size_t cj = (size_t)j * L.hq * 2;
    GemmArgs a = gemm_args(act, L.fl, at(P->w_down, cj), L.h, at(B.mlp_partial, rh + cj), L.h, Ms, L.hq, L.fl);
    LAUNCH(gemm_launch(GEMM_NN, EPI_STORE, a, -1, st), "mlp-down piece");
  }
  if (next) {  // F8 of this block and F1 of the next in one pass over the rows: y is written and normalised at once
    ProfScope ps(PC_NORM_FWD, st);
    NormFwdArgs a{};
    a.x = x1; a.add1 = at(B.mlp_partial, rh); a.add2 = B.mlp_others ? at(B.mlp_others, rh) : nullptr; a.vec = P->b_down;
    a.gamma = next->P->norm1_g; a.beta = next->P->norm1_b; a.xsum = at(B.y, rh); a.y = at(next->saved, L.ln1 + rh);
    a.mean = rms ? nullptr : reinterpret_cast<float*>(at(next->saved, L.mean1)) + r0;
    a.rstd = reinterpret_cast<float*>(at(next->saved, L.rstd1)) + r0;
    a.rows = Ms; a.h = L.h; a.rms = rms; a.eps = cfg->norm_eps;
    LAUNCH(norm_fwd_launch(a, st), "block output + next norm1");
  } else if (B.y) {  // F8
    ProfScope ps(PC_RESID_OUT, st);
    LAUNCH(residual_out_launch(x1, at(B.mlp_partial, rh), B.mlp_others ? at(B.mlp_others, rh) : nullptr, P->b_down,
                               at(B.y, rh), (long)Ms * L.h, L.h, st), "block output");
  }
  return DOMINO_OK;
}

// With one or two row slices (see merged_wgrads for more) the weight gradients are summed over the slices in slice
// order: slice i's product into a matrix waits for slice i-1's product into the same matrix (one event per matrix; the
// fifth is for the vector gradients).
struct WgChain {
  hipStream_t prev = nullptr, prev_w = nullptr;      // the previous slice's stream and weight-gradient stream
  hipEvent_t done[5] = {}, cur[5] = {};
  // the next slice of the block runs on other streams and will wait for this slice's sums: only then are the events
  // behind them recorded (a record between two kernels costs a few microseconds on the stream)
  bool feeds_next = true;
  void next_is(const StreamPlan& S, int i, int p) {
    feeds_next = i + 1 < p && (S.slice(i + 1) != S.slice(i) || S.second(i + 1) != S.second(i));
  }
};

// Backward of row slice i of one block; within the slice each input gradient is enqueued before the weight
// gradient of the same product (Sec. 4.1.2).
// The gradients of a block's intermediate activations that its weight gradients read (whole tensors, all row slices).
struct GradBufs { char *d_pre, *dx1, *dqkv; };
GradBufs grad_bufs(const Layout& L, void* ws) { return {at(ws, L.d_pre), at(ws, L.dx1), at(ws, L.dqkv)}; }

// With more than two row slices the weight gradients are not formed slice by slice: one launch per matrix contracts
// over all rows of the block after the last slice's input gradients (enqueue_block_end).  Slice by slice, every
// slice after the first reads and rewrites the whole fp32 gradient (for the 13B shard 0.94 GB of 9.4 GB per step at
// p = 4) in launches a quarter as deep; the step sits on the board's power cap, so the saved traffic is saved time
// (3.5-4.5 % of the step).  With one or two slices the slice-by-slice launches on second streams are faster (they fill
// a chip that two slices leave half empty), so the rule follows p alone and the arithmetic does not depend on the pool.
// cfg->wgrad_per_slice keeps the slice-by-slice order of Sec. 4.1.2 for any p.
inline bool merged_wgrads(const Layout& L) { return L.merged; }

// out (+)= the partial rows that `nslices` consecutive slices, the first one's block of partial sums at `red`, left for
// the eight vector gradients (norm gains and shifts, biases): one launch, slices and rows summed in index order
int vector_grads(const Layout& L, const BwdLayer& B, const float* red, int nslices, int accumulate, hipStream_t st) {
  const domino_grads* G = B.G;
  ProfScope ps(PC_COLSUM, st);
  struct { int k; float* out; } vec[NAREAS] = {
    {AREA_G1, G->norm1_g}, {AREA_B1, G->norm1_b}, {AREA_G2, G->norm2_g}, {AREA_B2, G->norm2_b},
    {AREA_BQKV, G->b_qkv}, {AREA_BO, G->b_o}, {AREA_BUP, G->b_up}, {AREA_BDOWN, G->b_down}};
  ColsumJobs jobs{};
  int njobs = 0;
  for (auto& v : vec) {
    if (!v.out) continue;
    if (L.llama && v.k != AREA_G1 && v.k != AREA_G2) continue;
    jobs.job[njobs++] = {red + L.area_off[v.k], v.out, L.area_rows[v.k], L.area_n[v.k], (long)L.area_n[v.k], nslices, (long)L.red_floats};
  }
  LAUNCH(colsum_finish_jobs_launch(jobs, njobs, accumulate, st), "vector gradient reduction");
  return DOMINO_OK;
}

// Points on a slice's stream after which the merged launches at the end of the block, on other streams, may read what
// the slice has written: `ready` behind the last kernel of the call that writes an operand of a weight gradient (the
// attention backward, which leaves the gradient of q, k, v; in a call of the MLP part alone the down-projection's input
// gradient), `dx` behind the Norm1 backward.  One record each: a record between two kernels costs a few microseconds.
struct SliceEvents {
  hipStream_t on = nullptr;
  hipEvent_t ready = nullptr, dx = nullptr;
};

int enqueue_bwd_slice(const Layout& L, const domino_cfg* cfg, void* ws, const GradBufs& gb, hipStream_t st, hipStream_t wst,
                      const BwdLayer& B, int i, WgChain& wg, int parts = DOMINO_BWD_ALL, hipEvent_t before_dx = nullptr,
                      SliceEvents* marks = nullptr) {
  const domino_params* P = B.P;
  const domino_grads* G = B.G;
  const void* saved = B.saved;
  const int Ms = L.Ms;
  const bool rms = L.llama;
  const size_t r0 = (size_t)i * Ms;
  const size_t rh = r0 * L.h * 2;
  const char* xi = B.x ? at(B.x, rh) : nullptr;
  const char* dyi = B.dy ? at(B.dy, rh) : nullptr;
  const char* ln1 = at(saved, L.ln1 + rh);
  const char* qkv = at(saved, L.qkv + r0 * 3 * L.hl * 2);
  const char* ctx = at(saved, L.ctx + r0 * L.hl * 2);
  const float* lse = reinterpret_cast<const float*>(at(saved, L.lse)) + (size_t)i * (L.b / L.p) * L.nl * L.s;
  const char* x1 = at(saved, L.x1 + rh);
  const char* ln2 = at(saved, L.ln2 + rh);
  const char* pre = at(saved, L.pre + r0 * L.upc * 2);
  const char* act = at(saved, L.act + r0 * L.fl * 2);
  const float* mean1 = reinterpret_cast<const float*>(at(saved, L.mean1)) + r0;
  const float* rstd1 = reinterpret_cast<const float*>(at(saved, L.rstd1)) + r0;
  const float* mean2 = reinterpret_cast<const float*>(at(saved, L.mean2)) + r0;
  const float* rstd2 = reinterpret_cast<const float*>(at(saved, L.rstd2)) + r0;
  char* d_pre = gb.d_pre + r0 * L.upc * 2;
  char* dx1 = gb.dx1 + rh;
  char* dctx = at(ws, L.dctx + r0 * L.hl * 2);
  char* dqkv = gb.dqkv + r0 * 3 * L.hl * 2;
  float* dot = reinterpret_cast<float*>(at(ws, L.dot)) + (size_t)i * (L.b / L.p) * L.nl * L.s;
  float* red = B.red + (size_t)i * L.red_floats;
  auto area = [&](int k) { return red + L.area_off[k]; };
  const int beta = (i > 0 || B.accumulate) ? 1 : 0;
  const bool chain = wg.prev && wg.prev != st;
  const bool chain_w = wg.prev_w && wg.prev_w != wst;
  const bool side = wst != st;
  const bool merged = merged_wgrads(L);
  for (hipEvent_t& e : wg.cur) e = nullptr;

  // the point on the slice's stream after which an operand of a weight gradient exists (only needed when the weight
  // gradients run on a stream of their own)
  if (marks) marks->on = st;
  auto produced = [&](hipEvent_t* ev) -> int {
    *ev = nullptr;
    if (!side) return DOMINO_OK;
    TRY(next_sync_event(ev));
    HIP_TRY(hipEventRecord(*ev, st), "hipEventRecord");
    return DOMINO_OK;
  };
  auto wgrad = [&](int which, int cls, hipEvent_t dep, const void* A, long lda, const void* Bm, long ldb, float* C, long ldc,
                   int M, int N) -> int {
    if (merged) return DOMINO_OK;      // formed over all slices at once, after the last slice
    if (dep) HIP_TRY(hipStreamWaitEvent(wst, dep, 0), "hipStreamWaitEvent");
    if (chain_w) HIP_TRY(hipStreamWaitEvent(wst, wg.done[which], 0), "hipStreamWaitEvent");
    {
      ProfScope ps(cls, wst);
      GemmArgs a = gemm_args(A, lda, Bm, ldb, C, ldc, M, N, Ms);
      a.beta = beta;
      LAUNCH(gemm_launch(GEMM_TN, EPI_ACC_F32, a, -1, wst), "weight gradient");
    }
    if (wg.feeds_next || (side && which == 0)) {       // (the second stream's reader of dy is waited for below)
      TRY(next_sync_event(&wg.cur[which]));
      HIP_TRY(hipEventRecord(wg.cur[which], wst), "hipEventRecord");
    }
    return DOMINO_OK;
  };
  auto colsum = [&](const void* g, long ld, int n, int k) -> int {
    ProfScope ps(PC_COLSUM, st);
    LAUNCH(colsum_partial_launch(g, ld, Ms, n, area(k), st), "bias gradient");
    return DOMINO_OK;
  };
  auto norm_bwd = [&](const void* ga, const void* gb, const void* xin, const void* gamma, const float* mean,
                      const float* rstd, const void* dres, void* out, int kg, int kb, int kres = -1, int kdx = -1) -> int {
    ProfScope ps(PC_NORM_BWD, st);
    NormBwdArgs a{};
    a.ga = ga; a.gb = gb; a.x = xin; a.gamma = gamma; a.mean = mean; a.rstd = rstd; a.dres = dres; a.dx = out;
    a.part_g = area(kg); a.part_b = area(kb); a.rows = Ms; a.h = L.h; a.rms = rms;
    if (kres >= 0) { a.part_dres = area(kres); a.part_dx = area(kdx); }   // bias gradients of the two row-cut products
    LAUNCH(norm_bwd_launch(a, st), "norm backward");
    return DOMINO_OK;
  };

  hipEvent_t read_dy = nullptr;   // set once the down-projection's weight gradient, a reader of dy on the second stream, is enqueued
  if (parts & DOMINO_BWD_MLP) {
  hipEvent_t have_dy;          // in a stack dy is what the block above has just written on this stream
  TRY(produced(&have_dy));
  {  // B1 + B3: input gradient of the down-projection (all q column slices inside the K loop), activation backward fused
    ProfScope ps(PC_DGRAD_DOWN, st);
    GemmArgs a = gemm_args(dyi, L.h, P->w_down, L.h, d_pre, L.upc, Ms, L.fl, L.h);
    a.aux = const_cast<char*>(pre); a.ldaux = L.upc; a.gelu_tanh = cfg->gelu_tanh;
    if (L.llama) { a.n_split = L.fl; LAUNCH(gemm_launch(GEMM_NT, EPI_DSWIGLU, a, -1, st), "mlp-down input gradient"); }
    else LAUNCH(gemm_launch(GEMM_NT, EPI_DGELU, a, -1, st), "mlp-down input gradient");
  }
  TRY(wgrad(0, PC_WGRAD_DOWN, have_dy, act, L.fl, dyi, L.h, G->w_down, L.h, L.fl, L.h));        // B2
  if (side) read_dy = wg.cur[0];
  hipEvent_t have_dpre;
  TRY(produced(&have_dpre));
  if (marks && !(parts & DOMINO_BWD_ATTN)) {
    TRY(next_sync_event(&marks->ready));
    HIP_TRY(hipEventRecord(marks->ready, st), "hipEventRecord");
  }
  {  // B4: input gradient of MLP-up: the tensor the third all-reduce would sum
    ProfScope ps(PC_DGRAD_UP, st);
    GemmArgs a = gemm_args(d_pre, L.upc, P->w_up, L.upc, at(B.dln2_partial, rh), L.h, Ms, L.h, L.upc);
    LAUNCH(gemm_launch(GEMM_NT, EPI_STORE, a, -1, st), "mlp-up input gradient");
  }
  TRY(wgrad(1, PC_WGRAD_UP, have_dpre, ln2, L.h, d_pre, L.upc, G->w_up, L.upc, L.h, L.upc));
  if (!L.llama) TRY(colsum(d_pre, L.upc, L.fl, AREA_BUP));
  }
  if (parts & DOMINO_BWD_ATTN) {
  // B5
  TRY(norm_bwd(at(B.dln2_partial, rh), B.dln2_others ? at(B.dln2_others, rh) : nullptr, x1, P->norm2_g, mean2, rstd2,
               dyi, dx1, AREA_G2, AREA_B2, L.llama ? -1 : AREA_BDOWN, L.llama ? -1 : AREA_BO));
  hipEvent_t have_dx1;
  TRY(produced(&have_dx1));
  {  // B6
    ProfScope ps(PC_DGRAD_OUT, st);
    GemmArgs a = gemm_args(dx1, L.h, P->w_o, L.h, dctx, L.hl, Ms, L.hl, L.h);
    LAUNCH(gemm_launch(GEMM_NT, EPI_STORE, a, -1, st), "out-projection input gradient");
  }
  TRY(wgrad(2, PC_WGRAD_OUT, have_dx1, ctx, L.hl, dx1, L.h, G->w_o, L.h, L.hl, L.h));
  {  // B7
    ProfScope ps(PC_ATTN_BWD, st);
    AttnArgs a{};
    a.qkv = qkv; a.ld = 3 * L.hl; a.ctx = const_cast<char*>(ctx); a.ld_ctx = L.hl; a.dctx = dctx;
    a.lse = const_cast<float*>(lse); a.dot = dot; a.dqkv = dqkv;
    a.batch = L.b / L.p; a.seq = L.s; a.heads = L.nl; a.head_dim = L.d; a.scale = 1.0f / sqrtf((float)L.d);
    a.rope = L.llama ? 1 : 0; a.rope_log2_base = log2f(cfg->rope_base);   // dq, dk are turned back where they are stored
    LAUNCH(attention_bwd_launch(a, st), "attention backward");
  }
  hipEvent_t have_dqkv;
  TRY(produced(&have_dqkv));
  if (marks) {
    TRY(next_sync_event(&marks->ready));
    HIP_TRY(hipEventRecord(marks->ready, st), "hipEventRecord");
  }
  {  // B8: input gradient of QKV: the tensor the fourth all-reduce would sum
    ProfScope ps(PC_DGRAD_QKV, st);
    GemmArgs a = gemm_args(dqkv, 3 * L.hl, P->w_qkv, 3 * L.hl, at(B.dln1_partial, rh), L.h, Ms, L.h, 3 * L.hl);
    LAUNCH(gemm_launch(GEMM_NT, EPI_STORE, a, -1, st), "qkv input gradient");
  }
  TRY(wgrad(3, PC_WGRAD_QKV, have_dqkv, ln1, L.h, dqkv, 3 * L.hl, G->w_qkv, 3 * L.hl, L.h, 3 * L.hl));
  if (!L.llama) TRY(colsum(dqkv, 3 * L.hl, 3 * L.hl, AREA_BQKV));
  }
  if (parts & DOMINO_BWD_NORM1) {
    // dx may be the tensor dy came in (a stack hands one tensor from block to block): its rows are overwritten only
    // after the second stream's reader of dy is through (long since, in practice: it was the first thing enqueued there)
    if (read_dy) HIP_TRY(hipStreamWaitEvent(st, read_dy, 0), "hipStreamWaitEvent");
    // in a stack with merged weight gradients dx goes into the tensor that the block above took its dy from, and that
    // block's down-projection weight gradient (on another stream, enqueued a whole block ago) reads all of it
    if (before_dx) HIP_TRY(hipStreamWaitEvent(st, before_dx, 0), "hipStreamWaitEvent");
    TRY(norm_bwd(at(B.dln1_partial, rh), B.dln1_others ? at(B.dln1_others, rh) : nullptr, xi, P->norm1_g, mean1, rstd1,
                 dx1, at(B.dx, rh), AREA_G1, AREA_B1));
    if (merged) {
      // the vector gradients are summed over all slices in one launch at the end of the block (enqueue_block_end)
      if (marks) {
        TRY(next_sync_event(&marks->dx));
        HIP_TRY(hipEventRecord(marks->dx, st), "hipEventRecord");
      }
    } else {
      // Vector gradients (norm gains and shifts, biases): the partial rows of all three parts of this slice lie in
      // its block of the workspace now; one launch adds them to the gradients, after slice i-1's launch did
      // (fixed order), so only the last slice's small sum is left at the end of the block.
      if (chain) HIP_TRY(hipStreamWaitEvent(st, wg.done[4], 0), "hipStreamWaitEvent");
      TRY(vector_grads(L, B, red, 1, beta, st));
      if (wg.feeds_next) {
        TRY(next_sync_event(&wg.cur[4]));
        HIP_TRY(hipEventRecord(wg.cur[4], st), "hipEventRecord");
      }
    }
  }

  // the slice's stream ends after the slice's weight gradients: whatever follows on it (the same slice of the block
  // below in a stack, a later part, the join) may overwrite what they read
  if (side) TRY(edge(wst, st));
  wg.prev = st;
  wg.prev_w = wst;
  for (int k = 0; k < 5; ++k) wg.done[k] = wg.cur[k];
  return DOMINO_OK;
}

// The end of a block whose weight gradients are merged (see merged_wgrads): the weight gradients of the matrices that
// `parts` owns, each in one launch over all rows of the block, and (with the Norm1 part) one launch that sums the
// vector gradients over all slices.  Enqueued after the slices of the block, the launches spread over the slices' streams starting at
// streams[turn % nslice] (largest first; a stack turns the assignment from block to block so that no stream always
// gets the big ones).  The sum over the rows runs inside the kernel in a fixed order, so results are run-to-run
// identical.
//   marks (one entry per slice, or NULL): with them a launch waits only for the events that the slices on other
//   streams recorded behind the last kernel that writes an operand of a weight gradient (long past when a stream
//   has finished its own slice, so the launches start without a stall and fill the time in which the slowest slice
//   finishes);
//   `above`: the marks of the block above in a stack, whose slices wrote this block's dy.  Without marks the
//   streams meet on streams[0] and part again first, the same join and fork that end one call and begin the next:
//   the form for a call under HIP graph capture (a graph captured with direct waits of every stream for every
//   other one crashed the runtime when it was instantiated).
//   done / done_on (4 entries, by matrix: down, up, qkv, out; or NULL): an event recorded after each launch and the
//   stream it ran on.
int enqueue_block_end(const Layout& L, const StreamPlan& S, const GradBufs& gb, const BwdLayer& B, int parts, int turn,
                          const std::vector<SliceEvents>* marks, const std::vector<SliceEvents>* above = nullptr,
                          hipEvent_t* done = nullptr, hipStream_t* done_on = nullptr) {
  const char* sv = static_cast<const char*>(B.saved);
  const domino_grads* G = B.G;
  // second operand: dy (written by the block above, or the caller's) for the down-projection, else a tensor of this block's slices
  struct { int part, cls; bool reads_dy; const void* A; long lda; const void* Bm; long ldb; float* C; long ldc; int M, N; } w[4] = {
    {DOMINO_BWD_MLP, PC_WGRAD_DOWN, true, sv + L.act, L.fl, B.dy, L.h, G->w_down, L.h, L.fl, L.h},
    {DOMINO_BWD_MLP, PC_WGRAD_UP, false, sv + L.ln2, L.h, gb.d_pre, L.upc, G->w_up, L.upc, L.h, L.upc},
    {DOMINO_BWD_ATTN, PC_WGRAD_QKV, false, sv + L.ln1, L.h, gb.dqkv, 3 * L.hl, G->w_qkv, 3 * L.hl, L.h, 3 * L.hl},
    {DOMINO_BWD_ATTN, PC_WGRAD_OUT, false, sv + L.ctx, L.hl, gb.dx1, L.h, G->w_o, L.h, L.hl, L.h}};
  if (!marks && S.nslice > 1) {
    const std::vector<char> slices = S.used(false);
    TRY(join_streams(S, slices));
    TRY(fork_streams(S, slices));
  }
  int slot = 0;
  for (int m = 0; m < 4; ++m) {
    if (!(parts & w[m].part)) continue;
    hipStream_t st = S.slice((slot++ + turn) % S.nslice);
    if (marks) {
      const std::vector<SliceEvents>* from = w[m].reads_dy ? above : marks;     // dy of a single block is the caller's
      if (from)
        for (const SliceEvents& e : *from) {
          hipEvent_t ev = w[m].reads_dy ? e.dx : e.ready;
          if (ev && e.on != st) HIP_TRY(hipStreamWaitEvent(st, ev, 0), "hipStreamWaitEvent");
        }
    }
    {
      ProfScope ps(w[m].cls, st);
      GemmArgs a = gemm_args(w[m].A, w[m].lda, w[m].Bm, w[m].ldb, w[m].C, w[m].ldc, w[m].M, w[m].N, L.M);
      a.beta = B.accumulate ? 1 : 0;
      LAUNCH(gemm_launch(GEMM_TN, EPI_ACC_F32, a, -1, st), "weight gradient");
    }
    if (done) {
      TRY(next_sync_event(&done[m]));
      HIP_TRY(hipEventRecord(done[m], st), "hipEventRecord");
      done_on[m] = st;
    }
  }
  if (parts & DOMINO_BWD_NORM1) {
    // the eight vector gradients from the partial rows of all slices, behind the smallest weight gradient: by the
    // time that stream gets here the last slice's Norm1 backward, whose partial rows it needs, is through
    hipStream_t st = S.slice((3 + turn) % S.nslice);
    if (marks)
      for (const SliceEvents& e : *marks)
        if (e.dx && e.on != st) HIP_TRY(hipStreamWaitEvent(st, e.dx, 0), "hipStreamWaitEvent");
    TRY(vector_grads(L, B, B.red, L.p, B.accumulate ? 1 : 0, st));
  }
  return DOMINO_OK;
}

// workspace of a stack: one block's workspace, the partial-sum areas of the other blocks, two gradient tensors
// handed from block to block in turn (a block reads its dy from one and writes its dx into the other) and, when the
// weight gradients are merged, a second set of the tensors they read, so that the block below can run on while
// they are formed
struct StackLayout {
  size_t red_bytes, extra_red, dmid[2], d_pre2, dx1_2, dqkv2, total;
};
StackLayout stack_layout(const Layout& L, int nlayers) {
  StackLayout s{};
  const size_t Mz = (size_t)L.M;
  s.red_bytes = align_up((size_t)L.p * L.red_floats * 4);
  s.extra_red = L.ws_total;
  size_t o = s.extra_red + (size_t)(nlayers - 1) * s.red_bytes;
  auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
  s.dmid[0] = take(Mz * L.h * 2);
  s.dmid[1] = take(Mz * L.h * 2);
  if (merged_wgrads(L) && nlayers > 1) {
    s.d_pre2 = take(Mz * L.upc * 2);
    s.dx1_2 = take(Mz * L.h * 2);
    s.dqkv2 = take(Mz * 3 * L.hl * 2);
  }
  s.total = o;
  return s;
}
constexpr int MAX_STACK_LAYERS = 1024;

}  // namespace

extern "C" {

const char* domino_last_error(void) { return g_err; }
const char* domino_last_warning(void) {
  std::lock_guard<std::mutex> lock(g_warn_mutex);
  return g_warn;
}
int domino_capture_supported(int nstreams, int p) {
  return (nstreams >= 1 && p >= 1 && capture_pool_ok(nstreams, p)) ? 1 : 0;
}
const char* domino_version(void) { return "domino-mi355x 0.1 (gfx950)"; }

int domino_validate_cfg(const domino_cfg* cfg) { return validate(cfg, nullptr); }

size_t domino_saved_bytes(const domino_cfg* cfg) {
  Layout L;
  return validate(cfg, &L) == DOMINO_OK ? L.saved_total : 0;
}
size_t domino_workspace_bytes(const domino_cfg* cfg) {
  Layout L;
  return validate(cfg, &L) == DOMINO_OK ? L.ws_total : 0;
}

int domino_saved_slot(const domino_cfg* cfg, const char* name, size_t* offset, size_t* bytes) {
  Layout L;
  TRY(validate(cfg, &L));
  if (!name || !offset || !bytes) return fail(DOMINO_ERR_NULL_POINTER, "name, offset or bytes is NULL");
  const size_t Mz = (size_t)L.M;
  struct { const char* n; size_t off, sz; } tab[] = {
    {"ln1", L.ln1, Mz * L.h * 2}, {"qkv", L.qkv, Mz * 3 * L.hl * 2}, {"ctx", L.ctx, Mz * L.hl * 2},
    {"lse", L.lse, (size_t)L.b * L.nl * L.s * 4}, {"x1", L.x1, Mz * L.h * 2}, {"ln2", L.ln2, Mz * L.h * 2},
    {"pre", L.pre, Mz * L.upc * 2}, {"act", L.act, Mz * L.fl * 2}, {"mean1", L.mean1, Mz * 4},
    {"rstd1", L.rstd1, Mz * 4}, {"mean2", L.mean2, Mz * 4}, {"rstd2", L.rstd2, Mz * 4}};
  for (auto& e : tab)
    if (!strcmp(e.n, name)) { *offset = e.off; *bytes = e.sz; return DOMINO_OK; }
  return fail(DOMINO_ERR_INVALID_ARG, "unknown saved tensor '%s'", name);
}

// ------------------------------------------------------------------------------------ forward
int domino_layer_fwd(const domino_cfg* cfg, const domino_params* P,
                     const void* x, const void* attn_others, const void* mlp_others,
                     void* attn_partial, void* mlp_partial, void* y,
                     void* saved, void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams) {
  return domino_layer_fwd_parts(cfg, P, x, attn_others, mlp_others, attn_partial, mlp_partial, y, saved, workspace,
                                workspace_bytes, streams, nstreams, DOMINO_FWD_ALL);
}

int domino_layer_fwd_parts(const domino_cfg* cfg, const domino_params* P,
                           const void* x, const void* attn_others, const void* mlp_others,
                           void* attn_partial, void* mlp_partial, void* y,
                           void* saved, void* workspace, size_t workspace_bytes,
                           void* const* streams, int nstreams, int parts) {
  Layout L;
  TRY(validate(cfg, &L));
  const FwdLayer B{P, x, attn_others, mlp_others, attn_partial, mlp_partial, y, saved};
  TRY(check_fwd_layer(L, B, parts));
  TRY(check_streams(streams, nstreams));
  if (!workspace) return fail(DOMINO_ERR_NULL_POINTER, "workspace is NULL");
  if (workspace_bytes < L.ws_total) return fail(DOMINO_ERR_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu needed", workspace_bytes, L.ws_total);
  std::lock_guard<std::mutex> lock(g_mutex);
  TRY(begin_call(streams, nstreams, L.p));
  ConcurrencyScope conc(nstreams < L.p ? nstreams : L.p);

  const StreamPlan S(streams, nstreams, L.p);
  const std::vector<char> used = S.used();
  TRY(fork_streams(S, used));
  for (int i = 0; i < L.p; ++i) TRY(enqueue_fwd_slice(L, cfg, S, B, i, parts));
  TRY(join_streams(S, used));
  return DOMINO_OK;
}

// ------------------------------------------------------------------------------------ backward
int domino_layer_bwd(const domino_cfg* cfg, const domino_params* P, const void* saved,
                     const void* x, const void* dy,
                     const void* dln2_others, const void* dln1_others,
                     void* dln2_partial, void* dln1_partial, void* dx,
                     const domino_grads* G, int accumulate,
                     void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams) {
  return domino_layer_bwd_parts(cfg, P, saved, x, dy, dln2_others, dln1_others, dln2_partial, dln1_partial, dx, G,
                                accumulate, workspace, workspace_bytes, streams, nstreams, DOMINO_BWD_ALL);
}

int domino_layer_bwd_parts(const domino_cfg* cfg, const domino_params* P, const void* saved,
                           const void* x, const void* dy,
                           const void* dln2_others, const void* dln1_others,
                           void* dln2_partial, void* dln1_partial, void* dx,
                           const domino_grads* G, int accumulate,
                           void* workspace, size_t workspace_bytes,
                           void* const* streams, int nstreams, int parts) {
  Layout L;
  TRY(validate(cfg, &L));
  BwdLayer B{P, G, saved, x, dy, dln2_others, dln1_others, dln2_partial, dln1_partial, dx, nullptr, accumulate};
  TRY(check_bwd_layer(L, B, parts));
  TRY(check_streams(streams, nstreams));
  if (!workspace) return fail(DOMINO_ERR_NULL_POINTER, "workspace is NULL");
  if (workspace_bytes < L.ws_total) return fail(DOMINO_ERR_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu needed", workspace_bytes, L.ws_total);
  std::lock_guard<std::mutex> lock(g_mutex);
  TRY(begin_call(streams, nstreams, L.p, true));
  ConcurrencyScope conc(StreamPlan(streams, nstreams, L.p).in_flight(true));

  B.red = reinterpret_cast<float*>(at(workspace, L.red));
  const StreamPlan S(streams, nstreams, L.p);
  const std::vector<char> used = S.used(true);
  TRY(fork_streams(S, used));
  WgChain wg;
  const GradBufs gb = grad_bufs(L, workspace);
  const bool merged = merged_wgrads(L);
  std::vector<SliceEvents> marks(merged && !g_capturing && S.nslice > 1 ? L.p : 0);     // (one stream orders itself)
  for (int i = 0; i < L.p; ++i) {
    wg.next_is(S, i, L.p);
    TRY(enqueue_bwd_slice(L, cfg, workspace, gb, S.slice(i), S.second(i), B, i, wg, parts, nullptr, marks.empty() ? nullptr : &marks[i]));
  }
  if (merged) TRY(enqueue_block_end(L, S, gb, B, parts, 0, marks.empty() ? nullptr : &marks));
  TRY(join_streams(S, used));
  return DOMINO_OK;
}

// ------------------------------------------------------------------------------------ stack of blocks
size_t domino_stack_workspace_bytes(const domino_cfg* cfg, int nlayers) {
  Layout L;
  if (validate(cfg, &L) != DOMINO_OK) return 0;
  if (nlayers < 1 || nlayers > MAX_STACK_LAYERS) { fail(DOMINO_ERR_INVALID_ARG, "nlayers %d outside [1, %d]", nlayers, MAX_STACK_LAYERS); return 0; }
  return stack_layout(L, nlayers).total;
}

int domino_stack_fwd(const domino_cfg* cfg, int nlayers, const domino_params* params, const void* x,
                     const domino_stack_fwd_io* io, void* workspace, size_t workspace_bytes,
                     void* const* streams, int nstreams) {
  Layout L;
  TRY(validate(cfg, &L));
  if (nlayers < 1 || nlayers > MAX_STACK_LAYERS) return fail(DOMINO_ERR_INVALID_ARG, "nlayers %d outside [1, %d]", nlayers, MAX_STACK_LAYERS);
  if (!params || !io) return fail(DOMINO_ERR_NULL_POINTER, "params or io is NULL");
  std::vector<FwdLayer> layers(nlayers);
  for (int l = 0; l < nlayers; ++l) {
    layers[l] = FwdLayer{&params[l], l == 0 ? x : io[l - 1].y, io[l].attn_others, io[l].mlp_others,
                         io[l].attn_partial, io[l].mlp_partial, io[l].y, io[l].saved};
    TRY(check_fwd_layer(L, layers[l]));
    if (!io[l].y) return fail(DOMINO_ERR_NULL_POINTER, "y of block %d is NULL: a stack needs every block's output", l);
  }
  TRY(check_streams(streams, nstreams));
  const size_t need = stack_layout(L, nlayers).total;
  if (!workspace) return fail(DOMINO_ERR_NULL_POINTER, "workspace is NULL");
  if (workspace_bytes < need) return fail(DOMINO_ERR_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
  std::lock_guard<std::mutex> lock(g_mutex);
  TRY(begin_call(streams, nstreams, L.p));
  ConcurrencyScope conc(nstreams < L.p ? nstreams : L.p);

  // a row slice of block l+1 needs only the same row slice of block l (Sec. 3.2): the slices run through the
  // whole stack on their own streams and meet only at the end
  const StreamPlan S(streams, nstreams, L.p);
  const std::vector<char> used = S.used();
  TRY(fork_streams(S, used));
  for (int l = 0; l < nlayers; ++l)
    for (int i = 0; i < L.p; ++i)
      TRY(enqueue_fwd_slice(L, cfg, S, layers[l], i, DOMINO_FWD_ALL, l > 0, l + 1 < nlayers ? &layers[l + 1] : nullptr));
  TRY(join_streams(S, used));
  return DOMINO_OK;
}

int domino_stack_bwd(const domino_cfg* cfg, int nlayers, const domino_params* params, const void* dy,
                     const domino_stack_bwd_io* io, void* dx, const domino_grads* grads, int accumulate,
                     void* workspace, size_t workspace_bytes, void* const* streams, int nstreams) {
  Layout L;
  TRY(validate(cfg, &L));
  if (nlayers < 1 || nlayers > MAX_STACK_LAYERS) return fail(DOMINO_ERR_INVALID_ARG, "nlayers %d outside [1, %d]", nlayers, MAX_STACK_LAYERS);
  if (!params || !io || !grads) return fail(DOMINO_ERR_NULL_POINTER, "params, io or grads is NULL");
  if (!workspace) return fail(DOMINO_ERR_NULL_POINTER, "workspace is NULL");
  const StackLayout SL = stack_layout(L, nlayers);
  if (workspace_bytes < SL.total) return fail(DOMINO_ERR_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu needed", workspace_bytes, SL.total);
  std::vector<BwdLayer> layers(nlayers);
  for (int l = 0; l < nlayers; ++l) {
    float* red = reinterpret_cast<float*>(l == 0 ? at(workspace, L.red) : at(workspace, SL.extra_red + (size_t)(l - 1) * SL.red_bytes));
    // the gradient handed down the stack lives in two tensors taken in turn: a slice's last kernel of block l writes
    // the rows that the same slice of block l-1, next on the same stream, reads
    const int turn = (nlayers - 1 - l) & 1;
    layers[l] = BwdLayer{&params[l], &grads[l], io[l].saved, io[l].x, l == nlayers - 1 ? dy : at(workspace, SL.dmid[turn ^ 1]),
                         io[l].dln2_others, io[l].dln1_others, io[l].dln2_partial, io[l].dln1_partial,
                         l == 0 ? dx : at(workspace, SL.dmid[turn]), red, accumulate};
    TRY(check_bwd_layer(L, layers[l]));
  }
  TRY(check_streams(streams, nstreams));
  std::lock_guard<std::mutex> lock(g_mutex);
  TRY(begin_call(streams, nstreams, L.p, true));
  ConcurrencyScope conc(StreamPlan(streams, nstreams, L.p).in_flight(true));

  const bool merged = merged_wgrads(L);
  // A graph captured from this call with merged weight gradients and more than one block crashed the runtime when
  // it was instantiated (the single-block call, whose capture is a chain of plain forks and joins, replays fine):
  // refused until the cause is known.
  if (g_capturing && merged && nlayers > 1)
    return fail(DOMINO_ERR_UNSUPPORTED, "streams[0] is being captured into a HIP graph: the backward of a stack of %d blocks with "
                "p = %d > 2 row slices cannot be captured; capture one domino_layer_bwd call per block instead", nlayers, L.p);
  const StreamPlan S(streams, nstreams, L.p);
  const std::vector<char> used = S.used(true);
  TRY(fork_streams(S, used));
  GradBufs gb[2] = {grad_bufs(L, workspace), grad_bufs(L, workspace)};
  if (merged && nlayers > 1) gb[1] = GradBufs{at(workspace, SL.d_pre2), at(workspace, SL.dx1_2), at(workspace, SL.dqkv2)};
  // merged weight gradients of the last block that used each set of gradient tensors: by matrix (down, up, qkv, out)
  hipEvent_t wdone[2][4] = {};
  hipStream_t won[2][4] = {};
  std::vector<SliceEvents> marks[2];       // of the current block and of the block above
  for (int l = nlayers - 1; l >= 0; --l) {
    const int turn = (nlayers - 1 - l) & 1;
    if (merged) {
      // this block overwrites the set of tensors that the merged weight gradients of the block two above read: they
      // were enqueued a whole block ago, so these waits order without stalling
      for (int k = 0; k < S.nslice; ++k)
        for (int m = 1; m < 4; ++m)
          if (wdone[turn][m] && won[turn][m] != S.slice(k)) HIP_TRY(hipStreamWaitEvent(S.slice(k), wdone[turn][m], 0), "hipStreamWaitEvent");
    }
    WgChain wg;
    // dx of this block goes where the block above read its dy: its down-projection weight gradient must be through
    hipEvent_t before_dx = merged ? wdone[turn ^ 1][0] : nullptr;
    std::vector<SliceEvents>& mk = marks[turn];
    mk.assign(merged && !g_capturing && S.nslice > 1 ? L.p : 0, SliceEvents{});
    for (int i = 0; i < L.p; ++i) {
      wg.next_is(S, i, L.p);
      TRY(enqueue_bwd_slice(L, cfg, workspace, gb[turn], S.slice(i), S.second(i), layers[l], i, wg, DOMINO_BWD_ALL, before_dx,
                            mk.empty() ? nullptr : &mk[i]));
    }
    if (merged)
      TRY(enqueue_block_end(L, S, gb[turn], layers[l], DOMINO_BWD_ALL, nlayers - 1 - l, mk.empty() ? nullptr : &mk,
                                l + 1 < nlayers && !marks[turn ^ 1].empty() ? &marks[turn ^ 1] : nullptr, wdone[turn], won[turn]));
  }
  TRY(join_streams(S, used));
  return DOMINO_OK;
}

// ------------------------------------------------------------------------------------ single kernels
int domino_gemm(int layout, int epilogue, int tile,
                const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                int M, int N, int K, const void* bias, void* aux, int64_t ldaux,
                int n_split, int beta, int gelu_tanh, void* stream) {
  if (!A || !B || !C) return fail(DOMINO_ERR_NULL_POINTER, "A, B or C is NULL");
  if (M <= 0 || N <= 0 || K <= 0) return fail(DOMINO_ERR_INVALID_ARG, "M, N, K must be positive");
  if (M % 8 || N % 8 || K % 8 || lda % 8 || ldb % 8 || ldc % 4) return fail(DOMINO_ERR_UNSUPPORTED, "dimensions must be multiples of 8");
  if (tile < -1 || tile > 3) return fail(DOMINO_ERR_INVALID_ARG, "tile %d outside [-1, 3]", tile);
  const bool ok = (layout == DOMINO_GEMM_NN && (epilogue == DOMINO_EPI_STORE || epilogue == DOMINO_EPI_BIAS_GELU || epilogue == DOMINO_EPI_SWIGLU)) ||
                  (layout == DOMINO_GEMM_NT && (epilogue == DOMINO_EPI_STORE || epilogue == DOMINO_EPI_DGELU || epilogue == DOMINO_EPI_DSWIGLU)) ||
                  (layout == DOMINO_GEMM_TN && epilogue == DOMINO_EPI_ACC_F32);
  if (!ok) return fail(DOMINO_ERR_INVALID_ARG, "epilogue %d is not defined for layout %d", epilogue, layout);
  const bool needs_aux = epilogue == DOMINO_EPI_BIAS_GELU || epilogue == DOMINO_EPI_SWIGLU || epilogue == DOMINO_EPI_DGELU || epilogue == DOMINO_EPI_DSWIGLU;
  if (needs_aux && !aux) return fail(DOMINO_ERR_NULL_POINTER, "this epilogue needs aux");
  if (needs_aux && ldaux % 8) return fail(DOMINO_ERR_UNSUPPORTED, "ldaux must be a multiple of 8");
  if (epilogue == DOMINO_EPI_SWIGLU || epilogue == DOMINO_EPI_DSWIGLU) {
    if (n_split != N) return fail(DOMINO_ERR_INVALID_ARG, "SwiGLU epilogues need n_split == N");
    if (epilogue == DOMINO_EPI_SWIGLU && n_split % 32) return fail(DOMINO_ERR_UNSUPPORTED, "n_split must be a multiple of 32");
  }
  GemmArgs a = gemm_args(A, lda, B, ldb, C, ldc, M, N, K);
  a.bias = bias; a.aux = aux; a.ldaux = ldaux; a.n_split = n_split; a.beta = beta; a.gelu_tanh = gelu_tanh;
  const long wide_b = (layout == DOMINO_GEMM_NT) ? ((long)(N - 1) * ldb + K) : ((long)(K - 1) * ldb + (epilogue == DOMINO_EPI_SWIGLU ? 2L * N : N));
  const long wide_a = (layout == DOMINO_GEMM_TN) ? ((long)(K - 1) * lda + M) : ((long)(M - 1) * lda + K);
  if (wide_a * 2 >= TWO_GIB || wide_b * 2 >= TWO_GIB) return fail(DOMINO_ERR_UNSUPPORTED, "an operand would reach 2 GiB");
  HIP_TRY(gemm_launch(layout, epilogue, a, tile, as_stream(stream)), "gemm launch");
  return DOMINO_OK;
}

int domino_gemm_rope(int tile, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int M, int N, int K, int seq, int head_dim, int rope_cols, float base, void* stream) {
  if (!A || !B || !C) return fail(DOMINO_ERR_NULL_POINTER, "A, B or C is NULL");
  if (M <= 0 || N <= 0 || K <= 0 || seq <= 0) return fail(DOMINO_ERR_INVALID_ARG, "M, N, K, seq must be positive");
  if (M % 8 || N % 8 || K % 8 || lda % 8 || ldb % 8 || ldc % 8) return fail(DOMINO_ERR_UNSUPPORTED, "dimensions must be multiples of 8");
  if (tile < -1 || tile > 3) return fail(DOMINO_ERR_INVALID_ARG, "tile %d outside [-1, 3]", tile);
  if (head_dim != 64 && head_dim != 128) return fail(DOMINO_ERR_UNSUPPORTED, "the rotary epilogue takes heads of 64 or 128 columns, not %d", head_dim);
  if (N % head_dim || rope_cols < 0 || rope_cols > N || rope_cols % head_dim)
    return fail(DOMINO_ERR_INVALID_ARG, "N and rope_cols must be multiples of head_dim, rope_cols <= N");
  if (!(base > 1.0f)) return fail(DOMINO_ERR_INVALID_ARG, "base must exceed 1");
  if (((long)(M - 1) * lda + K) * 2 >= TWO_GIB || ((long)(K - 1) * ldb + N) * 2 >= TWO_GIB) return fail(DOMINO_ERR_UNSUPPORTED, "an operand would reach 2 GiB");
  GemmArgs a = gemm_args(A, lda, B, ldb, C, ldc, M, N, K);
  a.rope_d = head_dim; a.rope_seq = seq; a.rope_cols = rope_cols; a.rope_log2_base = log2f(base);
  HIP_TRY(gemm_launch(GEMM_NN, EPI_ROPE, a, tile, as_stream(stream)), "gemm launch");
  return DOMINO_OK;
}

int domino_norm_fwd(const void* x, const void* add1, const void* add2, const void* vec,
                    const void* gamma, const void* beta, void* xsum, void* y, float* mean, float* rstd,
                    int rows, int h, int rms, float eps, void* stream) {
  if (!x || !gamma || !y || !rstd) return fail(DOMINO_ERR_NULL_POINTER, "x, gamma, y or rstd is NULL");
  if (rows <= 0 || h <= 0) return fail(DOMINO_ERR_INVALID_ARG, "rows and h must be positive");
  if (h % 8 || h > 8192) return fail(DOMINO_ERR_UNSUPPORTED, "h must be a multiple of 8 and at most 8192");
  NormFwdArgs a{};
  a.x = x; a.add1 = add1; a.add2 = add2; a.vec = vec; a.gamma = gamma; a.beta = beta; a.xsum = xsum; a.y = y;
  a.mean = rms ? nullptr : mean; a.rstd = rstd; a.rows = rows; a.h = h; a.rms = rms; a.eps = eps;
  HIP_TRY(norm_fwd_launch(a, as_stream(stream)), "norm forward launch");
  return DOMINO_OK;
}

size_t domino_norm_bwd_scratch_floats(int rows, int h) {
  if (rows <= 0 || h <= 0) return 0;
  return 2 * (size_t)norm_bwd_blocks(rows) * h;
}

int domino_norm_bwd(const void* ga, const void* gb, const void* x, const void* gamma,
                    const float* mean, const float* rstd, const void* dres, void* dx,
                    float* dgamma, float* dbeta, float* scratch,
                    int rows, int h, int rms, void* stream) {
  if (!ga || !x || !gamma || !rstd || !dx || !dgamma || !scratch) return fail(DOMINO_ERR_NULL_POINTER, "a required pointer is NULL");
  if (!rms && (!mean || !dbeta)) return fail(DOMINO_ERR_NULL_POINTER, "LayerNorm needs mean and dbeta");
  if (rows <= 0 || h <= 0) return fail(DOMINO_ERR_INVALID_ARG, "rows and h must be positive");
  if (h % 8 || h > 8192) return fail(DOMINO_ERR_UNSUPPORTED, "h must be a multiple of 8 and at most 8192");
  NormBwdArgs a{};
  a.ga = ga; a.gb = gb; a.x = x; a.gamma = gamma; a.mean = mean; a.rstd = rstd; a.dres = dres; a.dx = dx;
  const int nb = norm_bwd_blocks(rows);
  a.part_g = scratch; a.part_b = scratch + (size_t)nb * h; a.rows = rows; a.h = h; a.rms = rms;
  hipStream_t st = as_stream(stream);
  HIP_TRY(norm_bwd_launch(a, st), "norm backward launch");
  ColsumJobs jobs{};
  jobs.job[0] = {a.part_g, dgamma, nb, h, (long)h, 1, 0};
  jobs.job[1] = {a.part_b, dbeta, nb, h, (long)h, 1, 0};
  HIP_TRY(colsum_finish_jobs_launch(jobs, rms ? 1 : 2, 0, st), "norm gain / shift gradient");
  return DOMINO_OK;
}

static int check_attn(int64_t ld, int batch, int seq, int heads, int head_dim) {
  if (batch <= 0 || seq <= 0 || heads <= 0) return fail(DOMINO_ERR_INVALID_ARG, "batch, seq, heads must be positive");
  if (head_dim != 64 && head_dim != 80 && head_dim != 128) return fail(DOMINO_ERR_UNSUPPORTED, "head_dim %d not in {64, 80, 128}", head_dim);
  if (ld < 3L * heads * head_dim || ld % 8) return fail(DOMINO_ERR_INVALID_ARG, "ld must be a multiple of 8 and at least 3*heads*head_dim");
  if ((long)batch * seq * ld * 2 >= TWO_GIB) return fail(DOMINO_ERR_UNSUPPORTED, "qkv would reach 2 GiB");
  return DOMINO_OK;
}

int domino_attention_fwd(const void* qkv, int64_t ld, int batch, int seq, int heads, int head_dim,
                         void* ctx, float* lse, void* stream) {
  if (!qkv || !ctx || !lse) return fail(DOMINO_ERR_NULL_POINTER, "qkv, ctx or lse is NULL");
  TRY(check_attn(ld, batch, seq, heads, head_dim));
  AttnArgs a{};
  a.qkv = qkv; a.ld = ld; a.ctx = ctx; a.ld_ctx = (long)heads * head_dim; a.lse = lse;
  a.batch = batch; a.seq = seq; a.heads = heads; a.head_dim = head_dim; a.scale = 1.0f / sqrtf((float)head_dim);
  HIP_TRY(attention_fwd_launch(a, as_stream(stream)), "attention forward launch");
  return DOMINO_OK;
}

int domino_attention_bwd(const void* qkv, int64_t ld, const void* ctx, const void* dctx, const float* lse,
                         void* dqkv, float* dot, int batch, int seq, int heads, int head_dim, void* stream) {
  if (!qkv || !ctx || !dctx || !lse || !dqkv || !dot) return fail(DOMINO_ERR_NULL_POINTER, "a required pointer is NULL");
  TRY(check_attn(ld, batch, seq, heads, head_dim));
  AttnArgs a{};
  a.qkv = qkv; a.ld = ld; a.ctx = const_cast<void*>(ctx); a.ld_ctx = (long)heads * head_dim; a.dctx = dctx;
  a.lse = const_cast<float*>(lse); a.dot = dot; a.dqkv = dqkv;
  a.batch = batch; a.seq = seq; a.heads = heads; a.head_dim = head_dim; a.scale = 1.0f / sqrtf((float)head_dim);
  HIP_TRY(attention_bwd_launch(a, as_stream(stream)), "attention backward launch");
  return DOMINO_OK;
}

int domino_attention_bwd_rope(const void* qkv, int64_t ld, const void* ctx, const void* dctx, const float* lse,
                              void* dqkv, float* dot, int batch, int seq, int heads, int head_dim, float base, void* stream) {
  if (!qkv || !ctx || !dctx || !lse || !dqkv || !dot) return fail(DOMINO_ERR_NULL_POINTER, "a required pointer is NULL");
  TRY(check_attn(ld, batch, seq, heads, head_dim));
  if (!(base > 1.0f)) return fail(DOMINO_ERR_INVALID_ARG, "base must exceed 1");
  AttnArgs a{};
  a.qkv = qkv; a.ld = ld; a.ctx = const_cast<void*>(ctx); a.ld_ctx = (long)heads * head_dim; a.dctx = dctx;
  a.lse = const_cast<float*>(lse); a.dot = dot; a.dqkv = dqkv;
  a.batch = batch; a.seq = seq; a.heads = heads; a.head_dim = head_dim; a.scale = 1.0f / sqrtf((float)head_dim);
  a.rope = 1; a.rope_log2_base = log2f(base);
  HIP_TRY(attention_bwd_launch(a, as_stream(stream)), "attention backward launch");
  return DOMINO_OK;
}

int domino_rope(void* m, int64_t ld, int rows, int seq, int col0, int nblocks, int heads, int head_dim,
                float base, int inverse, void* stream) {
  if (!m) return fail(DOMINO_ERR_NULL_POINTER, "m is NULL");
  if (rows <= 0 || seq <= 0 || nblocks <= 0 || heads <= 0 || head_dim <= 0 || col0 < 0)
    return fail(DOMINO_ERR_INVALID_ARG, "rows, seq, nblocks, heads, head_dim must be positive");
  if (head_dim % 16 || col0 % 8 || ld % 8) return fail(DOMINO_ERR_UNSUPPORTED, "head_dim must be a multiple of 16, col0 and ld multiples of 8");
  if (col0 + (long)nblocks * heads * head_dim > ld) return fail(DOMINO_ERR_INVALID_ARG, "column blocks exceed ld");
  if (!(base > 1.0f)) return fail(DOMINO_ERR_INVALID_ARG, "base must exceed 1");
  HIP_TRY(rope_launch(m, ld, rows, seq, col0, nblocks, heads, head_dim, base, inverse, as_stream(stream)), "rope launch");
  return DOMINO_OK;
}

int domino_colsum(const void* g, int64_t ld, int rows, int n, float* out, int accumulate, float* scratch, void* stream) {
  if (!g || !out || !scratch) return fail(DOMINO_ERR_NULL_POINTER, "g, out or scratch is NULL");
  if (rows <= 0 || n <= 0) return fail(DOMINO_ERR_INVALID_ARG, "rows and n must be positive");
  if (n % 8 || ld % 8 || ld < n) return fail(DOMINO_ERR_UNSUPPORTED, "n and ld must be multiples of 8, ld >= n");
  hipStream_t st = as_stream(stream);
  HIP_TRY(colsum_partial_launch(g, ld, rows, n, scratch, st), "colsum launch");
  HIP_TRY(colsum_finish_launch(scratch, COLSUM_PARTS, n, out, accumulate, st), "colsum launch");
  return DOMINO_OK;
}

// ---- column sums without a scratch argument: for callers that cannot allocate -----------------------------------
// The first stage's partial rows live in a file-scope device array.  In host code the array's name is only a
// stand-in for the symbol: its device address is looked up once per device and only that address is handed to
// the kernels.
}  // extern "C"
namespace {
constexpr int COLSUM_STATIC_MAX_N = 8192;
static __device__ __align__(256) float scratch[COLSUM_PARTS * COLSUM_STATIC_MAX_N];     // 2 MiB on every GPU used
std::map<int, float*> g_scratch_ptr;       // per device: every GPU holds its own copy of the array at its own address

int static_scratch(float** ptr) {          // g_mutex held
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  auto it = g_scratch_ptr.find(dev);
  if (it == g_scratch_ptr.end()) {
    float* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (!p) return fail(DOMINO_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    it = g_scratch_ptr.emplace(dev, p).first;
  }
  *ptr = it->second;
  return DOMINO_OK;
}
}  // namespace
extern "C" {

int domino_colsum_noalloc(const void* g, int64_t ld, int rows, int n, float* out, int accumulate, void* stream) {
  if (!g || !out) return fail(DOMINO_ERR_NULL_POINTER, "g or out is NULL");
  if (rows <= 0 || n <= 0) return fail(DOMINO_ERR_INVALID_ARG, "rows and n must be positive");
  if (n % 8 || ld % 8 || ld < n) return fail(DOMINO_ERR_UNSUPPORTED, "n and ld must be multiples of 8, ld >= n");
  if (n > COLSUM_STATIC_MAX_N)
    return fail(DOMINO_ERR_UNSUPPORTED, "n = %d exceeds the %d columns the library's own scratch holds; use domino_colsum "
                "with a scratch buffer of the caller's", n, COLSUM_STATIC_MAX_N);
  std::lock_guard<std::mutex> lock(g_mutex);
  float* part = nullptr;
  TRY(static_scratch(&part));
  hipStream_t st = as_stream(stream);
  // the first stage writes every one of its COLSUM_PARTS x n partial sums (zeros for row ranges past the end), so
  // nothing of an earlier call's contents is read and nothing has to be cleared
  HIP_TRY(colsum_partial_launch(g, ld, rows, n, part, st), "colsum launch");
  HIP_TRY(colsum_finish_launch(part, COLSUM_PARTS, n, out, accumulate, st), "colsum launch");
  return DOMINO_OK;
}

int domino_mfma_probe(const void* a, const void* b, float* out, int blocks, int iters, double* flops, void* stream) {
  if (!a || !b || !out) return fail(DOMINO_ERR_NULL_POINTER, "a, b or out is NULL");
  if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24))
    return fail(DOMINO_ERR_INVALID_ARG, "blocks must lie in [1, 65536] and iters in [1, 2^24]");
  if (flops) *flops = (double)blocks * 4.0 * iters * MFMA_PROBE_FLOPS_PER_WAVE_ITER;
  HIP_TRY(mfma_probe_launch(a, b, out, blocks, iters, as_stream(stream)), "mfma probe launch");
  return DOMINO_OK;
}

// ------------------------------------------------------------------------------------ instrumentation
int domino_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_mutex);
  g_prof_on = on != 0;
  return DOMINO_OK;
}
int domino_profile_classes(void) { return PC_COUNT; }
const char* domino_profile_name(int cls) { return (cls >= 0 && cls < PC_COUNT) ? PROF_NAMES[cls] : ""; }

int domino_profile_read(int cls, double* total_ms, int* launches) {
  if (cls < 0 || cls >= PC_COUNT) return fail(DOMINO_ERR_INVALID_ARG, "class %d outside [0, %d)", cls, (int)PC_COUNT);
  if (!total_ms || !launches) return fail(DOMINO_ERR_NULL_POINTER, "total_ms or launches is NULL");
  std::lock_guard<std::mutex> lock(g_mutex);
  double tot = 0.0;
  int n = 0;
  for (auto& r : g_prof_recs) {
    if (r.cls != cls) continue;
    HIP_TRY(hipEventSynchronize(r.stop), "hipEventSynchronize");
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, r.start, r.stop), "hipEventElapsedTime");
    tot += ms;
    ++n;
  }
  *total_ms = tot;
  *launches = n;
  return DOMINO_OK;
}

int domino_profile_records(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  return (int)g_prof_recs.size();
}

int domino_profile_record(int index, int* cls, void** stream, double* start_ms, double* stop_ms) {
  if (!cls || !stream || !start_ms || !stop_ms) return fail(DOMINO_ERR_NULL_POINTER, "an output pointer is NULL");
  std::lock_guard<std::mutex> lock(g_mutex);
  if (index < 0 || index >= (int)g_prof_recs.size()) return fail(DOMINO_ERR_INVALID_ARG, "record %d outside [0, %d)", index, (int)g_prof_recs.size());
  const ProfRec& r = g_prof_recs[index];
  const ProfRec& first = g_prof_recs[0];
  HIP_TRY(hipEventSynchronize(first.start), "hipEventSynchronize");
  HIP_TRY(hipEventSynchronize(r.stop), "hipEventSynchronize");
  float a = 0.0f, b = 0.0f;
  HIP_TRY(hipEventElapsedTime(&a, first.start, r.start), "hipEventElapsedTime");
  HIP_TRY(hipEventElapsedTime(&b, first.start, r.stop), "hipEventElapsedTime");
  *cls = r.cls; *stream = r.stream; *start_ms = a; *stop_ms = b;
  return DOMINO_OK;
}

int domino_profile_reset(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  for (auto& r : g_prof_recs) { g_prof_free.push_back(r.start); g_prof_free.push_back(r.stop); }
  g_prof_recs.clear();
  return DOMINO_OK;
}

void domino_shutdown(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  for (auto& kv : g_pools)
    for (auto e : kv.second.events) (void)hipEventDestroy(e);
  g_pools.clear();
  g_pool = nullptr;
  for (auto& r : g_prof_recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  g_prof_recs.clear();
  for (auto e : g_prof_free) (void)hipEventDestroy(e);
  g_prof_free.clear();
}

}  // extern "C"
