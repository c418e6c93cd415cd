// Host-only check of the library's piece schedule (the host half of csrc/api.hip): this program links api.hip's host
// code against stand-ins for the HIP runtime and for the kernel launchers, lets the layer, parts and stack calls enqueue
// onto fake streams, and examines the recorded order of launches, event records and event waits:
//   - every launch is ordered after the call's first operation on streams[0] and before its last (fork and join);
//   - every stream other than streams[0] enters a call by waiting for an event recorded in that call (under HIP graph
//     capture this is how a stream joins the capture), and no wait refers to an event not yet recorded in the call;
//   - any two launches that touch overlapping memory, at least one of them writing, are ordered by stream order or by
//     a chain of events (the race check), over the buffers the launchers are handed;
//   - the weight gradients of a matrix, and the reductions of the vector gradients, are enqueued in slice order and
//     ordered one after the other (the fixed accumulation order);
//   - a captured call uses no event twice, and pools outside domino_capture_supported() are refused while capturing.
// Nothing here touches a GPU.  Exit status 0 = every expectation held.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <set>
#include <string>
#include <vector>

#include <hip/hip_runtime.h>

#include "../include/domino.h"
#include "../paper_2409_15241_amd/csrc/attention.h"
#include "../paper_2409_15241_amd/csrc/eltwise.h"
#include "../paper_2409_15241_amd/csrc/gemm.h"
#include "../paper_2409_15241_amd/csrc/norm.h"
#include "../paper_2409_15241_amd/csrc/probe.h"

// ------------------------------------------------------------------------------------------- the recorded schedule
struct Region {                      // rows x cols elements of `esz` bytes, `ld` elements from row to row
  const char* base; long ld; long rows, cols; int esz; bool write;
};
struct Op {
  enum Kind { LAUNCH, RECORD, WAIT } kind;
  hipStream_t stream;
  void* event;                       // RECORD / WAIT
  std::string what;                  // LAUNCH: step name
  std::vector<Region> regions;
  float* wgrad_c = nullptr;          // LAUNCH of a weight gradient: the matrix it accumulates into
  bool vec_reduce = false;           // LAUNCH of the vector-gradient reduction
};
static std::vector<Op> g_ops;
static bool g_merged = false;         // the configuration under test forms its weight gradients once per block
static long g_rows = 0;              // rows (batch x sequence) of the configuration under test
static bool g_capturing = false;
static int g_failures = 0;
static std::string g_case;

#define EXPECT(cond, ...)                                                        \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::printf("FAILED [%s] %s: ", g_case.c_str(), #cond);                   \
      std::printf(__VA_ARGS__);                                                  \
      std::printf("\n");                                                         \
      ++g_failures;                                                              \
    }                                                                            \
  } while (0)

static Region reg(const void* p, long ld, long rows, long cols, int esz, bool write) {
  return Region{static_cast<const char*>(p), ld, rows, cols, esz, write};
}
static void launch(hipStream_t st, const char* what, std::vector<Region> r, float* wgrad_c = nullptr, bool vec = false) {
  Op o;
  o.kind = Op::LAUNCH; o.stream = st; o.event = nullptr; o.what = what; o.wgrad_c = wgrad_c; o.vec_reduce = vec;
  for (auto& x : r)
    if (x.base) o.regions.push_back(x);
  g_ops.push_back(std::move(o));
}

// ------------------------------------------------------------------------------------------- HIP runtime stand-ins
extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = reinterpret_cast<hipEvent_t>(new int(1)); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = reinterpret_cast<hipEvent_t>(new int(0)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<int*>(e); return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
  Op o; o.kind = Op::RECORD; o.stream = s; o.event = e; g_ops.push_back(o); return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
  Op o; o.kind = Op::WAIT; o.stream = s; o.event = e; g_ops.push_back(o); return hipSuccess;
}
hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus* st) {
  *st = g_capturing ? hipStreamCaptureStatusActive : hipStreamCaptureStatusNone;
  return hipSuccess;
}
hipError_t hipGetSymbolAddress(void** p, const void*) { static float dummy[4]; *p = dummy; return hipSuccess; }
void** __hipRegisterFatBinary(const void*) { static void* h = nullptr; return &h; }
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterVar(void**, void*, char*, const char*, int, size_t, int, int) {}
}

// ------------------------------------------------------------------------------------------- launcher stand-ins
static const char* gemm_name(int layout, int epi) {
  if (layout == GEMM_TN) return "wgrad";
  if (layout == GEMM_NT) return epi == EPI_STORE ? "dgrad" : "dgrad+act'";
  return epi == EPI_STORE ? "gemm" : epi == EPI_ROPE ? "gemm+rope" : "gemm+act";
}
hipError_t gemm_launch(int layout, int epi, const GemmArgs& a, int, hipStream_t st) {
  std::vector<Region> r;
  const bool glu = epi == EPI_SWIGLU || epi == EPI_DSWIGLU;
  if (layout == GEMM_TN) r.push_back(reg(a.A, a.lda, a.K, a.M, 2, false)); else r.push_back(reg(a.A, a.lda, a.M, a.K, 2, false));
  if (layout == GEMM_NT) r.push_back(reg(a.B, a.ldb, a.N, a.K, 2, false));
  else r.push_back(reg(a.B, a.ldb, a.K, epi == EPI_SWIGLU ? 2L * a.n_split : a.N, 2, false));
  r.push_back(reg(a.C, a.ldc, a.M, epi == EPI_DSWIGLU ? 2L * a.n_split : a.N, layout == GEMM_TN ? 4 : 2, true));
  if (a.bias) r.push_back(reg(a.bias, a.N, 1, a.N, 2, false));
  if (a.aux) r.push_back(reg(a.aux, a.ldaux, a.M, glu ? 2L * a.n_split : a.N, 2, epi == EPI_BIAS_GELU || epi == EPI_SWIGLU));
  launch(st, gemm_name(layout, epi), r, layout == GEMM_TN ? static_cast<float*>(a.C) : nullptr);
  return hipSuccess;
}
int gemm_pick_tile(int, int, int) { return 0; }
hipError_t rope_launch(void* m, long ld, int rows, int, int col0, int nblocks, int heads, int d, float, int, hipStream_t st) {
  launch(st, "rope", {reg(static_cast<char*>(m) + 2L * col0, ld, rows, (long)nblocks * heads * d, 2, true)});
  return hipSuccess;
}
int norm_bwd_blocks(int rows) {
  const int want = (rows + NORM_BWD_ROWS - 1) / NORM_BWD_ROWS;
  return want < NORM_BWD_MAX_BLOCKS ? want : NORM_BWD_MAX_BLOCKS;
}
hipError_t norm_fwd_launch(const NormFwdArgs& a, hipStream_t st) {
  launch(st, "norm_fwd", {reg(a.x, a.h, a.rows, a.h, 2, false), reg(a.add1, a.h, a.rows, a.h, 2, false),
                          reg(a.add2, a.h, a.rows, a.h, 2, false), reg(a.xsum, a.h, a.rows, a.h, 2, true),
                          reg(a.y, a.h, a.rows, a.h, 2, true), reg(a.mean, a.rows, 1, a.rows, 4, true),
                          reg(a.rstd, a.rows, 1, a.rows, 4, true)});
  return hipSuccess;
}
hipError_t norm_bwd_launch(const NormBwdArgs& a, hipStream_t st) {
  const long nb = norm_bwd_blocks(a.rows);
  launch(st, "norm_bwd", {reg(a.ga, a.h, a.rows, a.h, 2, false), reg(a.gb, a.h, a.rows, a.h, 2, false),
                          reg(a.x, a.h, a.rows, a.h, 2, false), reg(a.dres, a.h, a.rows, a.h, 2, false),
                          reg(a.mean, a.rows, 1, a.rows, 4, false), reg(a.rstd, a.rows, 1, a.rows, 4, false),
                          reg(a.dx, a.h, a.rows, a.h, 2, true), reg(a.part_g, a.h, nb, a.h, 4, true),
                          reg(a.part_b, a.h, nb, a.h, 4, true), reg(a.part_dres, a.h, nb, a.h, 4, true),
                          reg(a.part_dx, a.h, nb, a.h, 4, true)});
  return hipSuccess;
}
hipError_t attention_fwd_launch(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.batch * a.seq;
  launch(st, "attn_fwd", {reg(a.qkv, a.ld, rows, 3L * a.heads * a.head_dim, 2, false),
                          reg(a.ctx, a.ld_ctx, rows, (long)a.heads * a.head_dim, 2, true),
                          reg(a.lse, rows * a.heads, 1, rows * a.heads, 4, true)});
  return hipSuccess;
}
hipError_t attention_bwd_launch(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.batch * a.seq;
  launch(st, "attn_bwd", {reg(a.qkv, a.ld, rows, 3L * a.heads * a.head_dim, 2, false),
                          reg(a.ctx, a.ld_ctx, rows, (long)a.heads * a.head_dim, 2, false),
                          reg(a.dctx, a.ld_ctx, rows, (long)a.heads * a.head_dim, 2, false),
                          reg(a.lse, rows * a.heads, 1, rows * a.heads, 4, false),
                          reg(a.dot, rows * a.heads, 1, rows * a.heads, 4, true),
                          reg(a.dqkv, a.ld, rows, 3L * a.heads * a.head_dim, 2, true)});
  return hipSuccess;
}
hipError_t colsum_partial_launch(const void* g, long ld, int rows, int n, float* part, hipStream_t st) {
  launch(st, "colsum_partial", {reg(g, ld, rows, n, 2, false), reg(part, n, COLSUM_PARTS, n, 4, true)});
  return hipSuccess;
}
hipError_t colsum_finish_jobs_launch(const ColsumJobs& jobs, int njobs, int, hipStream_t st) {
  std::vector<Region> r;
  for (int k = 0; k < njobs; ++k) {
    r.push_back(reg(jobs.job[k].out, jobs.job[k].n, 1, jobs.job[k].n, 4, true));
    for (int g = 0; g < jobs.job[k].nouter; ++g)
      r.push_back(reg(jobs.job[k].part + g * jobs.job[k].ostride, jobs.job[k].stride, jobs.job[k].nparts, jobs.job[k].n, 4, false));
  }
  launch(st, "vector_gradients", r, nullptr, true);
  return hipSuccess;
}
hipError_t colsum_finish_launch(const float* part, int nparts, int n, float* out, int, hipStream_t st) {
  launch(st, "colsum_finish", {reg(part, n, nparts, n, 4, false), reg(out, n, 1, n, 4, true)});
  return hipSuccess;
}
hipError_t residual_out_launch(const void* x1, const void* a, const void* b, const void*, void* y, long n, int h, hipStream_t st) {
  launch(st, "residual_out", {reg(x1, h, n / h, h, 2, false), reg(a, h, n / h, h, 2, false), reg(b, h, n / h, h, 2, false),
                              reg(y, h, n / h, h, 2, true)});
  return hipSuccess;
}
hipError_t mfma_probe_launch(const void*, const void*, float*, int, int, hipStream_t) { return hipSuccess; }

// ------------------------------------------------------------------------------------------- the checks
static bool overlap(const Region& a, const Region& b) {
  const char *a0 = a.base, *a1 = a.base + ((a.rows - 1) * a.ld + a.cols) * a.esz;
  const char *b0 = b.base, *b1 = b.base + ((b.rows - 1) * b.ld + b.cols) * b.esz;
  if (a1 <= b0 || b1 <= a0) return false;
  if (a.ld == b.ld && a.esz == b.esz && a.ld > 0 && a.cols <= a.ld) {   // two windows of one matrix: compare rows and columns
    const long d = (b.base - a.base) / a.esz;                            // b's first element relative to a's
    const long pitch = a.ld;
    const long r = d >= 0 ? d / pitch : -((-d + pitch - 1) / pitch), c = d - r * pitch;   // 0 <= c < pitch
    if (c + b.cols <= pitch)                                             // b's rows do not wrap on a's grid
      return r < a.rows && r + b.rows > 0 && c < a.cols;                 // b's columns start at c >= 0: they meet a's [0, cols) iff c < cols
  }
  return true;                                                           // conservatively
}

struct Analysis {
  std::vector<std::vector<uint64_t>> before;   // before[i]: bitset of operations that happen before operation i
  bool hb(int a, int b) const { return (before[b][a >> 6] >> (a & 63)) & 1; }
};

static Analysis analyse(const std::vector<Op>& ops, int first) {
  const int n = (int)ops.size(), W = (n + 63) / 64;
  Analysis A;
  A.before.assign(n, std::vector<uint64_t>(W, 0));
  std::map<hipStream_t, int> last_on;          // last operation on a stream
  std::map<void*, int> record_of;              // latest record of an event
  for (int i = first; i < n; ++i) {
    auto add = [&](int j) {
      for (int w = 0; w < W; ++w) A.before[i][w] |= A.before[j][w];
      A.before[i][j >> 6] |= 1ull << (j & 63);
    };
    auto it = last_on.find(ops[i].stream);
    if (it != last_on.end()) add(it->second);
    if (ops[i].kind == Op::WAIT) {
      auto r = record_of.find(ops[i].event);
      EXPECT(r != record_of.end(), "operation %d waits for an event that this call has not recorded", i);
      if (r != record_of.end()) add(r->second);
    }
    if (ops[i].kind == Op::RECORD) record_of[ops[i].event] = i;
    last_on[ops[i].stream] = i;
  }
  return A;
}

// one library call = operations [first, end) of g_ops
static void check_call(int first, hipStream_t s0, int p, bool capturing) {
  const int n = (int)g_ops.size();
  if (first == n) return;
  const Analysis A = analyse(g_ops, first);
  int origin = -1, last0 = -1;
  for (int i = first; i < n; ++i)
    if (g_ops[i].stream == s0) { if (origin < 0) origin = i; last0 = i; }
  EXPECT(origin >= 0, "the call put nothing on streams[0]");
  std::set<hipStream_t> entered;
  std::set<void*> recorded;
  for (int i = first; i < n; ++i) {
    const Op& o = g_ops[i];
    if (o.stream != s0 && !entered.count(o.stream)) {
      entered.insert(o.stream);
      EXPECT(o.kind == Op::WAIT && A.hb(origin, i),
             "stream %p enters the call with operation %d, which is not a wait ordered after the call's start", (void*)o.stream, i);
    }
    if (o.kind == Op::RECORD) {
      if (capturing) EXPECT(!recorded.count(o.event), "event recorded twice inside one capture (operation %d)", i);
      recorded.insert(o.event);
    }
    if (o.kind != Op::LAUNCH) continue;
    EXPECT(i == origin || A.hb(origin, i) || o.stream == s0, "launch %d (%s) is not ordered after the call's start", i, o.what.c_str());
    EXPECT(i == last0 || A.hb(i, last0), "launch %d (%s) is not ordered before the call's end on streams[0]", i, o.what.c_str());
  }
  // races
  std::vector<int> L;
  for (int i = first; i < n; ++i)
    if (g_ops[i].kind == Op::LAUNCH) L.push_back(i);
  for (size_t x = 0; x < L.size(); ++x)
    for (size_t y = x + 1; y < L.size(); ++y) {
      const Op &a = g_ops[L[x]], &b = g_ops[L[y]];
      if (A.hb(L[x], L[y])) continue;
      for (const Region& ra : a.regions)
        for (const Region& rb : b.regions)
          if ((ra.write || rb.write) && overlap(ra, rb)) {
            EXPECT(false, "launches %d (%s) and %d (%s) touch the same memory unordered", L[x], a.what.c_str(), L[y], b.what.c_str());
            goto next_pair;
          }
    next_pair:;
    }
  // fixed accumulation order: per matrix, and for the vector gradients, enqueue order = slice order, each ordered after the one before
  std::map<const void*, std::vector<int>> per_matrix, per_vector;     // keyed by the gradient tensor (one set per block of a stack)
  for (int i : L) {
    if (g_ops[i].wgrad_c) per_matrix[g_ops[i].wgrad_c].push_back(i);
    if (g_ops[i].vec_reduce)
      for (const Region& r : g_ops[i].regions)
        if (r.write) { per_vector[r.base].push_back(i); break; }
  }
  for (auto& kv : per_matrix) {
    // slice by slice for one or two slices, one launch over all rows beyond that; either way every row exactly once
    EXPECT((int)kv.second.size() == (g_merged ? 1 : p), "%zu weight-gradient launches into one matrix for %d slices", kv.second.size(), p);
    long rows = 0;
    for (int i : kv.second) rows += g_ops[i].regions[0].rows;
    EXPECT(rows == g_rows, "the weight-gradient launches into one matrix contract over %ld rows of %ld", rows, g_rows);
    for (size_t k = 1; k < kv.second.size(); ++k)
      EXPECT(A.hb(kv.second[k - 1], kv.second[k]), "weight gradients %d and %d into one matrix are not ordered", kv.second[k - 1], kv.second[k]);
    // rows of slice k start k * Ms rows into the activation operand: the k-th launch must be slice k's
    for (size_t k = 1; k < kv.second.size(); ++k)
      EXPECT(g_ops[kv.second[k]].regions[0].base > g_ops[kv.second[k - 1]].regions[0].base, "weight gradients into one matrix are not enqueued in slice order");
  }
  for (auto& kv : per_vector) {
    EXPECT((int)kv.second.size() == (g_merged ? 1 : p) || kv.second.empty(), "%zu vector-gradient reductions for %d slices", kv.second.size(), p);
    long groups = 0;                 // every slice's partial rows exactly once (read off the launch's first vector, a norm gain)
    for (int i : kv.second) {
      const std::vector<Region>& r = g_ops[i].regions;
      for (size_t k = 1; k < r.size() && !r[k].write; ++k) ++groups;
    }
    EXPECT(groups == p, "the vector-gradient reductions of a block sum %ld slices' partial rows of %d", groups, p);
    for (size_t k = 1; k < kv.second.size(); ++k)
      EXPECT(A.hb(kv.second[k - 1], kv.second[k]), "vector-gradient reductions %d and %d are not ordered", kv.second[k - 1], kv.second[k]);
  }
}

// ------------------------------------------------------------------------------------------- driving the library
struct Buffers {                                    // addresses only: one arena for all cases, never written or read
  char* mem;
  size_t size, used = 0;
  explicit Buffers(size_t bytes) : size(bytes) {
    static char* arena = static_cast<char*>(std::malloc(bytes));
    mem = arena;
  }
  void* take(size_t bytes) {
    void* p = mem + used;
    used += (bytes + 255) / 256 * 256;
    if (used > size) { std::printf("arena too small\n"); std::exit(2); }
    return p;
  }
};

static domino_cfg make_cfg(int arch, int p, int q, bool per_slice) {
  domino_cfg c{};
  c.wgrad_per_slice = per_slice ? 1 : 0;
  c.hidden = 256; c.heads = 4; c.tp = 2; c.rank = 1; c.p = p; c.q = q; c.batch = 8; c.seq = 64;
  c.ffn = arch == DOMINO_ARCH_LLAMA ? 704 : 1024;
  c.arch = arch; c.gelu_tanh = 1; c.norm_eps = 1e-5f; c.rope_base = 10000.0f;
  return c;
}

struct Layer {
  domino_params P{};
  domino_grads G{};
  void *attn_others, *mlp_others, *attn_partial, *mlp_partial, *y, *saved, *dln2_others, *dln1_others, *dln2_partial, *dln1_partial;
};

static Layer make_layer(Buffers& B, const domino_cfg& c) {
  Layer L;
  const size_t h = c.hidden, hl = h / c.tp, fl = c.ffn / c.tp, up = fl * (c.arch == DOMINO_ARCH_LLAMA ? 2 : 1);
  const size_t act = (size_t)c.batch * c.seq * h * 2;
  const bool gpt = c.arch == DOMINO_ARCH_GPT;
  L.P.norm1_g = B.take(h * 2); L.P.norm2_g = B.take(h * 2);
  L.P.w_qkv = B.take(h * 3 * hl * 2); L.P.w_o = B.take(hl * h * 2); L.P.w_up = B.take(h * up * 2); L.P.w_down = B.take(fl * h * 2);
  L.G.norm1_g = (float*)B.take(h * 4); L.G.norm2_g = (float*)B.take(h * 4);
  L.G.w_qkv = (float*)B.take(h * 3 * hl * 4); L.G.w_o = (float*)B.take(hl * h * 4);
  L.G.w_up = (float*)B.take(h * up * 4); L.G.w_down = (float*)B.take(fl * h * 4);
  if (gpt) {
    L.P.norm1_b = B.take(h * 2); L.P.norm2_b = B.take(h * 2); L.P.b_qkv = B.take(3 * hl * 2); L.P.b_o = B.take(h * 2);
    L.P.b_up = B.take(fl * 2); L.P.b_down = B.take(h * 2);
    L.G.norm1_b = (float*)B.take(h * 4); L.G.norm2_b = (float*)B.take(h * 4); L.G.b_qkv = (float*)B.take(3 * hl * 4);
    L.G.b_o = (float*)B.take(h * 4); L.G.b_up = (float*)B.take(fl * 4); L.G.b_down = (float*)B.take(h * 4);
  }
  L.attn_others = B.take(act); L.mlp_others = B.take(act); L.attn_partial = B.take(act); L.mlp_partial = B.take(act);
  L.y = B.take(act); L.saved = B.take(domino_saved_bytes(&c));
  L.dln2_others = B.take(act); L.dln1_others = B.take(act); L.dln2_partial = B.take(act); L.dln1_partial = B.take(act);
  return L;
}

static void run_case(int arch, int p, int q, int nstreams, bool capturing, int nlayers, bool parts, bool per_slice = false) {
  char name[160];
  std::snprintf(name, sizeof(name), "%s p=%d q=%d streams=%d%s layers=%d%s", arch ? "llama" : "gpt", p, q, nstreams,
                capturing ? " capturing" : "", nlayers, parts ? (per_slice ? " parts per-slice" : " parts") : (per_slice ? " per-slice" : ""));
  g_case = name;
  const domino_cfg c = make_cfg(arch, p, q, per_slice);
  g_merged = p > 2 && !per_slice;
  g_rows = (long)c.batch * c.seq;
  if (domino_validate_cfg(&c) != DOMINO_OK) { EXPECT(false, "configuration rejected: %s", domino_last_error()); return; }
  Buffers B((size_t)96 << 20);
  std::vector<Layer> layers;
  for (int l = 0; l < nlayers; ++l) layers.push_back(make_layer(B, c));
  const size_t act = (size_t)c.batch * c.seq * c.hidden * 2;
  void* x = B.take(act);
  void* dy = B.take(act);
  void* dx = B.take(act);
  const size_t wsb = nlayers > 1 ? domino_stack_workspace_bytes(&c, nlayers) : domino_workspace_bytes(&c);
  void* ws = B.take(wsb);
  std::vector<void*> streams;
  for (int k = 0; k < nstreams; ++k) streams.push_back(reinterpret_cast<void*>((uintptr_t)0x1000 * (k + 1)));
  hipStream_t s0 = static_cast<hipStream_t>(streams[0]);
  g_capturing = capturing;
  const bool ok_pool = !capturing || domino_capture_supported(nstreams, p);
  auto call = [&](int rc, const char* what) {
    if (ok_pool) EXPECT(rc == DOMINO_OK, "%s returned %d: %s", what, rc, domino_last_error());
    else EXPECT(rc == DOMINO_ERR_UNSUPPORTED, "%s under capture with an unsupported pool returned %d", what, rc);
  };
  g_ops.clear();
  if (nlayers == 1) {
    Layer& L = layers[0];
    if (!parts) {
      int first = (int)g_ops.size();
      call(domino_layer_fwd(&c, &L.P, x, L.attn_others, L.mlp_others, L.attn_partial, L.mlp_partial, L.y, L.saved, ws, wsb,
                            streams.data(), nstreams), "domino_layer_fwd");
      if (!ok_pool) { EXPECT(g_ops.empty(), "a refused call enqueued %zu operations", g_ops.size()); g_capturing = false; return; }
      if (!capturing) check_call(first, s0, p, false);
      const int mid = (int)g_ops.size();
      call(domino_layer_bwd(&c, &L.P, L.saved, x, dy, L.dln2_others, L.dln1_others, L.dln2_partial, L.dln1_partial, dx, &L.G, 0,
                            ws, wsb, streams.data(), nstreams), "domino_layer_bwd");
      // a capture holds the forward and the backward: checked as one unit (events must not repeat across the two calls)
      check_call(capturing ? first : mid, s0, p, capturing);
    } else {
      const int fparts[2] = {DOMINO_FWD_ATTN, DOMINO_FWD_MLP};
      for (int k = 0; k < 2; ++k) {
        const int first = (int)g_ops.size();
        call(domino_layer_fwd_parts(&c, &L.P, x, L.attn_others, L.mlp_others, L.attn_partial, L.mlp_partial, L.y, L.saved, ws, wsb,
                                    streams.data(), nstreams, fparts[k]), "domino_layer_fwd_parts");
        check_call(first, s0, p, false);
      }
      const int bparts[3] = {DOMINO_BWD_MLP, DOMINO_BWD_ATTN, DOMINO_BWD_NORM1};
      for (int k = 0; k < 3; ++k) {
        const int first = (int)g_ops.size();
        call(domino_layer_bwd_parts(&c, &L.P, L.saved, x, dy, L.dln2_others, L.dln1_others, L.dln2_partial, L.dln1_partial, dx, &L.G,
                                    0, ws, wsb, streams.data(), nstreams, bparts[k]), "domino_layer_bwd_parts");
        check_call(first, s0, p, false);
      }
    }
  } else {
    std::vector<domino_params> P;
    std::vector<domino_grads> G;
    std::vector<domino_stack_fwd_io> fio;
    std::vector<domino_stack_bwd_io> bio;
    for (int l = 0; l < nlayers; ++l) {
      Layer& L = layers[l];
      P.push_back(L.P); G.push_back(L.G);
      fio.push_back({L.attn_others, L.mlp_others, L.attn_partial, L.mlp_partial, L.y, L.saved});
      bio.push_back({l == 0 ? x : layers[l - 1].y, L.saved, L.dln2_others, L.dln1_others, L.dln2_partial, L.dln1_partial});
    }
    int first = (int)g_ops.size();
    call(domino_stack_fwd(&c, nlayers, P.data(), x, fio.data(), ws, wsb, streams.data(), nstreams), "domino_stack_fwd");
    if (!ok_pool) { g_capturing = false; return; }
    if (!capturing) check_call(first, s0, p, false);
    const int mid = (int)g_ops.size();
    const int rc = domino_stack_bwd(&c, nlayers, P.data(), dy, bio.data(), dx, G.data(), 0, ws, wsb, streams.data(), nstreams);
    if (capturing && g_merged && nlayers > 1) {   // merged weight gradients over several blocks: not under capture
      EXPECT(rc == DOMINO_ERR_UNSUPPORTED, "a captured stack backward with merged weight gradients returned %d", rc);
      EXPECT((int)g_ops.size() == mid, "a refused call enqueued %zu operations", g_ops.size() - mid);
      check_call(first, s0, p, true);             // the captured forward on its own
    } else {
      call(rc, "domino_stack_bwd");
      check_call(capturing ? first : mid, s0, p, capturing);
    }
  }
  g_capturing = false;
}

int main() {
  int cases = 0;
  for (int arch : {DOMINO_ARCH_GPT, DOMINO_ARCH_LLAMA})
    for (int p : {1, 2, 4, 8})
      for (int q : {1, 2})
        for (int ns = 1; ns <= 8; ++ns) {
          run_case(arch, p, q, ns, false, 1, false); ++cases;
          run_case(arch, p, q, ns, true, 1, false); ++cases;
          // four blocks: the tensors handed from block to block, taken in turn, come round again
          if (q == 2) { run_case(arch, p, q, ns, false, 4, false); run_case(arch, p, q, ns, true, 4, false); cases += 2; }
          if (q == 1) { run_case(arch, p, q, ns, false, 1, true); ++cases; }
          if (p > 2 && q == 2) {      // the slice-by-slice weight gradients of Sec. 4.1.2 for more than two slices
            run_case(arch, p, q, ns, false, 1, false, true); run_case(arch, p, q, ns, true, 1, false, true);
            run_case(arch, p, q, ns, false, 4, false, true); run_case(arch, p, q, ns, true, 4, false, true);
            cases += 4;
          }
          if (p == 4 && q == 1) { run_case(arch, p, q, ns, false, 1, true, true); ++cases; }
        }
  // the check must be able to fail: two launches on different fake streams that write one buffer, no event between them
  {
    g_case = "planted race";
    g_ops.clear();
    static char buf[4096];
    const int before = g_failures;
    hipStream_t a = reinterpret_cast<hipStream_t>((uintptr_t)0x1000), b = reinterpret_cast<hipStream_t>((uintptr_t)0x2000);
    hipEvent_t e;
    (void)hipEventCreateWithFlags(&e, 0);
    (void)hipEventRecord(e, a);
    (void)hipStreamWaitEvent(b, e, 0);
    launch(a, "writer 1", {reg(buf, 64, 8, 64, 2, true)});
    launch(b, "writer 2", {reg(buf + 64, 64, 8, 32, 2, true)});
    (void)hipEventRecord(e, b);
    (void)hipStreamWaitEvent(a, e, 0);
    std::printf("(the next FAILED line is the planted race being found)\n");
    check_call(0, a, 1, false);
    if (g_failures == before + 1) g_failures = before;
    else { std::printf("the race check did not find the planted race\n"); ++g_failures; }
    // ... and two windows of one matrix that do not meet (different column ranges) are not a race
    g_ops.clear();
    (void)hipEventRecord(e, a);
    (void)hipStreamWaitEvent(b, e, 0);
    launch(a, "piece 0", {reg(buf, 64, 8, 32, 2, true)});
    launch(b, "piece 1", {reg(buf + 64, 64, 8, 32, 2, true)});
    (void)hipEventRecord(e, b);
    (void)hipStreamWaitEvent(a, e, 0);
    check_call(0, a, 1, false);
  }
  domino_shutdown();
  std::printf(g_failures ? "host schedule driver: %d expectation(s) failed over %d cases\n" : "host schedule driver: ok (%d cases)\n",
              g_failures ? g_failures : cases, cases);
  return g_failures ? 1 : 0;
}
