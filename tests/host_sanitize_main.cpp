// Host-only driver for the sanitizer build of the library's host code (argument validation, layouts, the
// error paths of the entry points): every call below returns before any GPU call, so the program runs on a
// host without a GPU.  Exit status 0 = every expectation held; the sanitizers abort on their own findings.
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../include/domino.h"

static int failures = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { std::printf("FAILED: %s (line %d)\n", #cond, __LINE__); ++failures; } \
  } while (0)

static domino_cfg tiny() {
  domino_cfg c{};
  c.hidden = 256; c.heads = 4; c.tp = 2; c.rank = 0; c.p = 2; c.q = 2; c.batch = 2; c.seq = 128; c.ffn = 1024;
  c.arch = DOMINO_ARCH_GPT; c.gelu_tanh = 1; c.norm_eps = 1e-5f; c.rope_base = 10000.0f;
  return c;
}

static void validation_paths() {
  domino_cfg c = tiny();
  EXPECT(domino_validate_cfg(&c) == DOMINO_OK);
  EXPECT(domino_validate_cfg(nullptr) == DOMINO_ERR_NULL_POINTER);
  EXPECT(domino_saved_bytes(&c) > 0 && domino_workspace_bytes(&c) > 0);
  EXPECT(domino_stack_workspace_bytes(&c, 3) > domino_workspace_bytes(&c));
  EXPECT(domino_stack_workspace_bytes(&c, 0) == 0);
  size_t off = 0, bytes = 0;
  EXPECT(domino_saved_slot(&c, "lse", &off, &bytes) == DOMINO_OK && bytes == 2u * 2 * 128 * 4);
  EXPECT(domino_saved_slot(&c, "nope", &off, &bytes) == DOMINO_ERR_INVALID_ARG);
  EXPECT(std::strlen(domino_last_error()) > 0);
  for (int p = 1; p <= 9; ++p) {
    domino_cfg d = tiny();
    d.p = p; d.batch = 8;
    EXPECT(domino_validate_cfg(&d) == (8 % p ? DOMINO_ERR_INDIVISIBLE : DOMINO_OK));
  }
  domino_cfg big = tiny();
  big.hidden = 8192; big.heads = 64; big.tp = 8; big.ffn = 32768; big.batch = 64; big.seq = 4096; big.p = 8; big.q = 4;
  EXPECT(domino_validate_cfg(&big) == DOMINO_ERR_UNSUPPORTED);         // an activation tensor would reach 2 GiB
  big.batch = 8; big.seq = 2048;
  EXPECT(domino_validate_cfg(&big) == DOMINO_OK);
  EXPECT(domino_saved_bytes(&big) > (size_t)1 << 30);

  // layer calls with dummy pointers: each must fail in validation, before any pointer is used
  void* one = reinterpret_cast<void*>(0x1000);
  domino_params P{one, one, one, one, one, one, one, one, one, one, one, one};
  float* fone = reinterpret_cast<float*>(0x1000);
  domino_grads G{fone, fone, fone, fone, fone, fone, fone, fone, fone, fone, fone, fone};
  void* streams[1] = {nullptr};
  EXPECT(domino_layer_fwd(&c, &P, nullptr, nullptr, nullptr, one, one, nullptr, one, one, (size_t)1 << 40, streams, 1) == DOMINO_ERR_NULL_POINTER);
  EXPECT(domino_layer_fwd(&c, &P, one, nullptr, nullptr, one, one, nullptr, one, one, 16, streams, 1) == DOMINO_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(domino_layer_fwd(&c, &P, one, nullptr, nullptr, one, one, nullptr, one, one, (size_t)1 << 40, streams, 0) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_layer_fwd(&c, &P, one, nullptr, nullptr, one, one, nullptr, one, one, (size_t)1 << 40, nullptr, 1) == DOMINO_ERR_NULL_POINTER);
  EXPECT(domino_layer_fwd_parts(&c, &P, one, nullptr, nullptr, one, one, nullptr, one, one, (size_t)1 << 40, streams, 1, 8) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_layer_bwd(&c, &P, one, one, nullptr, nullptr, nullptr, one, one, one, &G, 0, one, (size_t)1 << 40, streams, 1) == DOMINO_ERR_NULL_POINTER);
  EXPECT(domino_layer_bwd(&c, &P, one, one, one, nullptr, nullptr, one, one, one, nullptr, 0, one, (size_t)1 << 40, streams, 1) == DOMINO_ERR_NULL_POINTER);
  domino_stack_fwd_io fio[2] = {};
  EXPECT(domino_stack_fwd(&c, 2, &P, one, fio, one, (size_t)1 << 40, streams, 1) == DOMINO_ERR_NULL_POINTER);
  EXPECT(domino_stack_fwd(&c, 2000, &P, one, fio, one, (size_t)1 << 40, streams, 1) == DOMINO_ERR_INVALID_ARG);
  domino_stack_bwd_io bio[2] = {};
  EXPECT(domino_stack_bwd(&c, 2, &P, one, bio, one, &G, 0, one, 8, streams, 1) == DOMINO_ERR_WORKSPACE_TOO_SMALL);

  // single-kernel entry points
  EXPECT(domino_gemm(DOMINO_GEMM_NN, DOMINO_EPI_ACC_F32, -1, one, 64, one, 64, one, 64, 64, 64, 64, nullptr, nullptr, 0, 0, 0, 1, nullptr) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_gemm(DOMINO_GEMM_NN, DOMINO_EPI_STORE, -1, one, 64, one, 64, one, 64, 60, 64, 64, nullptr, nullptr, 0, 0, 0, 1, nullptr) == DOMINO_ERR_UNSUPPORTED);
  EXPECT(domino_norm_fwd(one, nullptr, nullptr, nullptr, one, nullptr, nullptr, one, nullptr, fone, 4, 12, 0, 1e-5f, nullptr) == DOMINO_ERR_UNSUPPORTED);
  EXPECT(domino_norm_bwd_scratch_floats(2048, 5120) == 2u * 128 * 5120);
  EXPECT(domino_attention_fwd(one, 100, 1, 16, 1, 64, one, fone, nullptr) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_rope(one, 64, 4, 4, 0, 2, 1, 64, 10000.0f, 0, nullptr) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_colsum(one, 64, 4, 60, fone, 0, fone, nullptr) == DOMINO_ERR_UNSUPPORTED);
  EXPECT(domino_colsum_noalloc(one, 16384, 4, 16384, fone, 0, nullptr) == DOMINO_ERR_UNSUPPORTED);
  EXPECT(domino_mfma_probe(one, one, fone, 0, 1, nullptr, nullptr) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_capture_supported(4, 4) == 1 && domino_capture_supported(3, 4) == 0);
  double ms = 0.0;
  int n = 0;
  EXPECT(domino_profile_read(0, &ms, &n) == DOMINO_OK && n == 0);
  EXPECT(domino_profile_read(999, &ms, &n) == DOMINO_ERR_INVALID_ARG);
  EXPECT(domino_profile_records() == 0);
  EXPECT(std::strlen(domino_last_warning()) == 0);
}

int main() {
  validation_paths();
  // the error text is thread-local and the checks are re-entrant: several host threads at once
  std::vector<std::thread> th;
  for (int t = 0; t < 4; ++t) th.emplace_back(validation_paths);
  for (auto& t : th) t.join();
  domino_shutdown();
  std::printf(failures ? "host sanitize driver: %d expectation(s) failed\n" : "host sanitize driver: ok\n", failures);
  return failures ? 1 : 0;
}
