// Internal launcher interface of the attention kernels (see attention.hip).
#pragma once
#include <hip/hip_runtime.h>

struct AttnArgs {
  const void* qkv;     // bf16 [batch*seq, ld]: q | k | v column blocks, heads contiguous inside a block
  long ld;
  void* ctx;           // bf16 [batch*seq, ld_ctx]: forward output / backward input
  long ld_ctx;
  const void* dctx;    // bf16 [batch*seq, ld_ctx] (backward)
  float* lse;          // fp32 [batch, heads, seq]
  float* dot;          // fp32 [batch, heads, seq]: rowsum(dctx * ctx) (backward scratch)
  void* dqkv;          // bf16 [batch*seq, ld] (backward output)
  int batch, seq, heads, head_dim;
  float scale;         // 1 / sqrt(head_dim)
  int rope;            // backward: q and k of qkv carry the rotary embedding; dq and dk are turned back before the store
  float rope_log2_base;
};

hipError_t attention_fwd_launch(const AttnArgs& a, hipStream_t st);
hipError_t attention_bwd_launch(const AttnArgs& a, hipStream_t st);
