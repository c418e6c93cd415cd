// Internal launcher interface of the MFMA-only probe (see probe.hip).
#pragma once
#include <hip/hip_runtime.h>

constexpr double MFMA_PROBE_FLOPS_PER_WAVE_ITER = 8.0 * 2.0 * 32 * 32 * 16;
// a, b: bf16 [256 * 8]; out: fp32 [blocks * 256]
hipError_t mfma_probe_launch(const void* a, const void* b, float* out, int blocks, int iters, hipStream_t st);
