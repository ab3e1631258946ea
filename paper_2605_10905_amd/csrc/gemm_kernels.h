// Internal interface between the GEMM C-ABI entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

struct GemmParams {
  const void* a;  // bf16 [M, K]
  const void* b;  // bf16 [N, K] (nt kernels) or [K, N] (nn kernels)
  void* c;        // bf16 [M, N]
  int M, N, K;
  int tiles_m, tiles_n;
};

struct GemmVariant {
  const char* name;
  int bm, bn, bk;
  int kmult;  // K must be a multiple of this (some kernels run their k-stages in pairs)
  int (*launch)(const GemmParams& p, hipStream_t stream);
};

const GemmVariant* gemm_bf16_nt_variants(int* count);
const GemmVariant* gemm_bf16_nn_variants(int* count);  // second operand stored [K, N]
