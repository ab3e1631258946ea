// Internal interface between the GEMM C-ABI entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

struct GemmParams {
  const void* a;  // bf16 [M, K]
  const void* b;  // bf16 [N, K] (nt kernels) or [K, N] (nn kernels)
  void* c;        // bf16 [M, N]
  int M, N, K;
  int tiles_m, tiles_n;
  // split-K launches only: split s of `splits` contracts k in [s * klen, min(K, (s + 1) * klen)) and
  // writes its fp32 partial tile to partial[s][M][N]; a second kernel sums the splits into c
  float* partial = nullptr;
  int splits = 1;
  int klen = 0;
  int stream_c = 0;  // non-zero: C is written with non-temporal stores (it is not read again and should not displace the operands in the L2)
};

struct GemmVariant {
  const char* name;
  int bm, bn, bk;
  int kmult;  // K must be a multiple of this (some kernels run their k-stages in pairs)
  int (*launch)(const GemmParams& p, hipStream_t stream);
};

const GemmVariant* gemm_bf16_nt_variants(int* count);
const GemmVariant* gemm_bf16_nn_variants(int* count);  // second operand stored [K, N]
// 256 x 256 tiles, K split over p.splits workgroups per tile (p.klen a multiple of 64), then the sum
int gemm_bf16_nt_splitk_launch(const GemmParams& p, hipStream_t stream);
