// C-ABI entry points of the bf16 GEMM: argument checks, kernel choice, launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm.h"
#include "gemm_kernels.h"
#include "gemm_map.h"

namespace {

bool misaligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

int run(const void* a, const void* b, void* c, int M, int N, int K, int variant, void* stream) {
  if (!a || !b || !c) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0 || K <= 0) return ATTN_ERR_SHAPE;
  if (misaligned(a, 16) || misaligned(b, 16) || misaligned(c, 16)) return ATTN_ERR_SHAPE;
  int count = 0;
  const GemmVariant* table = gemm_bf16_nt_variants(&count);
  if (variant < 0 || variant >= count) return ATTN_ERR_UNSUPPORTED;
  const GemmVariant& v = table[variant];
  if (K % v.bk != 0) return ATTN_ERR_UNSUPPORTED;
  // per-lane offsets inside an operand panel are 32-bit: 256 rows of K bf16
  if ((long long)K * 2 * 256 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  GemmParams p;
  p.a = a; p.b = b; p.c = c;
  p.M = M; p.N = N; p.K = K;
  p.tiles_m = (M + v.bm - 1) / v.bm;
  p.tiles_n = (N + v.bn - 1) / v.bn;
  if ((long long)p.tiles_m * p.tiles_n > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  return v.launch(p, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int gemm_bf16_nt(const void* a, const void* b, void* c, int M, int N, int K, void* stream) {
  return run(a, b, c, M, N, K, 0, stream);
}

int gemm_bf16_nt_variant(const void* a, const void* b, void* c, int M, int N, int K, int variant, void* stream) {
  return run(a, b, c, M, N, K, variant, stream);
}

int gemm_num_variants(void) {
  int count = 0;
  gemm_bf16_nt_variants(&count);
  return count;
}

const char* gemm_variant_name(int variant) {
  int count = 0;
  const GemmVariant* table = gemm_bf16_nt_variants(&count);
  return variant >= 0 && variant < count ? table[variant].name : nullptr;
}

int gemm_num_workgroups(int M, int N) {
  if (M <= 0 || N <= 0) return 0;
  return ((M + 255) / 256) * ((N + 255) / 256);
}

int gemm_tile_coord(int wg, int M, int N, int* tm, int* tn) {
  if (!tm || !tn) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0) return ATTN_ERR_SHAPE;
  const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
  if (wg < 0 || wg >= tiles_m * tiles_n) return ATTN_ERR_SHAPE;
  const GemmTileCoord c = gemm_tile_coord_impl(wg, tiles_m, tiles_n);
  *tm = c.tm;
  *tn = c.tn;
  return ATTN_OK;
}
}
