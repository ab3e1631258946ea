// C-ABI entry points of the bf16 GEMM: argument checks, kernel choice, launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm.h"
#include "gemm_kernels.h"
#include "gemm_map.h"

namespace {

bool misaligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

// Kernel choice, from measurements on the paper's shapes: the 256 x 256 tile (best rate per CU)
// when it gives most of the 256 CUs a tile; the 128 x 128 tile with a deep ring when that yields
// at least 100 tiles (it then beats both the half-empty chip of the large tile and the operand
// re-reads of the small one); else 64 x 64.
int find(const GemmVariant* table, int count, int tile, int bk, int nth) {
  for (int i = 0; i < count; ++i)
    if (table[i].bm == tile && table[i].bk == bk && nth-- == 0) return i;
  return -1;
}

int choose(int M, int N, int K, const GemmVariant* table, int count) {
  auto tiles = [&](int t) { return (long long)((M + t - 1) / t) * ((N + t - 1) / t); };
  int v = -1;
  // (256 tile: the 16x16x32 MFMA form is 2-4 % faster at the same power; it runs its stages in pairs)
  // (with at most four of its k-stages the ring of two 64-column stages starts and drains faster
  // than the ring of four 32-column ones: 8-12 % on the K <= 256 shapes of the paper's tables)
  if (tiles(256) >= 200) v = K % 64 == 0 && K <= 256 ? find(table, count, 256, 64, 1) : find(table, count, 256, 32, K % 64 == 0 ? 1 : 0);
  else if (tiles(128) >= 100 && K % 64 == 0) v = find(table, count, 128, 64, 1);
  if (v < 0) v = find(table, count, 64, 32, 0);
  return v;
}

// Non-temporal stores of C in gemm_bf16_nt, measured on the paper's shapes (interleaved, one
// process): they pay where C's rows are short and the product is bound by memory traffic (442368 x
// 448 x 192: +11 %, 589824 x 256 x 128: +3 %) and where a long contraction makes C a small part of
// the traffic that should not displace operand panels in the L2 (8192 x 8192 x 8192 / 16384: +3 %);
// elsewhere they cost (8192 x 8192 x 1024: -8 %, 2048 x 64512 x 256: -9 %, 589824 x 512 x 2048:
// -5 %), and in gemm_bf16_nn they cost at every size tried (-2 .. -3 %), so that entry keeps plain stores.
int stream_c_pays(int M, int N, int K) {
  (void)M;
  return ((N <= 512 && K <= 256) || K >= 8192) ? 1 : 0;
}

int run(const void* a, const void* b, void* c, int M, int N, int K, int variant, void* stream) {
  if (!a || !b || !c) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0 || K <= 0) return ATTN_ERR_SHAPE;
  if (misaligned(a, 16) || misaligned(b, 16) || misaligned(c, 16)) return ATTN_ERR_SHAPE;
  int count = 0;
  const GemmVariant* table = gemm_bf16_nt_variants(&count);
  if (K % 32 != 0) return ATTN_ERR_UNSUPPORTED;
  if (variant == -1) variant = choose(M, N, K, table, count);
  if (variant < 0 || variant >= count) return ATTN_ERR_UNSUPPORTED;
  const GemmVariant& v = table[variant];
  if (K % v.bk != 0 || K % v.kmult != 0) return ATTN_ERR_UNSUPPORTED;
  // per-lane offsets inside an operand panel are 32-bit: 256 rows of K bf16
  if ((long long)K * 2 * 256 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  GemmParams p;
  p.a = a; p.b = b; p.c = c;
  p.M = M; p.N = N; p.K = K;
  p.tiles_m = (M + v.bm - 1) / v.bm;
  p.tiles_n = (N + v.bn - 1) / v.bn;
  if ((long long)p.tiles_m * p.tiles_n > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  p.stream_c = stream_c_pays(M, N, K);
  return v.launch(p, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int run_nn(const void* a, const void* b, void* c, int M, int N, int K, void* stream) {
  if (!a || !b || !c) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0 || K <= 0) return ATTN_ERR_SHAPE;
  if (misaligned(a, 16) || misaligned(b, 16) || misaligned(c, 16)) return ATTN_ERR_SHAPE;
  if (K % 32 != 0 || N % 8 != 0) return ATTN_ERR_UNSUPPORTED;
  if ((long long)K * 2 * 256 >= (1ll << 31) || (long long)N * 2 * 64 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  int count = 0;
  const GemmVariant* table = gemm_bf16_nn_variants(&count);
  const long long tiles256 = (long long)((M + 255) / 256) * ((N + 255) / 256);
  const GemmVariant& v = table[tiles256 >= 200 ? 0 : 1];
  GemmParams p;
  p.a = a; p.b = b; p.c = c;
  p.M = M; p.N = N; p.K = K;
  p.tiles_m = (M + v.bm - 1) / v.bm;
  p.tiles_n = (N + v.bn - 1) / v.bn;
  if ((long long)p.tiles_m * p.tiles_n > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  return v.launch(p, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int run_splitk(const void* a, const void* b, void* c, int M, int N, int K, int splits, float* workspace, void* stream) {
  if (!a || !b || !c || !workspace) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0 || K <= 0 || splits < 1 || splits > 64) return ATTN_ERR_SHAPE;
  if (misaligned(a, 16) || misaligned(b, 16) || misaligned(c, 16) || misaligned(workspace, 16)) return ATTN_ERR_SHAPE;
  if (K % 64 != 0) return ATTN_ERR_UNSUPPORTED;
  if ((long long)K * 2 * 256 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  GemmParams p;
  p.a = a; p.b = b; p.c = c;
  p.M = M; p.N = N; p.K = K;
  p.tiles_m = (M + 255) / 256;
  p.tiles_n = (N + 255) / 256;
  // slices of whole 64-column steps, none empty
  const int steps = K / 64;
  p.klen = ((steps + splits - 1) / splits) * 64;
  p.splits = (K + p.klen - 1) / p.klen;
  p.partial = workspace;
  if ((long long)p.tiles_m * p.tiles_n * p.splits > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  return gemm_bf16_nt_splitk_launch(p, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int gemm_bf16_nt_splitk(const void* a, const void* b, void* c, int M, int N, int K, int splits, float* workspace, void* stream) {
  return run_splitk(a, b, c, M, N, K, splits, workspace, stream);
}

long long gemm_splitk_workspace_bytes(int M, int N, int splits) {
  if (M <= 0 || N <= 0 || splits <= 0) return 0;
  return (long long)splits * M * N * 4;
}

// Measured on the paper's large-K shapes: splitting pays when the 256 x 256 tiles leave at least half
// of the 256 CUs idle and every slice still has 2048 or more of k to amortise its prologue and the
// fp32 round trip of the partial tiles.
int gemm_splitk_plan(int M, int N, int K) {
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 != 0) return 1;
  const long long tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
  if (tiles > 128) return 1;
  long long s = 256 / tiles;
  if (s > K / 2048) s = K / 2048;
  if (s > 64) s = 64;
  return s < 2 ? 1 : (int)s;
}

int gemm_bf16_nn(const void* a, const void* b, void* c, int M, int N, int K, void* stream) {
  return run_nn(a, b, c, M, N, K, stream);
}

int gemm_bf16_nt(const void* a, const void* b, void* c, int M, int N, int K, void* stream) {
  return run(a, b, c, M, N, K, -1, stream);
}

int gemm_bf16_nt_variant(const void* a, const void* b, void* c, int M, int N, int K, int variant, void* stream) {
  if (variant < 0) return ATTN_ERR_UNSUPPORTED;
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

int gemm_variant_kmult(int variant) {
  int count = 0;
  const GemmVariant* table = gemm_bf16_nt_variants(&count);
  return variant >= 0 && variant < count ? table[variant].kmult : 0;
}

int gemm_variant_tile(int variant) {
  int count = 0;
  const GemmVariant* table = gemm_bf16_nt_variants(&count);
  return variant >= 0 && variant < count ? table[variant].bm : 0;
}

int gemm_num_workgroups(int M, int N, int tile) {
  if (M <= 0 || N <= 0 || tile <= 0) return 0;
  return ((M + tile - 1) / tile) * ((N + tile - 1) / tile);
}

int gemm_tile_coord(int wg, int M, int N, int tile, int* tm, int* tn) {
  if (!tm || !tn) return ATTN_ERR_NULL;
  if (M <= 0 || N <= 0 || tile <= 0) return ATTN_ERR_SHAPE;
  const int tiles_m = (M + tile - 1) / tile, tiles_n = (N + tile - 1) / tile;
  if (wg < 0 || wg >= tiles_m * tiles_n) return ATTN_ERR_SHAPE;
  const GemmTileCoord c = gemm_tile_coord_impl(wg, tiles_m, tiles_n);
  *tm = c.tm;
  *tn = c.tn;
  return ATTN_OK;
}
}
