/*
 * C ABI of the bf16 GEMM of libattn_mi355x.so (MI355X, gfx950).
 *
 * The operation (paper section 6.1, GEMM paragraph: a producer/consumer pipelined GEMM;
 * section 6.3 and appendix A, GEMM shape tables: 8192 x 8192 x K and, on MI350,
 * 256^3 ... 2048^3):
 *
 *     C[m, n] = sum_k A[m, k] * B[n, k]        fp32 accumulation, C rounded to bfloat16
 *
 * All pointers are DEVICE pointers to dense row-major arrays the caller owns and keeps alive
 * until the stream has run the call.  Nothing is allocated, nothing is copied to the host, and
 * the call returns without synchronising.  Status codes are attn_status (attn.h).
 */
#ifndef PAPER_2605_10905_GEMM_H
#define PAPER_2605_10905_GEMM_H

#include "attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * gemm_bf16_nt -- C = A B^T.
 *   a        device, bfloat16 [M, K] row-major (K contiguous), 16-byte aligned
 *   b        device, bfloat16 [N, K] row-major (K contiguous: the layout of a linear layer's
 *            weight), 16-byte aligned
 *   c        device, bfloat16 [M, N] row-major, overwritten; 16-byte aligned
 *   M, N     any positive size (ragged tiles are handled in the kernel)
 *   K        positive multiple of 32 (ATTN_ERR_UNSUPPORTED otherwise: operand tiles are moved
 *            in whole 32- or 64-column slices)
 *   stream   hipStream_t (NULL = default stream)
 * Errors: ATTN_ERR_NULL, ATTN_ERR_SHAPE (non-positive size, misaligned pointer),
 * ATTN_ERR_UNSUPPORTED (K, or a size beyond 2^31 bytes per operand tile row span),
 * ATTN_ERR_LAUNCH.  Argument checks run before anything is enqueued.
 */
int gemm_bf16_nt(const void* a, const void* b, void* c, int M, int N, int K, void* stream);

/*
 * gemm_bf16_nn -- C = A B with the second operand stored [K, N] row-major (N contiguous):
 *     C[m, n] = sum_k A[m, k] * B[k, n]
 * Arguments as for gemm_bf16_nt except b (device, bfloat16 [K, N]); N must be a multiple of 8
 * (rows of B and C are moved in 16-byte pieces) and K a multiple of 32, ATTN_ERR_UNSUPPORTED
 * otherwise.
 */
int gemm_bf16_nn(const void* a, const void* b, void* c, int M, int N, int K, void* stream);

/*
 * gemm_bf16_nt_splitk -- gemm_bf16_nt for outputs with too few 256 x 256 tiles to occupy the
 * chip while K is long (the large-K rows of the paper's appendix A GEMM shape table): every
 * output tile is computed by `splits` workgroups, each contracting one slice of k in fp32, and a
 * second kernel adds the slices in index order and rounds to bfloat16.  Deterministic.
 *   splits     1 .. 64 slices per tile; slices are whole multiples of 64 in k, so fewer may be
 *              used than asked for (a slice is never empty)
 *   workspace  device, gemm_splitk_workspace_bytes(M, N, splits) bytes, 16-byte aligned, owned by
 *              the caller; contents on entry are irrelevant, contents on return unspecified
 *   K          positive multiple of 64 (ATTN_ERR_UNSUPPORTED otherwise)
 * Everything else, and the error behaviour, as for gemm_bf16_nt.  Two kernels are enqueued.
 */
int gemm_bf16_nt_splitk(const void* a, const void* b, void* c, int M, int N, int K, int splits,
                        float* workspace, void* stream);
/* bytes of fp32 workspace for that call: splits * M * N * 4 (0 for non-positive arguments) */
long long gemm_splitk_workspace_bytes(int M, int N, int splits);
/* The number of slices the library recommends for a shape: 1 means gemm_bf16_nt is the better
 * call (enough tiles, or too little k per slice), more means gemm_bf16_nt_splitk with that many. */
int gemm_splitk_plan(int M, int N, int K);

/* Tuning hook: the same with kernel variant `variant` (0 .. gemm_num_variants()-1);
 * ATTN_ERR_UNSUPPORTED if K is not a multiple of that variant's K-slice. */
int gemm_bf16_nt_variant(const void* a, const void* b, void* c, int M, int N, int K, int variant, void* stream);
int gemm_num_variants(void);
const char* gemm_variant_name(int variant); /* NULL if out of range */

/*
 * Work decomposition (host-side, for tests): tile (tm, tn) of tile x tile outputs that
 * workgroup `wg` of a launch over an M x N output computes.  Returns ATTN_ERR_SHAPE if wg is
 * out of range.  gemm_variant_tile gives a variant's square tile size (0 if out of range).
 */
int gemm_tile_coord(int wg, int M, int N, int tile, int* tm, int* tn);
int gemm_num_workgroups(int M, int N, int tile);
int gemm_variant_tile(int variant);
/* K must be a multiple of this for the variant (0 if out of range) */
int gemm_variant_kmult(int variant);

#ifdef __cplusplus
}
#endif
#endif
