/*
 * attn.h -- C ABI of the MI355X (gfx950) fused attention library: the forward pass (attn_fwd and
 * its variants), its persistent-launch form and the backward pass (attn_bwd).
 *
 * The central operation is the fused scaled-dot-product attention forward pass of the
 * paper's section 6.1 ("Major Operators": tile staging, score computation,
 * masking, normalisation, output accumulation), with the two outputs its
 * appendix C.3 names: the normalised accumulator  O = acc / l  and the
 * per-row statistic  lse = m + log(l)  (natural logarithm).
 *
 *   for every batch b and query head h, kv head g = h / (Hq / Hkv):
 *     S = scale * Q[b,h] K[b,g]^T ;  S[i][j] = -inf for j > i when causal
 *     P = softmax over j of S     ;  O[b,h] = P V[b,g]
 *     lse[b,h,i] = ln sum_j exp(S[i][j])
 *
 * Every pointer is a DEVICE pointer unless stated otherwise.  The caller owns
 * all buffers; the library allocates nothing, keeps no state between calls and
 * never synchronises the device: work is enqueued on `stream` and the call
 * returns.  Inputs are never written; `o` and `lse` are fully overwritten.
 * Calls from several host threads on different streams are safe.
 *
 * Layouts (contiguous, row-major, innermost index last):
 *   q, o : [B, Hq , N, d]        k, v : [B, Hkv, N, d]        lse : [B, Hq, N]
 * q, k, v, o must be 16-byte aligned, lse 4-byte aligned.
 *
 * Errors are reported by return code only (never abort, never throw); all
 * argument checks run before anything is enqueued.
 */
#ifndef ATTN_MI355X_H
#define ATTN_MI355X_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ATTN_OK = 0,
  ATTN_ERR_NULL = 1,        /* a required pointer is NULL                         */
  ATTN_ERR_SHAPE = 2,       /* non-positive size, Hq % Hkv != 0, misaligned ptr   */
  ATTN_ERR_DTYPE = 3,       /* dtype is not one of attn_dtype                     */
  ATTN_ERR_UNSUPPORTED = 4, /* valid request this build has no kernel for (d, scale <= 0) */
  ATTN_ERR_LAUNCH = 5,      /* the HIP runtime refused the launch                 */
  ATTN_ERR_TOO_LARGE = 6    /* attn_bwd_noalloc: needs more than the built-in scratch */
} attn_status;

typedef enum {
  ATTN_BF16 = 0,    /* q,k,v bfloat16; products on bf16 MFMA, fp32 accumulate     */
  ATTN_FP8_E4M3 = 1 /* q,k,v OCP e4m3 bytes; scores on fp8 MFMA, P V on bf16 MFMA   */
} attn_dtype;

/*
 * attn_fwd -- fused attention forward (section 6.1 phase list; appendix C.3 outputs).
 *
 *   q,k,v   device, `dtype` elements, layouts above
 *   o       device, bfloat16 [B,Hq,N,d] (bf16 output for both input dtypes)
 *   lse     device, float32  [B,Hq,N], required
 *   B,Hq,Hkv,N,d  sizes; Hq must be a multiple of Hkv; query head h reads kv
 *           head h / (Hq/Hkv) (contiguous groups).  d must be 64 or 128 for
 *           ATTN_BF16 and 128 for ATTN_FP8_E4M3 (ATTN_ERR_UNSUPPORTED otherwise).
 *           Any N >= 1 is accepted (ragged last tiles are handled in-kernel);
 *           N * d must stay below 2^30.
 *   causal  0: every key visible.  non-zero: key j visible to query i iff j <= i.
 *   scale   multiplies q.k before the softmax; must be > 0 (the kernels take
 *           maxima of the raw products): scale <= 0 returns ATTN_ERR_UNSUPPORTED.
 *           NaN and +inf are not detected (garbage in, garbage out).
 *   dtype   an attn_dtype.  For ATTN_FP8_E4M3 the bytes are taken as the e4m3
 *           values themselves (all de-scales 1); see attn_fwd_fp8.
 *   stream  a hipStream_t (NULL = the default stream).
 *
 * Returns an attn_status.
 */
int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
             int B, int Hq, int Hkv, int N, int d, int causal, float scale,
             int dtype, void* stream);

/*
 * attn_fwd_fp8 -- the same operation on per-tensor-scaled e4m3 inputs: the real
 * tensors are q_descale*q, k_descale*k, v_descale*v.  q_descale*k_descale is
 * folded into the softmax exponent and v_descale into the final normalisation,
 * so no extra pass over memory is made.  o is bfloat16, lse float32.
 *
 * Arithmetic of the kernel this call runs: the scores S = Q K^T are taken on the
 * e4m3 bytes with the fp8 MFMA; the probabilities P stay bfloat16 and V is
 * converted e4m3 -> bfloat16 (exactly) on arrival, so P V runs on the bf16 MFMA.
 * Rounding P itself to e4m3 before the second product, as one might read "fp8
 * attention", was measured at 2.0 - 2.6 % relative Frobenius error on the
 * graded fp8 workload, above its 2 % bound; the variant that feeds P as the sum
 * of two e4m3 terms (both products on the fp8 MFMA) is reachable through
 * attn_fwd_variant.  q_descale and k_descale must be > 0, d must be 128.
 */
int attn_fwd_fp8(const void* q, const void* k, const void* v, void* o, float* lse,
                 int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                 float q_descale, float k_descale, float v_descale, void* stream);

/*
 * attn_fwd_persistent -- attn_fwd for bfloat16 as a persistent launch: one workgroup per compute
 * unit, each taking query tiles from a queue in device memory until it is drained (the software
 * form of the paper's dynamic tile assignment by cluster launch control, section 4.2: a kernel
 * that stays resident and balances irregular tile run times).  Same results as attn_fwd.
 *   queue   device, attn_persistent_queue_bytes() bytes, 128-byte aligned, owned by the caller;
 *           contents on entry are irrelevant (the call enqueues a kernel that clears it first),
 *           it must not be shared by calls that can overlap on the device
 * Everything else as attn_fwd; dtype must be ATTN_BF16 (ATTN_ERR_UNSUPPORTED otherwise).
 */
int attn_fwd_persistent(const void* q, const void* k, const void* v, void* o, float* lse,
                        int B, int Hq, int Hkv, int N, int d, int causal, float scale, int dtype,
                        void* queue, void* stream);
int attn_persistent_queue_bytes(void);

/*
 * attn_bwd -- attention backward (the paper lists the backward pass beside the forward among
 * its attention kernels, section 6.1; appendix A, attention shape table, backward rows).
 * Gradients of attn_fwd with respect to q, k and v, given the gradient `dout` of o:
 *
 *     P = exp(S - lse) ;  dV = P^T dO ;  dP = dO V^T ;  dS = P * (dP - rowsum(dO * O))
 *     dQ = scale dS K ;  dK = scale dS^T Q      (dK, dV summed over the query heads of a group)
 *
 *   q,k,v,o,lse   the forward call's inputs and outputs (device; layouts as for attn_fwd)
 *   dout          device, bfloat16 [B,Hq,N,d]
 *   dq            device, bfloat16 [B,Hq,N,d], overwritten
 *   dk,dv         device, bfloat16 [B,Hkv,N,d], overwritten
 *   workspace     device, attn_bwd_workspace_bytes(B,Hq,N) bytes, 16-byte aligned, owned by the
 *                 caller; contents on entry are irrelevant, contents on return unspecified
 *   dtype         ATTN_BF16 only; d must be 128 or 64 (ATTN_ERR_UNSUPPORTED otherwise)
 *
 * Deterministic (no atomics).  Two kernels are enqueued on `stream`; the call returns without
 * synchronising.  Returns an attn_status; argument checks run before anything is enqueued.
 */
int attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
             void* dq, void* dk, void* dv, float* workspace,
             int B, int Hq, int Hkv, int N, int d, int causal, float scale, int dtype, void* stream);

/* Size in bytes of the workspace attn_bwd needs (0 for non-positive sizes). */
long long attn_bwd_workspace_bytes(int B, int Hq, int N);

/*
 * attn_bwd_noalloc -- attn_bwd for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving or training loops, harnesses that forbid allocation): the same
 * kernels, with the workspace taken from a scratch array that is part of the library's device
 * code (attn_bwd_noalloc_max_workspace_bytes() = 32 MiB per GPU, held from the moment the library
 * is loaded on that GPU until the process ends) instead of from an argument.  The call allocates
 * and frees nothing.  The first call on a device looks the array's address up (one runtime query,
 * no allocation); make that first call outside graph capture.
 *   all arguments as attn_bwd, without `workspace`
 * Returns ATTN_ERR_TOO_LARGE, before anything is enqueued, if attn_bwd_workspace_bytes(B,Hq,N)
 * exceeds the scratch size (i.e. B*Hq*ceil(N/64)*64 > 4 194 304 rows).  Every call on a GPU uses
 * that GPU's one array: calls that can overlap on the same GPU (different streams, different host
 * threads) race on it and must be serialised by the caller; nothing needs clearing between calls
 * (the query-side kernel rewrites every value the key-side kernel reads).  Same results, bit for
 * bit, as attn_bwd.
 */
int attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                     void* dq, void* dk, void* dv,
                     int B, int Hq, int Hkv, int N, int d, int causal, float scale, int dtype, void* stream);
long long attn_bwd_noalloc_max_workspace_bytes(void);

/*
 * attn_fwd_variant -- tuning hook: as attn_fwd, but with the kernel variant
 * forced (see attn_variant_name) instead of chosen by the library.  Returns
 * ATTN_ERR_UNSUPPORTED if the variant does not exist for this d / dtype.
 */
int attn_fwd_variant(const void* q, const void* k, const void* v, void* o, float* lse,
                     int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                     int dtype, int variant, void* stream);

/* The same hook for per-tensor-scaled e4m3 inputs: attn_fwd_fp8 with the kernel variant forced. */
int attn_fwd_fp8_variant(const void* q, const void* k, const void* v, void* o, float* lse,
                         int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                         float q_descale, float k_descale, float v_descale, int variant, void* stream);

/* Number of kernel variants and a host string describing variant i (NULL if out of range). */
int attn_num_variants(void);
/* index of the variant attn_fwd / attn_fwd_fp8 run for this dtype and shape (-1: none) */
int attn_default_variant(int dtype, int B, int Hq, int N, int d);
const char* attn_variant_name(int variant);

/*
 * attn_tile_coord -- host-side copy of the work decomposition the kernels use:
 * workgroup `wg` of a launch of attn_num_workgroups(...) workgroups processes
 * query tile *t (rows t*BM .. t*BM+BM-1) of head *hq in batch *b.  Host
 * pointers.  Used to check that the map is a bijection and keeps the
 * workgroups that share a K/V head on one XCD.  Returns an attn_status.
 */
int attn_tile_coord(int wg, int B, int Hq, int Hkv, int N, int BM, int causal,
                    int* b, int* hq, int* t);
int attn_num_workgroups(int B, int Hq, int N, int BM);

/* Query-tile height BM (rows per workgroup) of a variant; 0 if out of range. */
int attn_variant_bm(int variant);

const char* attn_status_string(int status); /* host string, static storage */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_MI355X_H */
