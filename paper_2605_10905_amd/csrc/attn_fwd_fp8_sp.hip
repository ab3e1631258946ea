// Fused attention forward, fp8 (OCP e4m3) inputs, gfx950: the software-pipelined kernel.
//
// Same operation and the same numerics as attn_fwd_fp8.hip (paper section 6.1 phases,
// appendix C.3 outputs; both products on the 32x32x64 f8f6f4 MFMA, transposed so that a lane
// holds one query; P enters the second product as the sum of two e4m3 terms; the row sum is
// taken in fp32 from the unrounded exponentials).  What differs is the orchestration, which
// follows the bf16 pipelined kernel:
//
//   * One step handles one 64-key tile j and carries three independent instruction streams:
//         vector:  P(j)    = 2^6 exp2(c S(j) - m), split into two e4m3 terms
//         matrix:  S(j+1)  = K(j+1) Q^T                      (4 MFMAs)
//         matrix:  O^T    += V(j-1)^T (P_hi + P_lo)(j-1)^T   (8 MFMAs)
//     A scheduling-group pipeline at the end of the step tells the compiler's scheduler how to
//     interleave them (per MFMA: its share of the vector work, two or three exponentials, two
//     LDS reads).  The fp8 path is bound by the vector pipe (5.5 vector instructions per score
//     against half the matrix time of bf16), so what matters is that the matrix work hides
//     completely underneath.
//   * No tile maximum on the common path: exponentials are taken against the current reference;
//     if a lane's partial row sum exceeds 448 (then, and only then, some 2^6-scaled exponential
//     could exceed the e4m3 range) or is not a number (first tile), the true maximum is taken,
//     the reference raised, the accumulator rescaled and the tile redone.
//   * K and V stream through two four-slot LDS rings (tile t in slot t mod 4) by direct-to-LDS
//     loads: K(j+4) and V(j+2) are requested at the start of step j and published by the
//     barrier that ends step j+1, so step j may already read the first operands of step j+1
//     (K(j+2), V(j)).  One workgroup barrier per tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) int i32x2;

template <int V>
using ic = std::integral_constant<int, V>;

constexpr float kPShift = 6.0f;      // P is stored as 2^6 * exp2(.)
constexpr float kSumLimit = 448.0f;  // largest finite e4m3 value: a 32-term partial sum below it bounds every term

// 16-byte-chunk swizzle of the V tile for the 8-bit transposing load (see attn_fwd_fp8.hip)
__device__ __forceinline__ constexpr int swz_v8(int row) { return ((row >> 1) & 1) | (((row >> 3) & 1) << 1); }

// Scheduling-group pipeline of one step: NM MFMAs, each followed by its share of the NVALU
// plain vector instructions, of the 32 exponentials and two LDS reads.
template <int M, int NM, int NVALU>
__device__ __forceinline__ void fp8_step_pipeline() {
  if constexpr (M < NM) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (M + 1)) / NM - (NVALU * M) / NM, 0);
    __builtin_amdgcn_sched_group_barrier(0x400, (32 * (M + 1)) / NM - (32 * M) / NM, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    fp8_step_pipeline<M + 1, NM, NVALU>();
  }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 2) attn_fwd_fp8_sp_kernel(const AttnParams p) {
  static_assert(D == 128, "fp8 path is built for head dimension 128");
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int ROWB = D;           // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row (8)
  constexpr int NKK = D / 64;       // MFMA k-steps of S^T = K Q^T (2)
  constexpr int NCB = D / 32;       // 32-row blocks of O^T (4)
  constexpr int TILEB = BN * ROWB;  // 8 KB
  constexpr int NSLOT = 4;
  constexpr int VBASE = NSLOT * TILEB;
  static_assert(BN * NCH == NT, "one 16-byte chunk per thread per tile");

  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31, h = lane >> 5;

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  const int hk = tc.hq / G;
  const int q0 = tc.t * BM;
  const int wq0 = q0 + w * 32;
  const bool wave_valid = wq0 < N;

  const char* const qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;  // keys the workgroup visits
  const int nt = (kv_end + BN - 1) / BN;            // 64-key tiles
  // last tile some query of this wave can see (-1: none)
  const int jl = wave_valid ? min(nt - 1, (CAUSAL ? min(wq0 + 31, N - 1) : N - 1) / BN) : -1;

  // ---- producer role: one direct-to-LDS 16-byte load per thread per tile and tensor --------
  const int ld_row = tid / NCH, ld_c = tid % NCH;
  const uint32_t ld_koff = ld_row * ROWB + ((ld_c ^ attn_swz_k<ROWB>(ld_row)) << 4);
  const uint32_t ld_voff = ld_row * ROWB + ((ld_c ^ swz_v8(ld_row)) << 4);
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_k = [&](int t, int slot) __attribute__((always_inline)) {
    const uint32_t over = (uint32_t)max(0, t * BN + ld_row - (N - 1)) * ROWB;  // rows past N-1 re-read row N-1
    attn_lds_dma16(khead + (size_t)t * TILEB, ld_koff - over, lds_wave + slot * TILEB);
  };
  auto issue_v = [&](int t, int slot) __attribute__((always_inline)) {
    const uint32_t over = (uint32_t)max(0, t * BN + ld_row - (N - 1)) * ROWB;
    attn_lds_dma16(vhead + (size_t)t * TILEB, ld_voff - over, lds_wave + VBASE + slot * TILEB);
  };
  issue_k(0, 0);

  // ---- Q operand: lane (qi,h) holds Q[row][64kk + 32h .. +31] -------------------------------
  i32x8 qf[NKK];
  {
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * ROWB + h * 32;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const u32x4 lo = *(const u32x4*)(src + kk * 64), hi = *(const u32x4*)(src + kk * 64 + 16);
      qf[kk] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
  }
  // prologue loads, oldest first: K0 Q K1 V0 K2 V1 K3
  if (nt > 1) issue_k(1, 1);
  issue_v(0, 0);
  if (nt > 2) issue_k(2, 2);
  if (nt > 1) issue_v(1, 1);
  if (nt > 3) issue_k(3, 3);

  // ---- LDS read addresses (slot 0) ------------------------------------------------------------
  // K operand: lane (qi,h) reads key row qi, bytes 64kk + 32h .. +31 = chunks 4kk + 2h, +1
  uint32_t kaddr[NKK][2];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
    for (int e = 0; e < 2; ++e) kaddr[kk][e] = qi * ROWB + (((4 * kk + 2 * h + e) ^ attn_swz_k<ROWB>(qi)) << 4);
  // V operand through the 8-bit transposing load (layout notes in attn_fwd_fp8.hip).  The
  // swizzle only exchanges the 32-byte column groups of blocks 2c and 2c+1, so two address
  // registers per read slot serve all four column blocks: vaddr[cb & 1][pr] + 64 * (cb >> 1).
  uint32_t vaddr[2][4];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
    const int e = s >> 1;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const int key = 32 * (pr >> 1) + 16 * (pr & 1) + 8 * (e >> 2) + 4 * h + (e & 3);
        const int chunk = cb * 2 + chalf;
        vaddr[cb][pr] = VBASE + key * ROWB + ((chunk ^ swz_v8(key)) << 4) + ((s & 1) << 3);
      }
  }
  // K operand of S^T block kb, k-step kk; V^T operand of column block cb (slot offset `off`)
  auto k_operand = [&](auto off, int kb, int kk) __attribute__((always_inline)) {
    const u32x4 lo = *(LDS_AS u32x4*)(smem + kaddr[kk][0] + off + kb * 32 * ROWB);
    const u32x4 hi = *(LDS_AS u32x4*)(smem + kaddr[kk][1] + off + kb * 32 * ROWB);
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
  };
  auto v_operand = [&](auto off, int cb) __attribute__((always_inline)) {
    i32x8 a;
#pragma unroll
    for (int pr = 0; pr < 4; ++pr) {
      const i32x2 t = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(smem + vaddr[cb & 1][pr] + off + 64 * (cb >> 1)));
      a[2 * pr] = t[0];
      a[2 * pr + 1] = t[1];
    }
    return a;
  };

  // ---- streaming-softmax state ------------------------------------------------------------------
  f32x16 oacc[NCB];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) oacc[cb][r] = 0.f;
  }
  float m_ref = -INFINITY, l_run = 0.f;
  const float c = p.scale_log2;
  const int qrow = wq0 + qi;
  const int limit = CAUSAL ? min(qrow, N - 1) : (N - 1);
  const int unit_scale = 0x7f7f7f7f;  // E8M0 exponent 127 = 2^0 for both block scales
  auto mfma = [&](const i32x8& a, const i32x8& b, const f32x16& acc) __attribute__((always_inline)) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, 0, 0, 0, unit_scale, 0, unit_scale);
  };

  // two score buffers and two probability buffers; step j reads buffer j mod 2 and writes the other
  f32x16 s_a[2], s_b[2];
  i32x8 phi_a, plo_a, phi_b, plo_b;
#pragma unroll
  for (int i = 0; i < 8; ++i) phi_a[i] = plo_a[i] = phi_b[i] = plo_b[i] = 0;

  // P^T = 2^6 exp2(c S^T - m) of one tile as two e4m3 terms (four keys to a dword, accumulator
  // order); returns this lane's share of the row sum
  auto exp_tile = [&](const f32x16 (&s)[2], i32x8& phi, i32x8& plo) __attribute__((always_inline)) {
    const float msub = m_ref - kPShift;
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][4 * b + 0], c, -msub));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][4 * b + 1], c, -msub));
        const float e2 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][4 * b + 2], c, -msub));
        const float e3 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][4 * b + 3], c, -msub));
        int hi = 0;
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, hi, true);
        const auto b01 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false);
        const auto b23 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
        int lo = 0;
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(e0 - b01[0], e1 - b01[1], lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(e2 - b23[0], e3 - b23[1], lo, true);
        phi[kb * 4 + b] = hi;
        plo[kb * 4 + b] = lo;
        if (kb == 0 && b == 0) {
          ls0 = e0 + e2;
          ls1 = e1 + e3;
        } else {
          ls0 += e0 + e2;
          ls1 += e1 + e3;
        }
      }
    return ls0 + ls1;
  };
  // slow pass: true tile maximum, raise the reference, rescale, redo the tile
  auto redo_tile = [&](const f32x16 (&s)[2], i32x8& phi, i32x8& plo) __attribute__((always_inline)) {
    float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
    mx = attn_max_halves(mx) * c;
    const float m_new = fmaxf(m_ref, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // exp2(-inf) = 0 on the first tile
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
    return exp_tile(s, phi, plo);
  };

  // ---- building blocks of the boundary steps (compiler-scheduled) ---------------------------------
  auto qk_tile = [&](f32x16 (&s)[2], int off) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) s[kb] = mfma(k_operand(off, kb, kk), qf[kk], s[kb]);
    }
  };
  auto pv_tile = [&](const i32x8& phi, const i32x8& plo, int off) __attribute__((always_inline)) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const i32x8 a = v_operand(off, cb);
      oacc[cb] = mfma(a, phi, oacc[cb]);
      oacc[cb] = mfma(a, plo, oacc[cb]);
    }
  };
  auto softmax_tile = [&](f32x16 (&s)[2], i32x8& phi, i32x8& plo, int j) __attribute__((always_inline)) {
    if ((CAUSAL && j * BN + BN - 1 > wq0) || j * BN + BN - 1 >= N) {
      const int kbase = j * BN + 4 * h;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kbase + kb * 32 + 8 * (r >> 2) + (r & 3) > limit) s[kb][r] = -INFINITY;
    }
    float ls = exp_tile(s, phi, plo);
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) ls = redo_tile(s, phi, plo);
    l_run += ls;
  };
  // step j for any tile: O += V(j-1) P(j-1) first (still relative to the old reference), then the
  // softmax of tile j (which may rescale O), then S(j+1)
  auto step_any = [&](int j, f32x16 (&s_in)[2], f32x16 (&s_out)[2], i32x8& phi_out, i32x8& plo_out, const i32x8& phi_pv,
                      const i32x8& plo_pv) __attribute__((always_inline)) {
    if (j >= 1 && j - 1 <= jl) pv_tile(phi_pv, plo_pv, ((j - 1) & (NSLOT - 1)) * TILEB);
    if (j <= jl) softmax_tile(s_in, phi_out, plo_out, j);
    if (j + 1 <= jl) qk_tile(s_out, ((j + 1) & (NSLOT - 1)) * TILEB);
  };

  // ---- the pipelined step on a fully visible tile j (1 <= j < jl) -------------------------------
  // MFMA order: no two consecutive MFMAs share an accumulator.
  //   Q00 P0h P1h Q01 P0l P1l Q10 P2h P3h Q11 P2l P3l     (Qbk: S^T block b, k-step k; Pch/Pcl: O^T block c)
  auto step_hot = [&](f32x16 (&s_in)[2], f32x16 (&s_out)[2], i32x8& phi_out, i32x8& plo_out, const i32x8& phi_pv, const i32x8& plo_pv,
                      auto koff, auto voff) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_out[kb][r] = 0.f;
    const i32x8 v0 = v_operand(voff, 0), v1 = v_operand(voff, 1);
    s_out[0] = mfma(k_operand(koff, 0, 0), qf[0], s_out[0]);
    oacc[0] = mfma(v0, phi_pv, oacc[0]);
    oacc[1] = mfma(v1, phi_pv, oacc[1]);
    s_out[0] = mfma(k_operand(koff, 0, 1), qf[1], s_out[0]);
    oacc[0] = mfma(v0, plo_pv, oacc[0]);
    oacc[1] = mfma(v1, plo_pv, oacc[1]);
    const i32x8 v2 = v_operand(voff, 2), v3 = v_operand(voff, 3);
    s_out[1] = mfma(k_operand(koff, 1, 0), qf[0], s_out[1]);
    oacc[2] = mfma(v2, phi_pv, oacc[2]);
    oacc[3] = mfma(v3, phi_pv, oacc[3]);
    s_out[1] = mfma(k_operand(koff, 1, 1), qf[1], s_out[1]);
    oacc[2] = mfma(v2, plo_pv, oacc[2]);
    oacc[3] = mfma(v3, plo_pv, oacc[3]);
    float ls = exp_tile(s_in, phi_out, plo_out);
    // the conversions belong to this step: keep the compiler from sinking them past the branch below
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(phi_out[i]), "+v"(plo_out[i]));
    // vector instructions of a tile: 32 x (multiply-add, add, subtract) + 48 conversions + a few
    fp8_step_pipeline<0, 12, 150>();
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) ls = redo_tile(s_in, phi_out, plo_out);
    l_run += ls;
  };

  // ---- prologue: S(0) ------------------------------------------------------------------------------
  // everything but the newest prologue load (K3, if it was issued) has landed
  if (nt > 3) ATTN_WAIT_VMCNT(1);
  else ATTN_WAIT_VMCNT(0);
  // Q is in registers from here on (touched one dword at a time: a 256-bit asm operand has no
  // host-side equivalent and silently drops the kernel's launch stub)
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(qf[kk][i]));
  attn_wg_barrier();
  if (jl >= 0) qk_tile(s_a, 0);
  attn_wg_barrier();  // every wave has read K(0): step 0 may hand its slot to K(4)

  // ---- main loop: step j = 0 .. nt (step nt only finishes the last PV product) ----------------------
  // loads of step j: K(j+4) into the slot K(j) has left, V(j+2) into the slot V(j-2) has left
  auto step_loads = [&](int j, int kslot, int vslot) __attribute__((always_inline)) {
    if (j + 4 < nt) issue_k(j + 4, kslot);
    if (j + 2 < nt) issue_v(j + 2, vslot);
  };
  // end of step j: the loads of step j-1 (and older) have landed, those of step j may be in flight
  auto step_end = [&](int j) __attribute__((always_inline)) {
    const int n = (j + 4 < nt ? 1 : 0) + (j + 2 < nt ? 1 : 0);
    if (n == 2) ATTN_WAIT_VMCNT(2);
    else if (n == 1) ATTN_WAIT_VMCNT(1);
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
  };
  auto any_step = [&](int j) __attribute__((always_inline)) {
    step_loads(j, j & (NSLOT - 1), (j + 2) & (NSLOT - 1));
    if (j & 1) step_any(j, s_b, s_a, phi_b, plo_b, phi_a, plo_a);
    else step_any(j, s_a, s_b, phi_a, plo_a, phi_b, plo_b);
    if (j < nt) step_end(j);
  };
  // hot steps are j in [1, hot_end): tile j fully visible to the wave, tiles j-1 and j+1 exist for it
  int hot_end = CAUSAL ? min(jl, (wq0 + 1) / BN) : jl;
  hot_end = hot_end <= 1 ? 1 : 1 + ((hot_end - 1) & ~3);  // whole groups of four, starting at j = 1

  any_step(0);
  int j = 1;
  if (hot_end > 1) {
    for (; j < hot_end; j += 4) {
      // step j (= 1 mod 4): K(j+1) in slot 2, V(j-1) in slot 0; next step reads K(j+2) in slot 3, V(j) in slot 1
      step_loads(j, 1, 3);
      step_hot(s_b, s_a, phi_b, plo_b, phi_a, plo_a, ic<2 * TILEB>{}, ic<0 * TILEB>{});
      step_end(j);
      step_loads(j + 1, 2, 0);
      step_hot(s_a, s_b, phi_a, plo_a, phi_b, plo_b, ic<3 * TILEB>{}, ic<1 * TILEB>{});
      step_end(j + 1);
      step_loads(j + 2, 3, 1);
      step_hot(s_b, s_a, phi_b, plo_b, phi_a, plo_a, ic<0 * TILEB>{}, ic<2 * TILEB>{});
      step_end(j + 2);
      step_loads(j + 3, 0, 2);
      step_hot(s_a, s_b, phi_a, plo_a, phi_b, plo_b, ic<1 * TILEB>{}, ic<3 * TILEB>{});
      step_end(j + 3);
    }
  }
  for (; j <= nt; ++j) any_step(j);

  // ---- epilogue -----------------------------------------------------------------------------------
  char* const ohead = (char*)p.o + ((size_t)(tc.b * p.Hq + tc.hq) * N) * (D * 2);
  float* const lsehead = p.lse + (size_t)(tc.b * p.Hq + tc.hq) * N;
  {
    const float l = attn_sum_halves(l_run);  // 2^6 * sum of the unrounded exponentials
    const float inv = p.out_scale / l;
    if (qrow < N && h == 0) lsehead[qrow] = (m_ref - kPShift + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        uint32_t x[2], y[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          bf16x2 tx, ty;
          tx[0] = (__bf16)(oacc[cb][(2 * a) * 4 + 2 * r] * inv);
          tx[1] = (__bf16)(oacc[cb][(2 * a) * 4 + 2 * r + 1] * inv);
          ty[0] = (__bf16)(oacc[cb][(2 * a + 1) * 4 + 2 * r] * inv);
          ty[1] = (__bf16)(oacc[cb][(2 * a + 1) * 4 + 2 * r + 1] * inv);
          auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, tx), __builtin_bit_cast(uint32_t, ty), false, false);
          x[r] = sw[0];
          y[r] = sw[1];
        }
        if (qrow < N) {
          u32x4 out = {x[0], x[1], y[0], y[1]};
          *(u32x4*)(ohead + (size_t)qrow * (D * 2) + (cb * 32 + a * 16 + h * 8) * 2) = out;
        }
      }
  }
}

template <int D>
int launch_fp8_sp(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_fp8_sp_kernel<D, true>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_fp8_sp_kernel<D, false>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_fp8_sp_variants(int* count) {
  static const AttnVariant table[] = {
      {"fp8 d128 pipelined BM256 BN64", 1, 128, 256, 64, 512, 2 * 4 * 64 * 128, launch_fp8_sp<128>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
