// Fused attention forward for fp8 (e4m3) inputs, gfx950: the software-pipelined bf16 kernel fed
// by a convert-on-arrival stage.
//
// Every e4m3 value is exactly representable in bfloat16, so the products can be taken on the
// bf16 matrix path without touching the inputs' values: P then needs one bf16 rounding instead
// of the two-term e4m3 split the all-fp8 kernel pays for (its vector work, not its MFMA time,
// is what limits that kernel).  Mathematics, register layout, the step pipeline, the
// no-maximum softmax and the three-slot bundle ring are those of attn_fwd_bf16_sp.hip (paper
// section 6.1 for the phases, appendix C.3 for the streaming-softmax state).  What differs is
// the producer side:
//   * K and V tiles arrive as fp8 bytes by direct-to-LDS loads in a two-slot staging area
//     (16 KB per bundle), one bundle earlier than the bf16 kernel requests its tiles;
//   * between the two steps of an iteration, after the barrier that frees a ring slot, every
//     thread converts the 16 + 16 bytes it staged itself (no extra synchronisation: a thread
//     only ever reads staging bytes its own wave loaded) with the packed fp8 -> bf16 conversion
//     and writes them, swizzled, into the freed slot of the bf16 ring;
//   * Q is converted once, in registers.
// The de-scales are folded into the softmax scale and the output scale by the caller.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2v;

// 16 e4m3 bytes -> 16 bf16 (two 16-byte chunks), exact
__device__ __forceinline__ void cvt16(const u32x4 in, u32x4& lo, u32x4& hi) {
  uint32_t o[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(in[i], 1.0f, false));
    o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(in[i], 1.0f, true));
  }
  lo = u32x4{o[0], o[1], o[2], o[3]};
  hi = u32x4{o[4], o[5], o[6], o[7]};
}


constexpr float kTau = 8.0f;
constexpr float kSumLimit = 65536.0f;  // a lane's 16-term partial sum above this redoes the block with a raised reference

template <int V>
using ic = std::integral_constant<int, V>;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

// Scheduling-group pipeline of one pipelined step (the builtin wants literal constants, hence the
// recursion): per MFMA its share of the plain vector work, of the 16 exponentials, and the LDS
// reads of the operand RA MFMAs ahead (one 128-bit K read or two transposing V reads).
template <int M, int NM, int RA, int NVALU>
__device__ __forceinline__ void step_pipeline() {
  if constexpr (M < NM) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                         // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (M + 1)) / NM - (NVALU * M) / NM, 0);  // VALU
    __builtin_amdgcn_sched_group_barrier(0x400, 16 / NM, 0);                                   // transcendental
    __builtin_amdgcn_sched_group_barrier(0x100, ((M + RA) & 1) ? 2 : 1, 0);                    // LDS read
    step_pipeline<M + 1, NM, RA, NVALU>();
  }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 2) attn_fwd_fp8_cv_kernel(const AttnParams p) {
  static_assert(D == 128, "the staging layout assumes 128-byte fp8 rows");
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int NKK = D / 16;       // MFMA k-steps of S^T = K Q^T
  constexpr int NCB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;       // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row
  constexpr int TILEB = BN * ROWB;  // bytes per K (or V) tile
  constexpr int SUBB = 32 * ROWB;   // bytes per 32-key block
#ifndef ATTN_SP_NSLOT
#define ATTN_SP_NSLOT 3
#endif
  constexpr int NSLOT = ATTN_SP_NSLOT;  // ring depth: bundles are requested NSLOT-1 ahead
  constexpr int VBASE = NSLOT * TILEB;  // K parts of the slots first, then the V parts
  constexpr int NLD = BN * NCH / NT;    // direct-to-LDS loads per thread per tile
#ifndef ATTN_RA
#define ATTN_RA 4
#endif
  constexpr int RA = ATTN_RA;           // operands are read from LDS this many MFMAs ahead
  static_assert(BN * NCH % NT == 0 && NLD >= 1, "tile must divide evenly over the workgroup");
  static_assert(NKK == 2 * NCB && RA >= 2 && RA <= 2 * NKK, "one PV step per QK^T step; read-ahead within a step");
  static_assert((NSLOT - 1) * TILEB + SUBB + 16 * ROWB < 65536 && (NSLOT == 3 || NSLOT == 4), "ring offsets must fit the 16-bit LDS immediate");

  constexpr int INROWB = D;              // bytes per fp8 row
  constexpr int STGTILE = BN * INROWB;   // one staged fp8 tile
  constexpr int STGBASE = 2 * NSLOT * TILEB;  // two staging slots of (K tile, V tile) behind the bf16 ring
  static_assert(STGTILE == NT * 16, "every thread stages one 16-byte chunk per tile");
  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB + 2 * 2 * STGTILE];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31;  // query column within the wave's 32-query block
  const int h = lane >> 5;   // which half of the k-slots / accumulator rows this lane holds

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  const int hk = tc.hq / G;
  const int q0 = tc.t * BM;
  const int wq0 = q0 + w * 32;  // first query row of this wave
  const bool wave_valid = wq0 < N;

  const char* const qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * INROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * INROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * INROWB;

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;  // keys the workgroup visits
  const int nt = (kv_end + BN - 1) / BN;            // 64-key tiles = bundles

  // ---- producer role: fp8 tiles by direct-to-LDS loads into staging, converted into the ring ------
  // thread tid stages chunk tid of a tile: row tid / 8, bytes 16 (tid % 8) .. +15 of that row
  const int st_row = tid >> 3, st_c = tid & 7;
  const uint32_t st_goff = st_row * INROWB + st_c * 16;
  const uint32_t lds_base = (uint32_t)(uintptr_t)smem;
  const uint32_t lds_wave_stg = lds_base + STGBASE + w * 1024;
  auto stage_tile = [&](const char* head, int t, uint32_t dst) __attribute__((always_inline)) {
    const char* const base = head + (size_t)t * STGTILE;
    // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
    const uint32_t over = (uint32_t)max(0, t * BN + st_row - (N - 1)) * INROWB;
    attn_lds_dma16(base, st_goff - over, dst);
  };
  // bundle b = key tile b+1 (the last tile again if there is none) and value tile b
  auto stage_bundle = [&](int b, int stg) __attribute__((always_inline)) {
    stage_tile(khead, min(b + 1, nt - 1), lds_wave_stg + stg * 2 * STGTILE);
    stage_tile(vhead, b, lds_wave_stg + stg * 2 * STGTILE + STGTILE);
  };
  // where this thread's 16 staged values go in a bf16 tile: row st_row, chunks 2 st_c and 2 st_c + 1
  const uint32_t cv_k0 = st_row * ROWB + (((2 * st_c) ^ attn_swz_k<ROWB>(st_row)) << 4);
  const uint32_t cv_k1 = st_row * ROWB + (((2 * st_c + 1) ^ attn_swz_k<ROWB>(st_row)) << 4);
  const uint32_t cv_v0 = st_row * ROWB + (((2 * st_c) ^ attn_swz_v<ROWB>(st_row)) << 4);
  const uint32_t cv_v1 = st_row * ROWB + (((2 * st_c + 1) ^ attn_swz_v<ROWB>(st_row)) << 4);
  const uint32_t st_self = STGBASE + tid * 16;  // this thread's chunk inside a staged tile
  auto convert_k = [&](int stg_off, int ring_off) __attribute__((always_inline)) {
    u32x4 lo, hi;
    cvt16(*(const LDS_AS u32x4*)(smem + st_self + stg_off), lo, hi);
    *(LDS_AS u32x4*)(smem + cv_k0 + ring_off) = lo;
    *(LDS_AS u32x4*)(smem + cv_k1 + ring_off) = hi;
  };
  auto convert_v = [&](int stg_off, int ring_off) __attribute__((always_inline)) {
    u32x4 lo, hi;
    cvt16(*(const LDS_AS u32x4*)(smem + st_self + stg_off), lo, hi);
    *(LDS_AS u32x4*)(smem + cv_v0 + ring_off) = lo;
    *(LDS_AS u32x4*)(smem + cv_v1 + ring_off) = hi;
  };
  auto convert_bundle = [&](int stg, int slot) __attribute__((always_inline)) {
    convert_k(stg * 2 * STGTILE, slot * TILEB);
    convert_v(stg * 2 * STGTILE + STGTILE, VBASE + slot * TILEB);
  };
  // staged bytes have been read into registers: the staging slot may be refilled
  auto staging_read_done = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };

  stage_tile(khead, 0, lds_wave_stg + 2 * STGTILE);  // key tile 0 borrows the K part of staging slot 1
  stage_bundle(0, 0);

  // ---- Q operand (B operand of S^T = K Q^T): lane (qi,h) holds Q[row][16kk+8h .. +7] ----------
  bf16x8 qf[NKK];
  {
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * INROWB + h * 8;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const u32x2 raw = *(const u32x2*)(src + kk * 16);
      u32x4 o;
      o[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[0], 1.0f, false));
      o[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[0], 1.0f, true));
      o[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[1], 1.0f, false));
      o[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[1], 1.0f, true));
      qf[kk] = __builtin_bit_cast(bf16x8, o);
    }
  }

  // ---- LDS read addresses (slot 0, first 32-key block) -----------------------------------------
  uint32_t kaddr[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = qi * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(qi)) << 4);
  // V through the transposing load: in a group of 16 lanes, lane s reads the four columns
  // 4*(s%4).. of key row s/4 and the hardware hands lane t the four keys of column t.
  uint32_t vaddr[NCB][2];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int key = 8 * e + 4 * h + (s >> 2);
        const int chunk = cb * 4 + chalf * 2 + ((s & 3) >> 1);
        vaddr[cb][e] = VBASE + key * ROWB + ((chunk ^ attn_swz_v<ROWB>(key)) << 4) + ((s & 1) << 3);
      }
  }
  auto k_operand = [&](auto koff, int kk) __attribute__((always_inline)) {
    return __builtin_bit_cast(u32x4, *(LDS_AS bf16x8*)(smem + kaddr[kk] + koff));
  };
  auto v_operand = [&](auto voff, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + voff + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + voff + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return __builtin_bit_cast(u32x4, av);
  };

  // ---- streaming-softmax state ----------------------------------------------------------------
  f32x16 oacc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_ref = -INFINITY;  // reference maximum, scaled log2 units
  float l_run = 0.f;        // this lane's share of the row sum (halves are added at the end)
  const float c = p.scale_log2;
  const int qrow = wq0 + qi;
  const int limit = CAUSAL ? min(qrow, N - 1) : (N - 1);  // last visible key of this lane's query
  const int wlast = wq0 + 31;

  f32x16 s_a, s_b;        // S^T of two consecutive blocks (one consumed, one produced)
  u32x4 p_a[2], p_b[2];   // packed P^T of two consecutive blocks (one produced, one consumed)
#pragma unroll
  for (int i = 0; i < 2; ++i) p_a[i] = p_b[i] = u32x4{0, 0, 0, 0};

  // rescale everything that is relative to the reference maximum: l, O and the packed P^T of
  // the block whose PV product has not been issued yet
  auto raise_reference = [&](float mx, u32x4 (&pend)[2]) __attribute__((always_inline)) {
    const float m_new = fmaxf(m_ref, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // exp2(-inf) = 0 on the first block
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t u = pend[i][r];
        pend[i][r] = pack_bf16(__uint_as_float(u << 16) * alpha, __uint_as_float(u & 0xffff0000u) * alpha);
      }
  };
  auto block_max = [&](const f32x16& s) __attribute__((always_inline)) {
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
    return attn_max_halves(mx) * c;
  };

  // ---- boundary-case building blocks (compiler-scheduled, not overlapped) ----------------------
  auto qk_block = [&](f32x16& s, auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, k_operand(koff, kk)), qf[kk], s, 0, 0, 0);
  };
  auto pv_block = [&](const u32x4 (&pk)[2], auto voff) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2 * NCB; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v_operand(voff, cb, kc)),
                                                         __builtin_bit_cast(bf16x8, pk[kc]), oacc[cb], 0, 0, 0);
    }
  };
  auto softmax_block = [&](f32x16& s, u32x4 (&pk)[2], u32x4 (&pend)[2], int key0, bool need_mask) __attribute__((always_inline)) {
    if (need_mask) {
      const int kbase = key0 + 4 * h;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kbase + 8 * (r >> 2) + (r & 3) > limit) s[r] = -INFINITY;
    }
    const float mx = block_max(s);
    if (__builtin_amdgcn_ballot_w64(mx > m_ref + kTau) != 0) raise_reference(mx, pend);
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * r], c, -m_ref));
      const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * r + 1], c, -m_ref));
      pk[r >> 2][r & 3] = pack_bf16(e0, e1);
      ls0 += e0;
      ls1 += e1;
    }
    l_run += ls0 + ls1;
  };
  auto is_active = [&](int key0) __attribute__((always_inline)) {
    return wave_valid && key0 < kv_end && (!CAUSAL || key0 <= wlast);
  };
  auto needs_mask = [&](int key0) __attribute__((always_inline)) {
    return (CAUSAL && key0 + 31 > wq0) || key0 + 31 >= N;
  };

  // ---- the pipelined step on fully visible blocks ------------------------------------------------
  //   s_in  : scores of the block exponentiated now                     -> p_out
  //   s_out : scores of the next block        (K operands at off)
  //   p_pv  : probabilities of the previous block, multiplied into O    (V operands at off)
  // The 2*NKK MFMAs alternate between the two products (the QK^T chain is dependent, the PV
  // accumulators are not), operands are read from LDS RA MFMAs ahead; the first RA operands of a
  // step are requested by the previous step (offnext = where the next step reads).
  // The vector work needs no block maximum: exponentials are taken against the current
  // reference and the block is redone, after raising the reference and rescaling, only if a
  // lane's partial sum comes out large or not a number (always on the very first block).
  // Source order inside the step does not matter: the scheduling-group pipeline at its end
  // tells the scheduler how to interleave the four instruction classes.
  constexpr int NM = 2 * NKK;
  u32x4 pre[RA];
  auto step_operand = [&](auto off, int m) __attribute__((always_inline)) {
    const int i = m >> 1;
    return (m & 1) ? v_operand(off, i % NCB, i / NCB) : k_operand(off, i);
  };
  auto exp_block = [&](const f32x16& s_in, u32x4 (&p_out)[2]) __attribute__((always_inline)) {
    f32x16 e;
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[r], c, -m_ref));
#pragma unroll
    for (int u = 0; u < 8; ++u) p_out[u >> 2][u & 3] = pack_bf16(e[2 * u], e[2 * u + 1]);
    float ls0 = e[0], ls1 = e[1];
#pragma unroll
    for (int u = 1; u < 8; ++u) {
      ls0 += e[2 * u];
      ls1 += e[2 * u + 1];
    }
    return ls0 + ls1;
  };
  auto step_hot = [&](f32x16& s_in, f32x16& s_out, u32x4 (&p_out)[2], u32x4 (&p_pv)[2], auto off, auto offnext) __attribute__((always_inline)) {
    u32x4 op[NM];
#pragma unroll
    for (int m = 0; m < RA; ++m) op[m] = pre[m];
#pragma unroll
    for (int r = 0; r < 16; ++r) s_out[r] = 0.f;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const int i = m >> 1;
      if (m & 1)
        oacc[i % NCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), __builtin_bit_cast(bf16x8, p_pv[i / NCB]),
                                                                oacc[i % NCB], 0, 0, 0);
      else
        s_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), qf[i], s_out, 0, 0, 0);
      if (m + RA < NM) op[m + RA] = step_operand(off, m + RA);
      else pre[m + RA - NM] = step_operand(offnext, m + RA - NM);
    }
    float ls = exp_block(s_in, p_out);
    // pipeline: per MFMA one exponential, the plain vector work spread evenly, and the LDS
    // reads of the operand RA MFMAs ahead (one 128-bit K read or two transposing V reads)
    constexpr int NVALU = 16 + 14 + 8 + 2;  // multiply-adds, adds, packs, final add + compare
    step_pipeline<0, NM, RA, NVALU>();
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) {
      float mx = fmaxf(s_in[0], s_in[1]);
#pragma unroll
      for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s_in[r]);
      mx = attn_max_halves(mx) * c;
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // exp2(-inf) = 0 on the first block
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
      ls = exp_block(s_in, p_out);
    }
    l_run += ls;
  };

  // the same step for blocks that may be masked or not visible to this wave (run-time offsets)
  auto step_any = [&](bool do_sm, int key0, bool do_mm, f32x16& s_in, f32x16& s_out, u32x4 (&p_out)[2], u32x4 (&p_pv)[2], int koff,
                      int voff) __attribute__((always_inline)) {
    if (do_sm) softmax_block(s_in, p_out, p_pv, key0, needs_mask(key0));
    if (do_mm) {
      qk_block(s_out, koff);
      pv_block(p_pv, voff);
    }
  };

  // ---- prologue: block 0 ---------------------------------------------------------------------------
  // everything requested so far has landed: convert key tile 0 and bundle 0, then stage bundles 1 and 2
  ATTN_WAIT_VMCNT(0);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) asm volatile("" ::"v"(qf[kk]));  // Q is in registers from here on
  convert_k(2 * STGTILE, (NSLOT - 1) * TILEB);
  convert_bundle(0, 0);
  staging_read_done();
  if (nt > 1) stage_bundle(1, 1);
  if (nt > 2) stage_bundle(2, 0);
  attn_wg_barrier();
  if (wave_valid) {
    qk_block(s_b, (NSLOT - 1) * TILEB);                          // S(0)
    softmax_block(s_b, p_b, p_a, 0, needs_mask(0));    // P(0) -> p_b (nothing pending yet)
    qk_block(s_a, (NSLOT - 1) * TILEB + SUBB);                   // S(1); ignored if block 1 is not visible
  }
  // bundle 1 has been staged once only bundle 2's two loads are outstanding: convert it into slot 1
  if (nt > 1) {
    if (nt > 2) ATTN_WAIT_VMCNT(2);
    else ATTN_WAIT_VMCNT(0);
    convert_bundle(1, 1);
  }
  attn_wg_barrier();  // the K part of the last slot is empty again
#pragma unroll
  for (int m = 0; m < RA; ++m) pre[m] = step_operand(ic<0>{}, m);  // first operands of the first pipelined step

  // ---- main loop over bundles ------------------------------------------------------------------------
  // iteration b: exponentiate blocks 2b+1 and 2b+2, compute the scores of blocks 2b+2 and 2b+3
  // (key tile b+1), accumulate blocks 2b and 2b+1 (value tile b)
  // between the two steps of iteration b: bundle b+1 (requested one iteration ago, the only
  // loads in flight) is published, and the slot of bundle b-1, which every wave has finished
  // reading, is handed to bundle b+2
  // (fp8 input) the barrier publishes the bf16 copy of bundle b+1, written one iteration ago, and
  // frees the slot of bundle b-1; bundle b+2, staged one iteration ago, is converted into that
  // slot and bundle b+3 is requested into the staging slot bundle b+1 was converted from
  auto bundle_mid = [&](int b, int free_slot) __attribute__((always_inline)) {
    ATTN_WAIT_VMCNT(0);  // this thread's part of staged bundle b+2
    attn_wg_barrier();
    if (b + 2 < nt) convert_bundle(b & 1, free_slot);
    // (the other staging slot was read one iteration ago)
    if (b + 3 < nt) stage_bundle(b + 3, (b + 1) & 1);
  };
  auto bundle_hot = [&](int b, auto slot_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    step_hot(s_a, s_b, p_a, p_b, ic<SLOT * TILEB>{}, ic<SLOT * TILEB + SUBB>{});
    bundle_mid(b, (SLOT + NSLOT - 1) % NSLOT);
    step_hot(s_b, s_a, p_b, p_a, ic<SLOT * TILEB + SUBB>{}, ic<((SLOT + 1) % NSLOT) * TILEB>{});
  };
  auto bundle_any = [&](int b, int slot) __attribute__((always_inline)) {
    const int k1 = (2 * b + 1) * 32, k2 = k1 + 32;
    step_any(is_active(k1), k1, is_active(k1 - 32), s_a, s_b, p_a, p_b, slot * TILEB, slot * TILEB);
    bundle_mid(b, slot >= 1 ? slot - 1 : NSLOT - 1);
    step_any(is_active(k2), k2, is_active(k1), s_b, s_a, p_b, p_a, slot * TILEB + SUBB, slot * TILEB + SUBB);
  };

  // bundles 0 .. n_hot-1 touch only blocks (up to 2b+2) that every query of this wave sees in full
  const int vis = CAUSAL ? min(wq0, N - 1) : N - 1;  // last key every query of the wave can see
  const int n_hot = (wave_valid && vis >= 95) ? (vis - 95) / 64 + 1 : 0;
  const int n_ring = n_hot - n_hot % NSLOT;  // whole turns of the ring, slot offsets as immediates
  int b = 0;
  for (; b < n_ring; b += NSLOT) {
    bundle_hot(b, ic<0>{});
    bundle_hot(b + 1, ic<1>{});
    bundle_hot(b + 2, ic<2>{});
    if (NSLOT > 3) bundle_hot(b + 3, ic<3 % NSLOT>{});
  }
  // the last fully visible bundles (fewer than a turn), then the masked / partly visible ones
  int slot = 0;
  if (b < n_hot) { bundle_hot(b, ic<0>{}); ++b; slot = 1; }
  if (b < n_hot) { bundle_hot(b, ic<1>{}); ++b; slot = 2; }
  if (NSLOT > 3 && b < n_hot) { bundle_hot(b, ic<2>{}); ++b; slot = 3 % NSLOT; }
  for (; b < nt; ++b) {
    bundle_any(b, slot);
    slot = slot == NSLOT - 1 ? 0 : slot + 1;
  }

  // ---- epilogue: O = acc / l (bf16), lse = (m + log2 l) * ln 2 ------------------------------------------
  char* const ohead = (char*)p.o + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  float* const lsehead = p.lse + (size_t)(tc.b * p.Hq + tc.hq) * N;
  {
    const float l = attn_sum_halves(l_run);
    const float inv = p.out_scale / l;
    if (qrow < N && h == 0) lsehead[qrow] = (m_ref + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    // lane (qi,h) holds O^T rows 32cb + 8b + 4h + r.  Exchange with the other half so that every
    // lane owns 8 consecutive output columns 32cb + 16a + 8h + (0..7): one 16-byte store each.
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        uint32_t x[2], y[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const uint32_t tx = pack_bf16(oacc[cb][(2 * a) * 4 + 2 * r] * inv, oacc[cb][(2 * a) * 4 + 2 * r + 1] * inv);
          const uint32_t ty = pack_bf16(oacc[cb][(2 * a + 1) * 4 + 2 * r] * inv, oacc[cb][(2 * a + 1) * 4 + 2 * r + 1] * inv);
          auto sw = __builtin_amdgcn_permlane32_swap(tx, ty, false, false);
          x[r] = sw[0];
          y[r] = sw[1];
        }
        if (qrow < N) {
          u32x4 out = {x[0], x[1], y[0], y[1]};
          *(u32x4*)(ohead + (size_t)qrow * ROWB + (cb * 32 + a * 16 + h * 8) * 2) = out;
        }
      }
  }
}

template <int D>
int launch_cv(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_fp8_cv_kernel<D, true>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_fp8_cv_kernel<D, false>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_fp8_cv_variants(int* count) {
  static const AttnVariant table[] = {
      {"fp8 d128 bf16-converted pipelined BM256 BN64", 1, 128, 256, 64, 512, 2 * 3 * 64 * 128 * 2 + 4 * 64 * 128, launch_cv<128>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
