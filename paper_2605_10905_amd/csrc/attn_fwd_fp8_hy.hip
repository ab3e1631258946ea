// Fused attention forward for fp8 (e4m3) inputs, gfx950: scores on the fp8 matrix path,
// probabilities times values on the bf16 path.
//
// S^T = K Q^T is taken directly on the e4m3 bytes with the 32x32x64 f8f6f4 MFMA (two MFMAs per
// 32-key block instead of eight bf16 ones, K tiles of half the size straight from memory into
// the LDS ring, half the K reads).  P, however, loses too much when it is rounded to e4m3 (a
// second residual term would be needed), so P stays bf16 and V is converted e4m3 -> bf16, exactly,
// once per tile on arrival (attn_fwd_fp8_cv.hip describes that stage; here only V takes it).
// Everything else -- transposed products with one query per lane, the step pipeline, the
// no-maximum softmax, the three-slot bundle ring with one barrier per 64 keys -- is the bf16
// pipelined kernel's (attn_fwd_bf16_sp.hip; paper section 6.1, appendix C.3).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2v;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) int i32x2;

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
// recursion): per MFMA its share of the plain vector work and of the 16 exponentials, and the two
// LDS reads of the operand RA MFMAs ahead.
// VREADS: LDS reads per V fragment (two transposing reads, or one 128-bit read of a transposed tile);
// a K fragment always takes two.  MFMAs 0 and 5 of a step are the score products.
template <int M, int NM, int NVALU, int RA, int VREADS>
__device__ __forceinline__ void hy_step_pipeline() {
  if constexpr (M < NM) {
    constexpr int T = (M + RA) % NM;  // the MFMA whose operand is requested behind MFMA M
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                         // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (M + 1)) / NM - (NVALU * M) / NM, 0);  // VALU
    __builtin_amdgcn_sched_group_barrier(0x400, (16 * (M + 1)) / NM - (16 * M) / NM, 0);       // transcendental
    __builtin_amdgcn_sched_group_barrier(0x100, (T == 0 || T == 5) ? 2 : VREADS, 0);           // LDS read
    hy_step_pipeline<M + 1, NM, NVALU, RA, VREADS>();
  }
}

// VT: the conversion pass also transposes.  The bf16 value tile then lies in LDS as V^T (one row per
// head-dimension column, 64 keys in the order of the P V product's k-slots) and a V fragment is one
// 128-bit read instead of two transposing 64-bit reads: an LDS read costs the LDS the same eight
// cycles whatever its width, and the LDS instruction rate is what caps this kernel's matrix pipe.
template <int D, bool CAUSAL, bool VT>
__global__ void __launch_bounds__(512, 2) attn_fwd_fp8_hy_kernel(const AttnParams p) {
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
  constexpr int KROWB = D;              // bytes per fp8 K row
  constexpr int KTILEB = BN * KROWB;    // bytes per fp8 K tile
  constexpr int KSUBB = 32 * KROWB;     // bytes per 32-key block of it
  constexpr int NK8 = D / 64;           // f8f6f4 MFMA k-steps of S^T = K Q^T
  constexpr int VBASE = NSLOT * KTILEB; // fp8 K parts of the slots first, then the bf16 V parts
  constexpr int NLD = BN * NCH / NT;    // direct-to-LDS loads per thread per tile
#ifndef ATTN_HY_RA
#define ATTN_HY_RA 4
#endif
  constexpr int RA = ATTN_HY_RA;        // operands are read from LDS this many MFMAs ahead
  static_assert(BN * NCH % NT == 0 && NLD >= 1, "tile must divide evenly over the workgroup");
  static_assert(NSLOT == 3 && NK8 == 2 && NCB == 4, "ring of three; the step below is written for d = 128");

  constexpr int INROWB = D;              // bytes per fp8 row
  constexpr int STGTILE = BN * INROWB;   // one staged fp8 tile
  constexpr int STGBASE = VBASE + NSLOT * TILEB;  // two staging slots of one fp8 V tile each, behind the rings
  static_assert(STGTILE == NT * 16 && KTILEB == NT * 16, "every thread moves one 16-byte chunk per tile");
  __shared__ __attribute__((aligned(1024))) char smem_raw[STGBASE + 2 * STGTILE];
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

  // ---- producer role ------------------------------------------------------------------------------
  // thread tid moves chunk tid of a tile: row tid / 8, 16 bytes.  K goes straight into the ring
  // (LDS chunk c of a row holds the row's chunk c ^ swizzle); V goes to staging, unswizzled.
  const int st_row = tid >> 3, st_c = tid & 7;
  const uint32_t k_goff = st_row * INROWB + ((st_c ^ attn_swz_k<KROWB>(st_row)) << 4);
  // VT: staged rows are read eight at a time (keys b + {0..3, 8..11}) by the 8-bit transposing read;
  // LDS chunk c of staged row r holds the row's chunk c ^ fkey(r), so those eight land in different banks
  auto fkey = [](int r) __attribute__((always_inline)) { return (r & 3) | (((r >> 3) & 1) << 2); };
  const uint32_t st_goff = st_row * INROWB + (VT ? ((st_c ^ fkey(st_row)) << 4) : st_c * 16);
  const uint32_t lds_base = (uint32_t)(uintptr_t)smem;
  const uint32_t lds_wave = lds_base + w * 1024;
  const uint32_t lds_wave_stg = lds_base + STGBASE + w * 1024;
  auto row_over = [&](int t) __attribute__((always_inline)) {
    // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
    return (uint32_t)max(0, t * BN + st_row - (N - 1)) * INROWB;
  };
  auto issue_k = [&](int t, int kslot) __attribute__((always_inline)) {
    attn_lds_dma16(khead + (size_t)t * KTILEB, k_goff - row_over(t), lds_wave + kslot * KTILEB);
  };
  auto stage_v = [&](int t, int stg) __attribute__((always_inline)) {
    attn_lds_dma16(vhead + (size_t)t * STGTILE, st_goff - row_over(t), lds_wave_stg + stg * STGTILE);
  };
  // where this thread's 16 staged values go in a bf16 V tile: row st_row, chunks 2 st_c and 2 st_c + 1
  const uint32_t cv_v0 = VBASE + st_row * ROWB + (((2 * st_c) ^ attn_swz_v<ROWB>(st_row)) << 4);
  const uint32_t cv_v1 = VBASE + st_row * ROWB + (((2 * st_c + 1) ^ attn_swz_v<ROWB>(st_row)) << 4);
  const uint32_t st_self = STGBASE + tid * 16;  // this thread's chunk inside a staged tile
  // VT: a 16-lane group transposes a block of 8 keys x 16 columns per round (two rounds cover the
  // 64 blocks of a tile): lane s reads 8 bytes of staged key row e = s / 2, the hardware hands lane t
  // the 8 keys of column t, which become one 16-byte chunk of row t of V^T.  Output chunk ch of a
  // V^T row holds the keys of k-slot group ch = 4 (32-key half) + 2 kc + h in the order the S^T
  // accumulator (and so the packed P^T operand) has them: 32 (ch / 4) + 16 kc + 4 h + {0..3, 8..11}.
  uint32_t tr_src[2], tr_dst[2];
#pragma unroll
  for (int rnd = 0; rnd < 2; ++rnd) {
    const int blk = rnd * 32 + w * 4 + (lane >> 4), ch = blk & 7, cg = blk >> 3;
    const int s16 = lane & 15, e = s16 >> 1;
    const int key = 32 * (ch >> 2) + 16 * ((ch >> 1) & 1) + 8 * (e >> 2) + 4 * (ch & 1) + (e & 3);
    const int dcol = 16 * cg + s16;
    tr_src[rnd] = STGBASE + key * INROWB + ((cg ^ fkey(key)) << 4) + ((s16 & 1) << 3);
    tr_dst[rnd] = VBASE + dcol * 128 + ((ch ^ attn_swz_k<128>(dcol)) << 4);
  }
  auto convert_v = [&](int stg, int slot) __attribute__((always_inline)) {
    if constexpr (VT) {
#pragma unroll
      for (int rnd = 0; rnd < 2; ++rnd) {
        const i32x2 t = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(smem + tr_src[rnd] + stg * STGTILE));
        u32x4 o;
        o[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t[0], 1.0f, false));
        o[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t[0], 1.0f, true));
        o[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t[1], 1.0f, false));
        o[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t[1], 1.0f, true));
        *(LDS_AS u32x4*)(smem + tr_dst[rnd] + slot * TILEB) = o;
      }
    } else {
      u32x4 lo, hi;
      cvt16(*(const LDS_AS u32x4*)(smem + st_self + stg * STGTILE), lo, hi);
      *(LDS_AS u32x4*)(smem + cv_v0 + slot * TILEB) = lo;
      *(LDS_AS u32x4*)(smem + cv_v1 + slot * TILEB) = hi;
    }
  };
  // bundle b = key tile b+1 (the last tile again if there is none) and value tile b
  auto issue_bundle_k = [&](int b, int slot) __attribute__((always_inline)) { issue_k(min(b + 1, nt - 1), slot); };
  auto staging_read_done = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };

  issue_k(0, NSLOT - 1);  // key tile 0 borrows the K part of the last slot
  issue_bundle_k(0, 0);
  stage_v(0, 0);

  // ---- Q operand (B operand of S^T = K Q^T), fp8: lane (qi,h) holds Q[row][64kk + 32h .. +31] ----
  i32x8 qf[NK8];
  {
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * INROWB + h * 32;
#pragma unroll
    for (int kk = 0; kk < NK8; ++kk) {
      const u32x4 lo = *(const u32x4*)(src + kk * 64), hi = *(const u32x4*)(src + kk * 64 + 16);
      qf[kk] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
  }
  const int unit_scale = 0x7f7f7f7f;  // E8M0 exponent 127 = 2^0 for both block scales

  // ---- LDS read addresses (slot 0, first 32-key block) -----------------------------------------
  // K operand: lane (qi,h) reads key row qi, bytes 64kk + 32h .. +31 = chunks 4kk + 2h, +1
  uint32_t kaddr[NK8][2];
#pragma unroll
  for (int kk = 0; kk < NK8; ++kk)
#pragma unroll
    for (int e = 0; e < 2; ++e) kaddr[kk][e] = qi * KROWB + (((4 * kk + 2 * h + e) ^ attn_swz_k<KROWB>(qi)) << 4);
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
  // block id = 2 * slot + (which 32-key half): byte offsets of that block in the K and in the V ring
  auto koff_of = [](auto bid) __attribute__((always_inline)) { return (bid >> 1) * KTILEB + (bid & 1) * KSUBB; };
  auto voff_of = [](auto bid) __attribute__((always_inline)) { return (bid >> 1) * TILEB; };  // slot of the value tile; bid & 1 is the half
  auto k_half = [&](int koff, int kk, int e) __attribute__((always_inline)) { return *(LDS_AS u32x4*)(smem + kaddr[kk][e] + koff); };
  // VT: fragment (cb, kc) of 32-key half kb: row 32 cb + qi of V^T, chunk 4 kb + 2 kc + h
  uint32_t vtaddr[2][NCB][2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int kc = 0; kc < 2; ++kc) {
        const int dcol = 32 * cb + qi;
        vtaddr[kb][cb][kc] = VBASE + dcol * 128 + (((4 * kb + 2 * kc + h) ^ attn_swz_k<128>(dcol)) << 4);
      }
  // voff: offset of the value tile's ring slot; kb: which 32-key half
  auto v_operand = [&](auto voff, int kb, int cb, int kc) __attribute__((always_inline)) {
    if constexpr (VT) {
      return *(LDS_AS u32x4*)(smem + vtaddr[kb][cb][kc] + voff);
    } else {
      const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + voff + kb * SUBB + kc * 16 * ROWB));
      const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + voff + kb * SUBB + kc * 16 * ROWB));
      s16x8 av;
      av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
      av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
      return __builtin_bit_cast(u32x4, av);
    }
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
  auto join = [](const u32x4 lo, const u32x4 hi) __attribute__((always_inline)) {
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
  };
  auto qk_block = [&](f32x16& s, int koff) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NK8; ++kk)
      s = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(join(k_half(koff, kk, 0), k_half(koff, kk, 1)), qf[kk], s, 0, 0, 0, unit_scale, 0,
                                                          unit_scale);
  };
  auto pv_block = [&](const u32x4 (&pk)[2], int voff, int kb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2 * NCB; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb ? v_operand(voff, 1, cb, kc) : v_operand(voff, 0, cb, kc)),
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
  // MFMA m of a step: m = 0 and m = 5 are the two fp8 QK^T MFMAs (a dependent chain, kept four
  // PV MFMAs apart), the others the eight bf16 PV MFMAs.  Every MFMA's operand is two LDS reads:
  // the two 16-byte halves of a K fragment, or the two transposing reads of a V fragment.
  constexpr int NM = 10;
  struct Operand {
    u32x4 x, y;  // K: low and high half; V: the fragment in x
  };
  Operand pre[RA];
  auto step_operand = [&](auto bid, int m) __attribute__((always_inline)) {
    Operand o;
    if (m == 0 || m == 5) {
      o.x = k_half(koff_of(bid), m / 5, 0);
      o.y = k_half(koff_of(bid), m / 5, 1);
    } else {
      const int i = m - 1 - (m > 5);
      o.x = v_operand(voff_of(bid), bid & 1, i % NCB, i / NCB);
      o.y = o.x;
    }
    return o;
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
  auto step_hot = [&](f32x16& s_in, f32x16& s_out, u32x4 (&p_out)[2], u32x4 (&p_pv)[2], auto bid, auto bidnext) __attribute__((always_inline)) {
    Operand op[NM];
#pragma unroll
    for (int m = 0; m < RA; ++m) op[m] = pre[m];
#pragma unroll
    for (int r = 0; r < 16; ++r) s_out[r] = 0.f;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      if (m == 0 || m == 5) {
        s_out = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(join(op[m].x, op[m].y), qf[m / 5], s_out, 0, 0, 0, unit_scale, 0, unit_scale);
      } else {
        const int i = m - 1 - (m > 5);
        oacc[i % NCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m].x), __builtin_bit_cast(bf16x8, p_pv[i / NCB]),
                                                                oacc[i % NCB], 0, 0, 0);
      }
      if (m + RA < NM) op[m + RA] = step_operand(bid, m + RA);
      else pre[m + RA - NM] = step_operand(bidnext, m + RA - NM);
    }
    float ls = exp_block(s_in, p_out);
    constexpr int NVALU = 16 + 14 + 8 + 2;  // multiply-adds, adds, packs, final add + compare
    hy_step_pipeline<0, NM, NVALU, RA, VT ? 1 : 2>();
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
                      int voff, int kb) __attribute__((always_inline)) {
    if (do_sm) softmax_block(s_in, p_out, p_pv, key0, needs_mask(key0));
    if (do_mm) {
      qk_block(s_out, koff);
      pv_block(p_pv, voff, kb);
    }
  };

  // ---- prologue: block 0 ---------------------------------------------------------------------------
  // everything requested so far has landed: convert value tile 0, request bundle 1 and value tile 2
  ATTN_WAIT_VMCNT(0);
#pragma unroll
  for (int kk = 0; kk < NK8; ++kk)
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(qf[kk][i]));  // Q is in registers from here on
  if (VT) attn_wg_barrier();  // the transposing pass reads what other threads staged
  convert_v(0, 0);
  staging_read_done();
  if (nt > 1) {
    issue_bundle_k(1, 1);
    stage_v(1, 1);
  }
  if (!VT && nt > 2) stage_v(2, 0);
  attn_wg_barrier();
  if (VT && nt > 2) stage_v(2, 0);  // only now has every thread read staging slot 0
  if (wave_valid) {
    qk_block(s_b, (NSLOT - 1) * KTILEB);                         // S(0)
    softmax_block(s_b, p_b, p_a, 0, needs_mask(0));    // P(0) -> p_b (nothing pending yet)
    qk_block(s_a, (NSLOT - 1) * KTILEB + KSUBB);                 // S(1); ignored if block 1 is not visible
  }
  // bundle 1 has arrived once only value tile 2's load is outstanding: convert its value tile into slot 1
  if (nt > 1) {
    if (nt > 2) ATTN_WAIT_VMCNT(1);
    else ATTN_WAIT_VMCNT(0);
    if (VT) attn_wg_barrier();
    convert_v(1, 1);
  }
  attn_wg_barrier();  // the K part of the last slot is empty again
#pragma unroll
  for (int m = 0; m < RA; ++m) pre[m] = step_operand(ic<0>{}, m);  // first operands of the first pipelined step (block id 0)

  // ---- main loop over bundles ------------------------------------------------------------------------
  // iteration b: exponentiate blocks 2b+1 and 2b+2, compute the scores of blocks 2b+2 and 2b+3
  // (key tile b+1), accumulate blocks 2b and 2b+1 (value tile b)
  // between the two steps of iteration b: bundle b+1 (requested one iteration ago, the only
  // loads in flight) is published, and the slot of bundle b-1, which every wave has finished
  // reading, is handed to bundle b+2
  // the barrier publishes bundle b+1 (its key tile straight from memory, its value tile converted
  // one iteration ago) and frees the slot of bundle b-1: the key tile of bundle b+2 is requested
  // into it, the staged value tile of bundle b+2 is converted into it, and the value tile of
  // bundle b+3 is requested into the staging slot that of bundle b+1 was converted from
  auto bundle_mid = [&](int b, int free_slot) __attribute__((always_inline)) {
    ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
    if (b + 2 < nt) {
      issue_bundle_k(b + 2, free_slot);
      convert_v(b & 1, free_slot);
    }
    if (b + 3 < nt) stage_v(b + 3, (b + 1) & 1);
  };
  auto bundle_hot = [&](int b, auto slot_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    step_hot(s_a, s_b, p_a, p_b, ic<2 * SLOT>{}, ic<2 * SLOT + 1>{});
    bundle_mid(b, (SLOT + NSLOT - 1) % NSLOT);
    step_hot(s_b, s_a, p_b, p_a, ic<2 * SLOT + 1>{}, ic<2 * ((SLOT + 1) % NSLOT)>{});
  };
  auto bundle_any = [&](int b, int slot) __attribute__((always_inline)) {
    const int k1 = (2 * b + 1) * 32, k2 = k1 + 32;
    step_any(is_active(k1), k1, is_active(k1 - 32), s_a, s_b, p_a, p_b, slot * KTILEB, slot * TILEB, 0);
    bundle_mid(b, slot >= 1 ? slot - 1 : NSLOT - 1);
    step_any(is_active(k2), k2, is_active(k1), s_b, s_a, p_b, p_a, slot * KTILEB + KSUBB, slot * TILEB, 1);
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
  }
  // the last fully visible bundles (fewer than a turn), then the masked / partly visible ones
  int slot = 0;
  if (b < n_hot) { bundle_hot(b, ic<0>{}); ++b; slot = 1; }
  if (b < n_hot) { bundle_hot(b, ic<1>{}); ++b; slot = 2; }
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

template <int D, bool VT>
int launch_hy(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_fp8_hy_kernel<D, true, VT>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_fp8_hy_kernel<D, false, VT>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_fp8_hy_variants(int* count) {
  static const AttnVariant table[] = {
      {"fp8 d128 fp8-QK bf16-PV pipelined BM256 BN64", 1, 128, 256, 64, 512, 3 * 64 * 128 + 3 * 64 * 256 + 2 * 64 * 128, launch_hy<128, false>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}

const AttnVariant* attn_fp8_ht_variants(int* count) {
  static const AttnVariant table[] = {
      {"fp8 d128 fp8-QK bf16-PV transposed-V pipelined BM256 BN64", 1, 128, 256, 64, 512, 3 * 64 * 128 + 3 * 64 * 256 + 2 * 64 * 128, launch_hy<128, true>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
