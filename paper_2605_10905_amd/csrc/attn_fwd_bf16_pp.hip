// Fused attention forward, bf16, gfx950: the two-wave-group ("ping-pong") kernel.
//
// Same mathematics and the same transposed-product register layout as
// attn_fwd_bf16.hip (S^T = K Q^T, O^T += V^T P^T on 32x32x16 bf16 MFMA, one query
// per lane).  What differs is the orchestration, which is this build's rendering
// of the paper's multi-warp-group model (sections 1 and 4.1: wave groups that run
// different instruction streams, joined by explicit wait/arrive points):
//
//   * The 8 waves of a workgroup form two groups of four (one wave of each group
//     per SIMD).  Every wave alternates between a VALU phase (row max, exponentials,
//     packing P for one 32-key block) and an MFMA phase (the PV product of that
//     block fused with the QK^T product of the NEXT block, 16 MFMA back to back).
//     Group 1 runs one phase behind group 0, so on every SIMD one wave is feeding
//     the matrix pipe while the other is feeding the vector pipe; a workgroup
//     barrier at every phase boundary keeps the two groups in anti-phase.
//   * K/V tiles (64 keys) stream through a THREE-slot LDS ring by direct-to-LDS
//     loads issued two tiles ahead; s_waitcnt vmcnt(n) with n = the loads of the
//     newest tile lets those stay in flight while the older tile is published by
//     the next barrier ("full"); a slot is overwritten only after the barrier that
//     ends the last phase reading it ("empty").  stage = tile mod 3.
//   * No block maximum is taken on the common path.  The exponentials of a block are
//     computed against the CURRENT reference maximum; only when a lane's partial row sum
//     comes out large (or not a number, as on the very first block where the reference
//     is -inf) is the true block maximum taken, the reference raised, the accumulator
//     rescaled and the block redone.  This is exact: any reference value is valid for
//     the streaming softmax as long as nothing overflows.  The rescale then runs once
//     or twice per row instead of once per tile, and the per-score vector work is one
//     multiply-add, one exponential, one add and half a pack.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

__device__ __forceinline__ constexpr int ilog2c(int x) { return x <= 1 ? 0 : 1 + ilog2c(x >> 1); }

// 16-byte-chunk XOR swizzles of the K and V tiles (see attn_fwd_bf16.hip)
template <int ROWB>
__device__ __forceinline__ constexpr int swz_k(int row) {
  constexpr int NCH = ROWB / 16, BITS = ilog2c(NCH), RP = 256 / ROWB;
  const int a = (row / RP) & (NCH - 1);
  return ((a << 1) | (a >> (BITS - 1))) & (NCH - 1);
}
template <int ROWB>
__device__ __forceinline__ constexpr int swz_v(int row) {
  constexpr int NCH = ROWB / 16, RP = 256 / ROWB;
  return ((row / RP) & (NCH / 4 - 1)) << 2;
}

__device__ __forceinline__ float max_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Direct-to-LDS 128-bit load: lane i of the wave copies 16 bytes from sbase + voff to LDS
// address lds_base + 16*i.  Written as inline assembly (uniform 64-bit base in SGPRs plus
// a per-lane 32-bit offset, no VALU address arithmetic) so that the compiler does not
// serialise later LDS reads of OTHER ring slots behind it; completion is tracked by hand
// with s_waitcnt vmcnt before the barrier that publishes the slot.
__device__ __forceinline__ void lds_dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase));
}

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left alone)
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))

__device__ __forceinline__ void wg_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

#ifdef ATTN_PHASE_TIMING
__device__ long long g_phase_timing[8][4];
#define PT_NOW() __builtin_readcyclecounter()
#define PT_ADD(slot, t0) do { const long long t1_ = PT_NOW(); pt[slot] += t1_ - (t0); (t0) = t1_; } while (0)
#else
#define PT_ADD(slot, t0) do { } while (0)
#endif

// A lane's partial row sum of one 32-key block (16 exponentials) above this sends the block
// through the slow pass that raises the reference maximum; below it every exponential is
// < 2^16 and fp32 / bf16 ranges are nowhere near.
constexpr float kSumLimit = 65536.0f;

#ifndef ATTN_PP_FULLRA
#define ATTN_PP_FULLRA 1
#endif
#ifndef ATTN_PP_RA_EARLY
#define ATTN_PP_RA_EARLY 1
#endif

template <int D, bool CAUSAL, int NSLOT>
__global__ void __launch_bounds__(512, 2) attn_fwd_bf16_pp_kernel(const AttnParams p) {
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int NKK = D / 16;       // MFMA k-steps over the head dimension
  constexpr int NCB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;       // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row
  constexpr int TILEB = BN * ROWB;  // bytes per K (or V) tile
  constexpr int SUBB = 32 * ROWB;   // bytes per 32-key block
  constexpr int PD = NSLOT - 1;  // tiles requested ahead of the one being consumed
  constexpr int VBASE = NSLOT * TILEB;  // K slots first, then V slots
  constexpr int NLD = BN * NCH / NT;    // direct-to-LDS loads per thread per tile per tensor
  static_assert(BN * NCH % NT == 0 && NLD >= 1, "tile must divide evenly over the workgroup");
  static_assert((NSLOT - 1) * TILEB + SUBB + 16 * ROWB < 65536, "ring offsets must fit the 16-bit LDS immediate");
  static_assert(NSLOT == 3 || NSLOT == 4, "ring depth");

  // static allocation: the ring then sits at a link-time-known LDS address and every ring
  // offset folds into the 16-bit immediate of the LDS instructions
  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int grp = w >> 2;    // wave group: 0 leads, 1 runs one phase behind
  const int qi = lane & 31;  // query column within the wave's 32-query block
  const int h = lane >> 5;   // which half of the k-slots / accumulator rows this lane holds

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  const int hk = tc.hq / G;
  const int q0 = tc.t * BM;
  const int wq0 = q0 + w * 32;  // first query row of this wave
  const bool wave_valid = wq0 < N;

  const char* const qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;  // keys the workgroup visits
  const int nt = (kv_end + BN - 1) / BN;

  // ---- producer role: direct-to-LDS tile loads ---------------------------------------
  int ld_row[NLD];
  uint32_t ld_koff[NLD], ld_voff[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCH, c = s % NCH;
    ld_row[it] = r;
    ld_koff[it] = r * ROWB + ((c ^ swz_k<ROWB>(r)) << 4);
    ld_voff[it] = r * ROWB + ((c ^ swz_v<ROWB>(r)) << 4);
  }
  auto issue_tile_loads = [&](int j, int slot) __attribute__((always_inline)) {
    const uint32_t kdst = (uint32_t)(uintptr_t)(smem + slot * TILEB + w * 1024);
    const uint32_t vdst = kdst + VBASE;
    const char* const kt = khead + (size_t)j * TILEB;
    const char* const vt = vhead + (size_t)j * TILEB;
    if ((j + 1) * BN <= N) {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        lds_dma16(kt, ld_koff[it], kdst + it * NT * 16);
        lds_dma16(vt, ld_voff[it], vdst + it * NT * 16);
      }
    } else {
      // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const uint32_t over = (uint32_t)max(0, j * BN + ld_row[it] - (N - 1)) * ROWB;
        lds_dma16(kt, ld_koff[it] - over, kdst + it * NT * 16);
        lds_dma16(vt, ld_voff[it] - over, vdst + it * NT * 16);
      }
    }
  };

  issue_tile_loads(0, 0);

  // ---- Q operand (B operand of S^T = K Q^T): lane (qi,h) holds Q[row][16kk+8h .. +7] ----
  bf16x8 qf[NKK];
  {
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8*)(src + kk * 32);
  }
  if (nt > 1) issue_tile_loads(1, 1);
  if (PD > 2 && nt > 2) issue_tile_loads(2, 2);

  // ---- LDS read addresses (slot 0, first 32-key block) ---------------------------------
  uint32_t kaddr[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = qi * ROWB + (((2 * kk + h) ^ swz_k<ROWB>(qi)) << 4);
  uint32_t vaddr[NCB][2];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int key = 8 * e + 4 * h + (s >> 2);
        const int chunk = cb * 4 + chalf * 2 + ((s & 3) >> 1);
        vaddr[cb][e] = VBASE + key * ROWB + ((chunk ^ swz_v<ROWB>(key)) << 4) + ((s & 1) << 3);
      }
  }

  // ---- streaming-softmax state ---------------------------------------------------------
  f32x16 oacc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_ref = -INFINITY;  // reference maximum, in scaled log2 units
  float l_run = 0.f;        // this lane's share of the row sum (the two halves are added at the end)
  const float c = p.scale_log2;
  const int qrow = wq0 + qi;
  const int limit = CAUSAL ? min(qrow, N - 1) : (N - 1);  // last visible key of this lane's query
  const int wlast = wq0 + 31;                             // last query row of the wave

  f32x16 s;        // S^T of the block the next VALU phase consumes
  u32x4 pk[2];     // P^T of the block the next MFMA phase consumes (two 16-key operands)

  // S^T block = K[32 keys] Q^T from LDS slot/sub-block at byte offset `koff`
  auto qk_block = [&](int koff) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const bf16x8 a = *(LDS_AS bf16x8*)(smem + kaddr[kk] + koff);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s, 0, 0, 0);
    }
  };
  // one O^T update: column block cb, 16-key operand kc of the block at byte offset `voff`
  auto pv_step = [&](auto voff, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + voff + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + voff + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, pk[kc]), oacc[cb], 0, 0, 0);
  };

  // VALU phase: mask, row max, (rare) rescale, P = exp2(c S - m_ref), row sum
  auto valu_phase = [&](int key0, bool need_mask) __attribute__((always_inline)) {
    if (need_mask) {
      const int kbase = key0 + 4 * h;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kbase + 8 * (r >> 2) + (r & 3) > limit) s[r] = -INFINITY;
    }
    // Optimistic pass: exponentials relative to the CURRENT reference maximum, no block
    // maximum taken.  Any reference is valid for the streaming softmax as long as nothing
    // overflows, so the pass stands unless some lane's partial sum is large (or not a
    // number: the first block starts from m_ref = -inf and always lands in the slow pass).
    f32x16 e;
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -m_ref));
    float ls0 = e[0], ls1 = e[1];
#pragma unroll
    for (int r = 1; r < 8; ++r) {
      ls0 += e[2 * r];
      ls1 += e[2 * r + 1];
    }
    float ls = ls0 + ls1;
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) {
      // slow pass: raise the reference to the true block maximum, rescale, redo the block
      float mx = fmaxf(s[0], s[1]);
#pragma unroll
      for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
      mx = max_halves(mx) * c;
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // exp2(-inf) = 0 on the first block
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -m_ref));
      ls0 = e[0], ls1 = e[1];
#pragma unroll
      for (int r = 1; r < 8; ++r) {
        ls0 += e[2 * r];
        ls1 += e[2 * r + 1];
      }
      ls = ls0 + ls1;
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      bf16x2 t;
      t[0] = (__bf16)e[2 * r];
      t[1] = (__bf16)e[2 * r + 1];
      pk[r >> 2][r & 3] = __builtin_bit_cast(uint32_t, t);
    }
    l_run += ls;
    // everything above belongs to this phase: keep the compiler from sinking the
    // exponentials past the phase barrier into the matrix phase
    asm volatile("" : "+v"(pk[0]), "+v"(pk[1]), "+v"(l_run));
  };

  // MFMA phase: O^T += V^T P^T for the current block, interleaved with S^T of the next block
  // (the two chains are independent, so consecutive MFMAs never wait on each other).  When
  // the next block is one this wave never consumes, its S^T is computed on whatever the
  // LDS slot holds and then ignored.
  auto mfma_phase = [&](auto voff, auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    constexpr int NPV = NCB * 2;
#pragma unroll
    for (int i = 0; i < (NKK > NPV ? NKK : NPV); ++i) {
      if (i < NKK) {
        const bf16x8 a = *(LDS_AS bf16x8*)(smem + kaddr[i] + koff);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[i], s, 0, 0, 0);
      }
      if (i < NPV) pv_step(voff, i % NCB, i / NCB);
    }
  };

  // Operands of the first half of an MFMA phase, read from LDS at the END of the preceding
  // VALU phase (before the phase barrier), so that the matrix pipe starts the moment the
  // barrier opens instead of waiting for LDS latency.
  constexpr int KP = NKK / 2;  // K operands read ahead (k-steps 0 .. KP-1)
  bf16x8 kpre[KP];
  s16x8 vpre[NCB];             // V operands of the first 16 keys, all column blocks
  auto v_operand = [&](auto voff, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + voff + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + voff + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return av;
  };
  auto read_ahead = [&](auto voff, auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < (KP > NCB ? KP : NCB); ++i) {
      if (i < KP) kpre[i] = *(LDS_AS bf16x8*)(smem + kaddr[i] + koff);
      if (i < NCB) vpre[i] = v_operand(voff, i, 0);
    }
  };
  // The phase itself, in a fixed order: step i issues the i-th QK^T MFMA and the i-th PV MFMA
  // (independent accumulators, so neither waits for the other), then requests the operands of
  // step i + KP into the registers it has just freed.
  auto mfma_phase_ra = [&](auto voff, auto koff) __attribute__((always_inline)) {
    static_assert(NKK == 2 * NCB && KP == NCB, "step pairing assumes D/16 QK steps and 2*D/32 PV steps");
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int i = 0; i < NKK; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kpre[i % KP], qf[i], s, 0, 0, 0);
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vpre[cb]), __builtin_bit_cast(bf16x8, pk[kc]), oacc[cb], 0, 0, 0);
      if (i < KP) {
        kpre[i] = *(LDS_AS bf16x8*)(smem + kaddr[i + KP] + koff);
        vpre[cb] = v_operand(voff, cb, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Variant with every operand of the phase read ahead (the vector phase has the slack to
  // carry all the LDS reads): the matrix phase is then 2*NKK MFMAs back to back, no LDS wait.
  bf16x8 kall[NKK];
  s16x8 vall[NKK];
  auto read_all = [&](auto voff, auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NKK; ++i) {
      kall[i] = *(LDS_AS bf16x8*)(smem + kaddr[i] + koff);
      vall[i] = v_operand(voff, i % NCB, i / NCB);
    }
  };
  auto mfma_burst = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int i = 0; i < NKK; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kall[i], qf[i], s, 0, 0, 0);
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vall[i]), __builtin_bit_cast(bf16x8, pk[kc]), oacc[cb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // tile 0 (and Q) have landed once only the loads of the later tiles are outstanding
  if (PD > 2 && nt > 2) WAIT_VMCNT(4 * NLD);
  else if (nt > 1) WAIT_VMCNT(2 * NLD);
  else WAIT_VMCNT(0);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) asm volatile("" ::"v"(qf[kk]));  // Q is in registers from here on
  wg_barrier();
  if (grp == 1) wg_barrier();  // group 1 starts one phase late
  if (wave_valid) qk_block(0);

  // does the 32-key block starting at key0 hold a key some query of this wave can see?
  auto is_active = [&](int key0) __attribute__((always_inline)) {
    return wave_valid && key0 < kv_end && (!CAUSAL || key0 <= wlast);
  };
  // producer step: tile j+2 is requested at the start of the first MFMA phase of tile j and
  // waited for at the end of the first VALU phase of tile j+1, so that the barrier closing
  // that phase publishes it
  auto prefetch = [&](int j, int slot) __attribute__((always_inline)) {
    if (j + PD < nt) issue_tile_loads(j + PD, slot);
  };
  // tile j+1 must have landed; with a four-slot ring the loads of tile j+2 may stay in flight
  auto publish_wait = [&](int j) __attribute__((always_inline)) {
    if (PD > 2 && j + 2 < nt) WAIT_VMCNT(2 * NLD);
    else WAIT_VMCNT(0);
  };

  // A tile whose 64 keys are visible to every query of the wave: straight-line code, all
  // LDS offsets are immediates (SLOT is a compile-time constant).
#ifdef ATTN_PHASE_TIMING
  long long pt[4] = {0, 0, 0, 0};
  long long tp = PT_NOW();
#else
  int tp = 0;
#endif
  auto tile_hot = [&](int j, auto slot_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    constexpr std::integral_constant<int, SLOT * TILEB> v0off{};
    constexpr std::integral_constant<int, SLOT * TILEB + SUBB> v1off{}, k1off{};
    constexpr std::integral_constant<int, ((SLOT + 1) % NSLOT) * TILEB> knoff{};
    // first 32 keys
#if ATTN_PP_FULLRA
    if (ATTN_PP_RA_EARLY) { read_all(v0off, k1off); __builtin_amdgcn_sched_barrier(0); }
    valu_phase(0, false);
    if (!ATTN_PP_RA_EARLY) read_all(v0off, k1off);
#else
    valu_phase(0, false);
    read_ahead(v0off, k1off);
#endif
    publish_wait(j);
    PT_ADD(0, tp);
    wg_barrier();
    PT_ADD(1, tp);
    prefetch(j, (SLOT + PD) % NSLOT);
    __builtin_amdgcn_s_setprio(1);
#if ATTN_PP_FULLRA
    mfma_burst();
#else
    mfma_phase_ra(v0off, k1off);
#endif
    __builtin_amdgcn_s_setprio(0);
    PT_ADD(2, tp);
    wg_barrier();
    PT_ADD(3, tp);
    // second 32 keys; the S^T computed here belongs to the first block of tile j+1
#if ATTN_PP_FULLRA
    if (ATTN_PP_RA_EARLY) { read_all(v1off, knoff); __builtin_amdgcn_sched_barrier(0); }
    valu_phase(0, false);
    if (!ATTN_PP_RA_EARLY) read_all(v1off, knoff);
#else
    valu_phase(0, false);
    read_ahead(v1off, knoff);
#endif
    PT_ADD(0, tp);
    wg_barrier();
    PT_ADD(1, tp);
    __builtin_amdgcn_s_setprio(1);
#if ATTN_PP_FULLRA
    mfma_burst();
#else
    mfma_phase_ra(v1off, knoff);
#endif
    __builtin_amdgcn_s_setprio(0);
    PT_ADD(2, tp);
    wg_barrier();
    PT_ADD(3, tp);
  };
  // Any tile: blocks may be partly masked (causal diagonal, ragged end of K) or not visible
  // to this wave at all; the ring slot is a run-time value.
  auto tile_any = [&](int j, int slot) __attribute__((always_inline)) {
    const int nslot = slot == NSLOT - 1 ? 0 : slot + 1;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int key0 = j * BN + kb * 32;
      const bool active = is_active(key0);
      if (active) valu_phase(key0, (CAUSAL && key0 + 31 > wq0) || key0 + 31 >= N);
      if (kb == 0) publish_wait(j);
      wg_barrier();
      if (kb == 0) prefetch(j, slot >= 1 ? slot - 1 : NSLOT - 1);
      if (active) {
        __builtin_amdgcn_s_setprio(1);
        if (kb == 0) mfma_phase(slot * TILEB, slot * TILEB + SUBB);
        else mfma_phase(slot * TILEB + SUBB, nslot * TILEB);
        __builtin_amdgcn_s_setprio(0);
      }
      wg_barrier();
    }
  };

  // tiles 0 .. n_hot-1 need neither masking nor activity checks for this wave
  int n_hot = wave_valid ? (CAUSAL ? min(wq0 + 1, N) : N) / BN : 0;
  n_hot -= n_hot % NSLOT;
  int j = 0;
  for (; j < n_hot; j += NSLOT) {
    tile_hot(j, std::integral_constant<int, 0>{});
    tile_hot(j + 1, std::integral_constant<int, 1>{});
    tile_hot(j + 2, std::integral_constant<int, 2>{});
    if (NSLOT > 3) tile_hot(j + 3, std::integral_constant<int, 3 % NSLOT>{});
  }
  for (int slot = 0; j < nt; ++j) {  // j is a multiple of NSLOT here, so the ring is at slot 0
    tile_any(j, slot);
    slot = slot == NSLOT - 1 ? 0 : slot + 1;
  }
  if (grp == 0) wg_barrier();  // balance group 1's extra leading barrier
#ifdef ATTN_PHASE_TIMING
  if (blockIdx.x == 0 && lane == 0)
    for (int i = 0; i < 4; ++i) g_phase_timing[w][i] = pt[i];
#endif

  // ---- epilogue: O = acc / l (bf16), lse = (m + log2 l) * ln 2 ---------------------------
  char* const ohead = (char*)p.o + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  float* const lsehead = p.lse + (size_t)(tc.b * p.Hq + tc.hq) * N;
  {
    const float l = sum_halves(l_run);
    const float inv = p.out_scale / l;
    if (qrow < N && h == 0) lsehead[qrow] = (m_ref + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
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
          *(u32x4*)(ohead + (size_t)qrow * ROWB + (cb * 32 + a * 16 + h * 8) * 2) = out;
        }
      }
  }
}

template <int D, int NSLOT>
int launch_pp(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_pp_kernel<D, true, NSLOT>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_bf16_pp_kernel<D, false, NSLOT>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

#ifdef ATTN_PHASE_TIMING
extern "C" int attn_debug_phase_timing(long long* out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_timing), sizeof(long long) * 32);
}
#endif

const AttnVariant* attn_bf16_pp_variants(int* count) {
  static const AttnVariant table[] = {
      {"bf16 d128 ping-pong BM256 BN64 ring3", 0, 128, 256, 64, 512, 2 * 3 * 64 * 128 * 2, launch_pp<128, 3>},
      {"bf16 d64 ping-pong BM256 BN64 ring4", 0, 64, 256, 64, 512, 2 * 4 * 64 * 64 * 2, launch_pp<64, 4>},
      {"bf16 d128 ping-pong BM256 BN64 ring4", 0, 128, 256, 64, 512, 2 * 4 * 64 * 128 * 2, launch_pp<128, 4>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
