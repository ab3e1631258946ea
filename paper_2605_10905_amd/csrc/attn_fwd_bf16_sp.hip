// Fused attention forward, bf16, gfx950: the software-pipelined kernel.
//
// Mathematics and register layout are those of attn_fwd_bf16.hip (transposed products on
// 32x32x16 bf16 MFMA, one query per lane): paper section 6.1 for the phases, appendix C.3
// for the streaming-softmax state and the overlap of one block's QK^T product with the
// previous block's PV product.
//
// Orchestration.  All 8 waves of a workgroup run the same instruction stream, and that
// stream is pipelined over 32-key blocks so that the matrix pipe and the vector pipe are fed
// from the SAME wave at the same time (measured on gfx950: a wave that issues only MFMAs and
// a sibling that issues only VALU work delay each other at the shared issue port; one MFMA
// followed by three to five independent VALU instructions from the same wave is nearly
// free).  In the step that handles block u a wave
//     * exponentiates block u            (VALU:  P(u)   = exp2(c S(u) - m))
//     * computes the scores of block u+1 (MFMA:  S(u+1) = K(u+1) Q^T)
//     * accumulates block u-1            (MFMA:  O^T   += V(u-1)^T P(u-1)^T)
// The three streams are independent inside a step; a scheduling-group pipeline at the end of
// the step tells the compiler's scheduler the interleave: per MFMA one exponential, two or
// three plain vector instructions and the LDS reads of the operand a few MFMAs ahead.
//
// K/V streaming.  Block u+1 of K and block u-1 of V travel together: "bundle" b holds key
// tile b+1 and value tile b (64 keys each) and is consumed by exactly one loop iteration, so
// a three-slot LDS ring with direct-to-LDS loads issued two bundles ahead needs one
// workgroup barrier per 64 keys: it is both the "full" signal of bundle b+1 and the "empty"
// signal of bundle b-1 (stage = b mod 3).  The barrier sits between the two 32-key steps of an
// iteration so that the first K operands of the next iteration can be read one step early.
//
// No block maximum is taken on the common path: exponentials are computed against the
// current reference maximum, and only when a lane's partial row sum comes out large (or not a
// number, as on the very first block) is the true block maximum taken, the reference raised,
// the accumulator rescaled and the block redone (exact: any reference is valid for the
// streaming softmax as long as nothing overflows).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

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
template <int M, int M1, int RA, int NVALU, int NEXP, int M0 = M>
__device__ __forceinline__ void step_pipeline() {
  if constexpr (M < M1) {
    constexpr int NS = M1 - M0;  // MFMAs of this scheduling region; each has NEXP exponentials
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (M - M0 + 1)) / NS - (NVALU * (M - M0)) / NS, 0);    // VALU
    __builtin_amdgcn_sched_group_barrier(0x400, NEXP, 0);                                                     // transcendental
    __builtin_amdgcn_sched_group_barrier(0x100, ((M + RA) & 1) ? 2 : 1, 0);                                   // LDS read
    step_pipeline<M + 1, M1, RA, NVALU, NEXP, M0>();
  }
}

// PERSIST: the launch has one workgroup per CU, and each takes query tiles from a queue until
// it is drained.  The queue is 8 counters, one per XCD list of the static tile order (a tile
// index wg belongs to list wg % 8, the XCD the static launch would run it on, and lists are
// consumed heaviest tile first); a workgroup serves the list of the XCD it was dispatched to
// and, when that is empty, the lists after it, so every tile is taken exactly once whatever the
// dispatch order was.  This is the software stand-in for the paper's cluster launch control
// (section 4.2): dynamic assignment of tiles to resident workgroups.
template <int D, bool CAUSAL, bool PERSIST>
__global__ void __launch_bounds__(512, 2) attn_fwd_bf16_sp_kernel(const AttnParams p) {
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int NKK = D / 16;       // MFMA k-steps of S^T = K Q^T
  constexpr int NCB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;       // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row
  constexpr int TILEB = BN * ROWB;  // bytes per K (or V) tile
  constexpr int SUBB = 32 * ROWB;   // bytes per 32-key block
  constexpr int NSLOT = 3;  // ring depth: bundles are requested NSLOT-1 ahead
  constexpr int VBASE = NSLOT * TILEB;  // K parts of the slots first, then the V parts
  constexpr int NLD = BN * NCH / NT;    // direct-to-LDS loads per thread per tile
#ifndef ATTN_RA
#define ATTN_RA 4
#endif

  constexpr int RA = ATTN_RA;           // operands are read from LDS this many MFMAs ahead
  static_assert(BN * NCH % NT == 0 && NLD >= 1, "tile must divide evenly over the workgroup");
  static_assert(NKK == 2 * NCB && RA >= 2 && RA <= 2 * NKK, "one PV step per QK^T step; read-ahead within a step");
  static_assert((NSLOT - 1) * TILEB + SUBB + 16 * ROWB < 65536 && (NSLOT == 3 || NSLOT == 4), "ring offsets must fit the 16-bit LDS immediate");

  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;
  __shared__ int next_tile;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31;  // query column within the wave's 32-query block
  const int h = lane >> 5;   // which half of the k-slots / accumulator rows this lane holds

  int lists_tried = 0;  // used by thread 0 only
  for (;;) {
  int wg = blockIdx.x;
  if constexpr (PERSIST) {
    if (tid == 0) {
      int t = -1;
      while (lists_tried < 8) {
        const int x = (blockIdx.x + lists_tried) & 7;
        const int s = atomicAdd(p.queue + x * 32, 1);
        if (s * 8 + x < p.total) {
          t = s * 8 + x;
          break;
        }
        ++lists_tried;  // that list is drained (its counter keeps growing, which is harmless)
      }
      next_tile = t;
    }
    __syncthreads();  // also: every wave is done with the LDS ring of the previous tile
    wg = __builtin_amdgcn_readfirstlane(next_tile);
    __syncthreads();
    if (wg < 0) break;
  }
  const AttnTileCoord tc = attn_tile_coord_impl(wg, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
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
  const int nt = (kv_end + BN - 1) / BN;            // 64-key tiles = bundles

  // ---- producer role: direct-to-LDS tile loads ---------------------------------------------
  int ld_row[NLD];
  uint32_t ld_koff[NLD], ld_voff[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCH, c = s % NCH;
    ld_row[it] = r;
    ld_koff[it] = r * ROWB + ((c ^ attn_swz_k<ROWB>(r)) << 4);
    ld_voff[it] = r * ROWB + ((c ^ attn_swz_v<ROWB>(r)) << 4);
  }
  auto issue_tile = [&](const char* head, int t, const uint32_t (&off)[NLD], uint32_t dst) __attribute__((always_inline)) {
    const char* const base = head + (size_t)t * TILEB;
    if ((t + 1) * BN <= N) {
#pragma unroll
      for (int it = 0; it < NLD; ++it) attn_lds_dma16(base, off[it], dst + it * NT * 16);
    } else {
      // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const uint32_t over = (uint32_t)max(0, t * BN + ld_row[it] - (N - 1)) * ROWB;
        attn_lds_dma16(base, off[it] - over, dst + it * NT * 16);
      }
    }
  };
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  // Offsets of this thread's chunks inside the ragged last tile (rows past N-1 re-read row N-1),
  // so that a tile load inside the pipelined step is one select away from the regular one.
  uint32_t ld_koff_r[NLD], ld_voff_r[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const uint32_t over = (uint32_t)max(0, (nt - 1) * BN + ld_row[it] - (N - 1)) * ROWB;
    ld_koff_r[it] = ld_koff[it] - over;
    ld_voff_r[it] = ld_voff[it] - over;
  }
  // bundle b = key tile b+1 (the last tile again if there is none) and value tile b
  auto issue_bundle = [&](int b, int slot) __attribute__((always_inline)) {
    issue_tile(khead, min(b + 1, nt - 1), ld_koff, lds_wave + slot * TILEB);
    issue_tile(vhead, b, ld_voff, lds_wave + VBASE + slot * TILEB);
  };

  issue_tile(khead, 0, ld_koff, lds_wave + (NSLOT - 1) * TILEB);  // key tile 0 borrows the K part of the last slot
  issue_bundle(0, 0);

  // ---- Q operand (B operand of S^T = K Q^T): lane (qi,h) holds Q[row][16kk+8h .. +7] ----------
  bf16x8 qf[NKK];
  {
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8*)(src + kk * 32);
  }
  if (nt > 1) issue_bundle(1, 1);
  if (NSLOT > 3 && nt > 2) issue_bundle(2, 2);

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
  // NSEG > 1 cuts the step into NSEG scheduling regions of NM/NSEG MFMAs each (each with its own
  // share of the exponentials, sums and packs); between() runs at the cuts, which is where the
  // producer role's tile loads go.
  auto step_hot = [&](f32x16& s_in, f32x16& s_out, u32x4 (&p_out)[2], u32x4 (&p_pv)[2], auto off, auto offnext, auto nseg_tag, auto between) __attribute__((always_inline)) {
    constexpr int NSEG = decltype(nseg_tag)::value, SEG = NM / NSEG;
    static_assert(NM % NSEG == 0 && (16 / NSEG) % 2 == 0, "segments hold whole MFMAs and whole pairs of scores");
    u32x4 op[NM];
#pragma unroll
    for (int m = 0; m < RA; ++m) op[m] = pre[m];
#pragma unroll
    for (int r = 0; r < 16; ++r) s_out[r] = 0.f;
    float ls0 = 0.f, ls1 = 0.f;
    float e[16];
    auto segment = [&](auto seg_tag) __attribute__((always_inline)) {
      constexpr int SG = decltype(seg_tag)::value, M0 = SG * SEG, M1 = M0 + SEG;
      constexpr int R0 = 16 * SG / NSEG, R1 = 16 * (SG + 1) / NSEG;  // scores exponentiated in this region
#pragma unroll
      for (int m = M0; m < M1; ++m) {
        const int i = m >> 1;
        if (m & 1)
          oacc[i % NCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), __builtin_bit_cast(bf16x8, p_pv[i / NCB]),
                                                                  oacc[i % NCB], 0, 0, 0);
        else
          s_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), qf[i], s_out, 0, 0, 0);
        if (m + RA < NM) op[m + RA] = step_operand(off, m + RA);
        else pre[m + RA - NM] = step_operand(offnext, m + RA - NM);
      }
#pragma unroll
      for (int r = R0; r < R1; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[r], c, -m_ref));
#pragma unroll
      for (int u = R0 / 2; u < R1 / 2; ++u) {
        p_out[u >> 2][u & 3] = pack_bf16(e[2 * u], e[2 * u + 1]);
        ls0 = u == 0 ? e[0] : ls0 + e[2 * u];
        ls1 = u == 0 ? e[1] : ls1 + e[2 * u + 1];
      }
      // per MFMA one exponential, the plain vector work spread evenly, and the LDS reads of the
      // operand RA MFMAs ahead (one 128-bit K read or two transposing V reads)
      // multiply-adds, packs and adds of this region (the first pair starts the two sums, the
      // last region adds them and compares)
      constexpr int NVALU = (R1 - R0) + 3 * ((R1 - R0) / 2) - (SG == 0 ? 2 : 0) + (SG == NSEG - 1 ? 2 : 0);
      if constexpr (SG == NSEG - 1) ls0 += ls1;
      step_pipeline<M0, M1, RA, NVALU, 16 / NM>();
      if constexpr (SG + 1 < NSEG) {
        __builtin_amdgcn_sched_barrier(0);
        between(SG + 1);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    between(0);
    segment(ic<0>{});
    if constexpr (NSEG > 1) segment(ic<1>{});
    if constexpr (NSEG > 2) segment(ic<2>{});
    if constexpr (NSEG > 3) segment(ic<3>{});
    static_assert(NSEG <= 4, "at most four regions per step");
    float ls = ls0;
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) {
      // the redo path "reads" the optimistic packs, so that they are computed inside the
      // pipelined region above and not sunk below this branch into the common path's tail
      asm volatile("" ::"v"(p_out[0]), "v"(p_out[1]));
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
  // key tile 0 (and Q) have landed once only the bundle loads issued after them are outstanding
  if (NSLOT > 3 && nt > 2) ATTN_WAIT_VMCNT(6 * NLD);
  else if (nt > 1) ATTN_WAIT_VMCNT(4 * NLD);
  else ATTN_WAIT_VMCNT(2 * NLD);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) asm volatile("" ::"v"(qf[kk]));  // Q is in registers from here on
  attn_wg_barrier();
  if (wave_valid) {
    qk_block(s_b, (NSLOT - 1) * TILEB);                          // S(0)
    softmax_block(s_b, p_b, p_a, 0, needs_mask(0));    // P(0) -> p_b (nothing pending yet)
    qk_block(s_a, (NSLOT - 1) * TILEB + SUBB);                   // S(1); ignored if block 1 is not visible
  }
  if (NSLOT > 3 && nt > 2) ATTN_WAIT_VMCNT(4 * NLD);
  else if (nt > 1) ATTN_WAIT_VMCNT(2 * NLD);
  else ATTN_WAIT_VMCNT(0);
  attn_wg_barrier();  // bundle 0 is full; the K part of the last slot is empty again
#pragma unroll
  for (int m = 0; m < RA; ++m) pre[m] = step_operand(ic<0>{}, m);  // first operands of the first pipelined step

  // ---- main loop over bundles ------------------------------------------------------------------------
  // iteration b: exponentiate blocks 2b+1 and 2b+2, compute the scores of blocks 2b+2 and 2b+3
  // (key tile b+1), accumulate blocks 2b and 2b+1 (value tile b)
  // between the two steps of iteration b: bundle b+1 (requested one iteration ago, the only
  // loads in flight) is published, and the slot of bundle b-1, which every wave has finished
  // reading, is handed to bundle b+2
  auto bundle_mid = [&](int b, int free_slot) __attribute__((always_inline)) {
    if (NSLOT > 3 && b + 2 < nt) ATTN_WAIT_VMCNT(2 * NLD);  // bundle b+2 may stay in flight
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
    if (b + NSLOT - 1 < nt) issue_bundle(b + NSLOT - 1, free_slot);
  };
  auto no_loads = [](int) __attribute__((always_inline)) {};
  // Producer role inside the pipelined step: the barrier between the two steps of an iteration
  // frees a slot, and the loads of bundle b+NSLOT-1 into it are issued one at a time at the
  // region cuts of the second step, between its operand reads, instead of in a burst behind the
  // barrier (a burst keeps every wave of the workgroup off the matrix pipe at the same time).
  // A bundle index past the end re-requests the last bundle into the free slot, which is never
  // read again: the number of loads in flight per wave is then the same in every iteration.
  auto bundle_hot = [&](int b, auto slot_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    constexpr int FREE = (SLOT + NSLOT - 1) % NSLOT;
    constexpr int NSEG = 2 * NLD < 2 ? 2 : 2 * NLD;
    step_hot(s_a, s_b, p_a, p_b, ic<SLOT * TILEB>{}, ic<SLOT * TILEB + SUBB>{}, ic<1>{}, no_loads);
    const int bl = min(b + NSLOT - 1, nt - 1);        // bundle to request
    const int kt = min(bl + 1, nt - 1), vt = bl;      // its key and value tiles
    const char* const kbase = khead + (size_t)kt * TILEB;
    const char* const vbase = vhead + (size_t)vt * TILEB;
    const bool k_ragged = (kt + 1) * BN > N, v_ragged = (vt + 1) * BN > N;
    auto mid_and_loads = [&](int sg) __attribute__((always_inline)) {
      if (sg == 0) {
        if (NSLOT > 3) ATTN_WAIT_VMCNT(2 * NLD);  // bundle b+2 may stay in flight
        else ATTN_WAIT_VMCNT(0);
        attn_wg_barrier();
      }
#pragma unroll
      for (int j = 0; j < 2 * NLD; ++j) {
        if ((j < NSEG ? j : NSEG - 1) != sg) continue;
        if (j < NLD) attn_lds_dma16(kbase, k_ragged ? ld_koff_r[j] : ld_koff[j], lds_wave + FREE * TILEB + j * NT * 16);
        else attn_lds_dma16(vbase, v_ragged ? ld_voff_r[j - NLD] : ld_voff[j - NLD], lds_wave + VBASE + FREE * TILEB + (j - NLD) * NT * 16);
      }
    };
    step_hot(s_b, s_a, p_b, p_a, ic<SLOT * TILEB + SUBB>{}, ic<((SLOT + 1) % NSLOT) * TILEB>{}, ic<NSEG>{}, mid_and_loads);
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
  if constexpr (!PERSIST) break;
  }  // tile loop
}

template <int D>
int launch_sp(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<D, true, false>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<D, false, false>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

// zero the 8 list counters (a kernel, not a memset, so that the pair can be captured in a graph)
__global__ void attn_queue_reset_kernel(int* queue) {
  if (threadIdx.x < 8) queue[threadIdx.x * 32] = 0;
}

}  // namespace

int attn_fwd_bf16_persistent_launch(const AttnParams& p, int d, int workgroups, hipStream_t stream) {
  if (!p.queue || p.total <= 0 || workgroups <= 0) return -1;
  hipLaunchKernelGGL(attn_queue_reset_kernel, dim3(1), dim3(64), 0, stream, p.queue);
  const dim3 grid(workgroups < p.total ? workgroups : p.total);
  if (d == 128) {
    if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<128, true, true>), grid, dim3(512), 0, stream, p);
    else hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<128, false, true>), grid, dim3(512), 0, stream, p);
  } else if (d == 64) {
    if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<64, true, true>), grid, dim3(512), 0, stream, p);
    else hipLaunchKernelGGL((attn_fwd_bf16_sp_kernel<64, false, true>), grid, dim3(512), 0, stream, p);
  } else {
    return -1;
  }
  return (int)hipGetLastError();
}

const AttnVariant* attn_bf16_sp_variants(int* count) {
  static const AttnVariant table[] = {
      {"bf16 d128 pipelined BM256 BN64", 0, 128, 256, 64, 512, 2 * 3 * 64 * 128 * 2, launch_sp<128>},
      {"bf16 d64 pipelined BM256 BN64", 0, 64, 256, 64, 512, 2 * 3 * 64 * 64 * 2, launch_sp<64>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
