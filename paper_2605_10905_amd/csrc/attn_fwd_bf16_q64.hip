// Attention forward, bf16, head dimension 128, gfx950: 64 queries per wave, one wave per SIMD.
//
// Same operation and the same formulation as the pipelined kernel (section 6.1 phase list;
// appendix C.3 outputs): transposed products S^T = K Q^T and O^T += V^T P^T on the 32x32x16 MFMA,
// one query per lane, streaming softmax against a reference maximum that is only raised when a
// partial row sum overflows a limit.  What differs is the shape of a wave: it owns two 32-query
// blocks, so every K or V fragment read from LDS feeds two MFMAs (0.5 KB of LDS reads per MFMA
// instead of 1 KB, and the LDS's 128 bytes per cycle are what caps the matrix pipe of the
// one-block-per-wave kernel).  Two blocks' accumulators (128 registers) and Q operands (64) need
// the whole 512-register file: four waves per workgroup, one per SIMD, so nothing but the wave
// itself can hide its vector work.  A step therefore works on three 32-key blocks at once (scores
// of block i+1, exponentials of block i, P V of block i-1: no MFMA of a step depends on its vector
// work) and its instruction order is fixed by hand, one MFMA per slot, fenced slot by slot:
//   * 16 operands per step, each used by the two query blocks in turn: four V fragments first (the
//     previous step requested them from a tile that is certainly resident), then groups of two K
//     fragments and one V fragment, so that the score products end three operands before the step;
//   * operands are requested two pairs ahead, newest first inside a pair, so that one wait serves
//     four MFMAs;
//   * one of the 32 exponentials (with its multiply-add, add and half a pack) per slot from slot 2;
//   * the second step of a tile also carries the 8 direct-to-LDS loads of the tile three ahead, one
//     per slot.
// The score products are written as inline assembly with vector-register results (the compiler
// would accumulate them in the other half of the register file and copy all 32 values out at the
// top of the next step with the matrix pipe idle); the build checks the generated assembly for the
// wait states the compiler cannot know about.
// K/V tiles of 64 keys travel into a ring of four slots, two tiles ahead, one workgroup barrier per
// tile; the loop is unrolled over the ring so that every LDS offset is an instruction immediate.
// Every wave computes every block of the workgroup's key range: blocks beyond a wave's causal
// limit or past N are masked to -inf and add exact zeros (the workgroup's last wave needs them
// anyway).
// Measured against the pipelined kernel on the headline shape: the same time within 1-4 % (matrix
// pipe 60 % busy at 1.94 GHz against 67 % at 1.77 GHz).  It is kept as a variant, not the default.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

constexpr float kSumLimit = 65536.0f;  // a lane's 16-term partial sum above this redoes the block with a raised reference

template <int V>
using ic = std::integral_constant<int, V>;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

struct Q64 {
  static constexpr int D = 128, BN = 64, NWAVES = 4, BM = NWAVES * 64, NT = NWAVES * 64;
  static constexpr int NKK = D / 16, NCB = D / 32, ROWB = D * 2, NCH = ROWB / 16;
  static constexpr int TILEB = BN * ROWB, SUBB = 32 * ROWB, NSLOT = 4;
  static constexpr int VBASE = NSLOT * TILEB;       // K parts of the slots first, then the V parts
  static constexpr int LDS_BYTES = 2 * NSLOT * TILEB;
  static constexpr int NLD = BN * NCH / NT;          // direct-to-LDS loads per thread and tensor tile: 4
  static constexpr int NOP = 16, LEAD = 4;                     // operands per step; V operands the previous step requests
  // operand position p of a step: V fragments 0..LEAD-1, then groups (K, K, V): the score products
  // end three operands before the step does, so their results are long finished when the next
  // step's vector work reads them
  static constexpr bool is_k(int p) { return p >= LEAD && (p - LEAD) % 3 != 2; }
  static constexpr int index(int p) {
    if (p < LEAD) return p;
    const int q = p - LEAD;
    return q % 3 == 2 ? LEAD + q / 3 : 2 * (q / 3) + q % 3;
  }
  // position p requests operand target(p): two pairs ahead, the pair's second operand first
  static constexpr int target(int p) { return (p / 2 + 2) * 2 + 1 - p % 2; }
  static constexpr int DM0 = 2;                                          // first MFMA slot that requests a tile load
  static constexpr int VP0 = 2;                                          // first MFMA slot with vector work
  static constexpr int vslot(int e) { return VP0 + (e * (2 * NOP - VP0)) / 32; }  // slot of element e = 16 qb + r
};

template <bool CAUSAL>
__global__ void __launch_bounds__(256, 1) attn_fwd_bf16_q64_kernel(const AttnParams p) {
  using C = Q64;
  constexpr int NKK = C::NKK, NCB = C::NCB, ROWB = C::ROWB, NCH = C::NCH, TILEB = C::TILEB, SUBB = C::SUBB, NSLOT = C::NSLOT;
  constexpr int NLD = C::NLD, NT = C::NT, BN = C::BN, BM = C::BM, VBASE = C::VBASE, NOP = C::NOP, LEAD = C::LEAD;

  __shared__ __attribute__((aligned(1024))) char smem_raw[C::LDS_BYTES];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31, h = lane >> 5;

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int hk = tc.hq / (p.Hq / p.Hkv);
  const int q0 = tc.t * BM;
  const int wq0 = q0 + w * 64;  // first query row of this wave

  const char* const qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;  // keys the workgroup visits
  const int nt = (kv_end + BN - 1) / BN;            // 64-key tiles

  // ---- producer role: direct-to-LDS tile loads --------------------------------------------------
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
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_tile = [&](int t, int slot) __attribute__((always_inline)) {
    const char* const kb = khead + (size_t)t * TILEB;
    const char* const vb = vhead + (size_t)t * TILEB;
    if ((t + 1) * BN <= N) {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        attn_lds_dma16(kb, ld_koff[it], lds_wave + slot * TILEB + it * NT * 16);
        attn_lds_dma16(vb, ld_voff[it], lds_wave + VBASE + slot * TILEB + it * NT * 16);
      }
    } else {
      // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const uint32_t over = (uint32_t)max(0, t * BN + ld_row[it] - (N - 1)) * ROWB;
        attn_lds_dma16(kb, ld_koff[it] - over, lds_wave + slot * TILEB + it * NT * 16);
        attn_lds_dma16(vb, ld_voff[it] - over, lds_wave + VBASE + slot * TILEB + it * NT * 16);
      }
    }
  };
  constexpr int LPT = 2 * NLD;  // loads per thread and tile
  issue_tile(0, 0);

  // ---- Q operands (B operands of S^T = K Q^T): lane (qi,h) of block qb holds Q[row][16kk+8h .. +7]
  bf16x8 qf[2][NKK];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int row = min(wq0 + qb * 32 + qi, N - 1);
    const char* src = qhead + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[qb][kk] = *(const bf16x8*)(src + kk * 32);
  }
  issue_tile(min(1, nt - 1), 1);
  issue_tile(min(2, nt - 1), 2);

  // ---- LDS read addresses; slot and block offsets are immediates --------------------------------
  uint32_t kaddr[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = qi * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(qi)) << 4);
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
  auto k_operand = [&](int off, int kk) __attribute__((always_inline)) { return *(LDS_AS u32x4*)(smem + kaddr[kk] + off); };
  // V fragment i of a block: 32-row block cb = i % 4 of O^T, keys 16 kc .. 16 kc + 15 with kc = i / 4
  auto v_operand = [&](int off, int i) __attribute__((always_inline)) {
    const int cb = i & 3, kc = i >> 2;
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + off + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + off + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return __builtin_bit_cast(u32x4, av);
  };

  // ---- streaming-softmax state, per query block -------------------------------------------------
  f32x16 oacc[2][NCB];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qb][cb][r] = 0.f;
  float m_ref[2] = {-INFINITY, -INFINITY};  // reference maximum, scaled log2 units
  float l_run[2] = {0.f, 0.f};              // this lane's share of the row sum (halves are added at the end)
  const float c = p.scale_log2;
  int limit[2];                             // last visible key of this lane's query
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) limit[qb] = CAUSAL ? min(wq0 + qb * 32 + qi, N - 1) : (N - 1);

  auto pv_mfma = [&](int i, u32x4 o, const u32x4 (&pk)[2][2]) __attribute__((always_inline)) {
    const int cb = i & 3, kc = i >> 2;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
      oacc[qb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o), __builtin_bit_cast(bf16x8, pk[qb][kc]), oacc[qb][cb], 0, 0, 0);
  };
  auto exp_element = [&](float s, int qb) __attribute__((always_inline)) { return __builtin_amdgcn_exp2f(__builtin_fmaf(s, c, -m_ref[qb])); };

  u32x4 pre[LEAD];  // the next step's first V operands
  // One step.  s_in: finished scores of the block whose first key is key0 (V part at CUR);
  // s_out <- scores of the next block (K part at NEXT); p_out <- P of this block; p_acc: P of the
  // previous block (V part at PREV), multiplied into O.  PREV, CUR, NEXT are compile-time offsets.
  // DMA >= 0: the step also requests key/value tile dma_t into ring slot DMA, one load per slot
  auto step = [&](f32x16 (&s_in)[2], f32x16 (&s_out)[2], u32x4 (&p_out)[2][2], const u32x4 (&p_acc)[2][2], auto PREV, auto CUR, auto NEXT,
                  int key0, auto DMA, int dma_t) __attribute__((always_inline)) {
    constexpr int prev = decltype(PREV)::value, cur = decltype(CUR)::value, next = decltype(NEXT)::value, dma = decltype(DMA)::value;
    const char* const dma_k = khead + (size_t)dma_t * TILEB;
    const char* const dma_v = vhead + (size_t)dma_t * TILEB;
    uint32_t dma_over = 0;
    u32x4 op[NOP];
#pragma unroll
    for (int i = 0; i < LEAD; ++i) op[i] = pre[i];
    float mneg[2] = {-m_ref[0], -m_ref[1]};
    float ls[2] = {0.f, 0.f}, e_even = 0.f, e_last = 0.f;  // e_last: the previous slot's exponential, added one slot late
    const bool need_mask = (CAUSAL && key0 + 31 > wq0) || key0 + 31 >= N;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < 2 * NOP; ++m) {
      const int pos = m >> 1, qb = m & 1;
      if (qb == 0) {  // LDS requests, once per operand position
        const int t = C::target(pos);
        if (t < NOP) op[t] = C::is_k(t) ? k_operand(next, C::index(t)) : v_operand(prev, C::index(t));
        else pre[t - NOP] = v_operand(cur, t - NOP);
      }
      if (dma >= 0 && m >= C::DM0 && m < C::DM0 + 2 * NLD) {
        const int it = (m - C::DM0) >> 1;
        if (((m - C::DM0) & 1) == 0) {
          dma_over = (uint32_t)max(0, dma_t * BN + ld_row[it] - (N - 1)) * ROWB;  // rows past N-1 re-read row N-1
          attn_lds_dma16(dma_k, ld_koff[it] - dma_over, lds_wave + dma * TILEB + it * NT * 16);
        } else {
          attn_lds_dma16(dma_v, ld_voff[it] - dma_over, lds_wave + VBASE + dma * TILEB + it * NT * 16);
        }
      }
      const int i = C::index(pos);
      if (C::is_k(pos)) {
        // written as assembly so that the scores land in the vector registers the exponentials read
        // (the compiler would accumulate them in the other half of the register file and copy all
        // 32 values out at the top of the next step, with the matrix pipe idle meanwhile)
        // (Q, never read by a vector instruction, lives in the accumulation half of the register file)
        // The compiler does not know these are MFMAs and inserts no wait states behind them.  Inside
        // the chain nothing but the next link touches the result; the last links of both query
        // blocks go out as one statement followed by the 11 wait states a vector instruction needs
        // behind an 8-pass MFMA, so that whatever the compiler puts next (it may move the finished
        // scores) is safe.
        if (i == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s_out[qb]) : "v"(op[pos]), "a"(qf[qb][0]));
        else if (i == NKK - 1 && qb == 0) ;
        else if (i == NKK - 1)
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %3, %0\n\tv_mfma_f32_32x32x16_bf16 %1, %2, %4, %1\n\ts_nop 10"
                       : "+v"(s_out[0]), "+v"(s_out[1])
                       : "v"(op[pos]), "a"(qf[0][NKK - 1]), "a"(qf[1][NKK - 1]));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s_out[qb]) : "v"(op[pos]), "a"(qf[qb][i]));
      } else {
        const int cb = i & 3, kc = i >> 2;
        oacc[qb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[pos]), __builtin_bit_cast(bf16x8, p_acc[qb][kc]), oacc[qb][cb], 0, 0, 0);
      }
      // invisible keys (causal diagonal and beyond, ragged tail): -inf scores behind a wave-uniform branch
      if (m == C::VP0 - 1 && need_mask) {
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (key0 + 4 * h + 8 * (r >> 2) + (r & 3) > limit[b2]) s_in[b2][r] = -INFINITY;
      }
      // vector work of this slot: one exponential, its share of the row sum, half a pack
#pragma unroll
      for (int e = 0; e < 32; ++e)
        if (C::vslot(e) == m) {
          const int b2 = e >> 4, r = e & 15;
          // (the add and the pack of an exponential wait one slot: the result of a transcendental
          // instruction cannot be read by the instruction right behind it)
          if (e > 0) ls[(e - 1) >> 4] += e_last;
          if (e > 0 && ((e - 1) & 1)) {
            const int pb = (e - 1) >> 4, pr = (e - 1) & 15;
            p_out[pb][pr >> 3][(pr >> 1) & 3] = pack_bf16(e_even, e_last);
            asm volatile("" ::"v"(p_out[pb][pr >> 3][(pr >> 1) & 3]));  // not later than this slot
          }
          if (e > 0 && !((e - 1) & 1)) e_even = e_last;
          // (an empty statement that defines the reference operand here keeps the exponential from
          // starting before this slot)
          asm volatile("" : "+v"(mneg[b2]));
          e_last = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[b2][r], c, mneg[b2]));
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    ls[1] += e_last;
    p_out[1][1][3] = pack_bf16(e_even, e_last);
    // a partial sum that is large or not a number (always on the very first block, whose reference
    // is -inf): take the true block maximum, raise the reference, rescale, and redo the block
    if (__builtin_amdgcn_ballot_w64(!(ls[0] <= kSumLimit) || !(ls[1] <= kSumLimit)) != 0) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = fmaxf(s_in[qb][0], s_in[qb][1]);
#pragma unroll
        for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s_in[qb][r]);
        mx = attn_max_halves(mx) * c;
        const float m_new = fmaxf(m_ref[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f(m_ref[qb] - m_new);  // exp2(-inf) = 0 on the first block
        m_ref[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) oacc[qb][cb] *= alpha;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float e0 = exp_element(s_in[qb][2 * u], qb), e1 = exp_element(s_in[qb][2 * u + 1], qb);
          p_out[qb][u >> 2][u & 3] = pack_bf16(e0, e1);
          s0 += e0;
          s1 += e1;
        }
        ls[qb] = s0 + s1;
      }
    }
    l_run[0] += ls[0];
    l_run[1] += ls[1];
  };

  // the block "before the first" lives in the V part of the last half of slot 3: zeros, so that its
  // P V products (with P = 0) add exact zeros
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < SUBB / (NT * 16); ++i) *(LDS_AS u32x4*)(smem + VBASE + 3 * TILEB + SUBB + (i * NT + tid) * 16) = z;
  }
  ATTN_WAIT_VMCNT(2 * LPT);
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+a"(qf[qb][kk]));  // Q is in registers from here on
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the zero fill is written
  attn_wg_barrier();

  // ---- prologue: scores of block 0 ---------------------------------------------------------------
  f32x16 s_a[2], s_b[2];
  u32x4 p_a[2][2], p_b[2][2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s_a[qb][r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t) p_b[qb][t] = u32x4{0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    const u32x4 o = k_operand(0, kk);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) s_a[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o), qf[qb][kk], s_a[qb], 0, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < LEAD; ++i) pre[i] = v_operand(3 * TILEB + SUBB, i);

  // ---- main loop: tile j lives in slot j % 4 = S --------------------------------------------------
  auto tile = [&](auto S, int j) __attribute__((always_inline)) {
    constexpr int s = decltype(S)::value;
    constexpr int b0 = s * TILEB, b1 = b0 + SUBB, bp = ((s + 3) & 3) * TILEB + SUBB, bn = ((s + 1) & 3) * TILEB;
    step(s_a, s_b, p_a, p_b, ic<bp>{}, ic<b0>{}, ic<b1>{}, j * BN, ic<-1>{}, 0);
    // tile j+1 has landed (the loads of tile j+2 stay in flight); every wave is done with tile j-1,
    // whose slot the second step refills with tile j+3 (past the end: the last tile once more, so
    // that the count of loads in flight stays the same; nobody reads that slot again)
    ATTN_WAIT_VMCNT(LPT);
    attn_wg_barrier();
    step(s_b, s_a, p_b, p_a, ic<b0>{}, ic<b1>{}, ic<bn>{}, j * BN + 32, ic<(s + 3) & 3>{}, min(j + 3, nt - 1));
  };
  int j = 0;
  for (; j + 4 <= nt; j += 4) {
    tile(ic<0>{}, j);
    tile(ic<1>{}, j + 1);
    tile(ic<2>{}, j + 2);
    tile(ic<3>{}, j + 3);
  }
  if (j < nt) {
    tile(ic<0>{}, j);
    if (j + 1 < nt) {
      tile(ic<1>{}, j + 1);
      if (j + 2 < nt) tile(ic<2>{}, j + 2);
    }
  }
  ATTN_WAIT_VMCNT(0);  // no load may still be writing LDS when the workgroup ends
  // the P V products of the last block (its first operands are already here)
  {
    const int last = ((nt - 1) & 3) * TILEB + SUBB;
#pragma unroll
    for (int i = LEAD; i < 2 * NCB; ++i) pv_mfma(i, v_operand(last, i), p_b);
#pragma unroll
    for (int i = 0; i < LEAD; ++i) pv_mfma(i, pre[i], p_b);
  }

  // ---- epilogue: O = acc / l (bf16), lse = (m + log2 l) * ln 2 --------------------------------------
  char* const ohead = (char*)p.o + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  float* const lsehead = p.lse + (size_t)(tc.b * p.Hq + tc.hq) * N;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int qrow = wq0 + qb * 32 + qi;
    const float l = attn_sum_halves(l_run[qb]);
    const float inv = p.out_scale / l;
    if (qrow < N && h == 0) lsehead[qrow] = (m_ref[qb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    // lane (qi,h) holds O^T rows 32cb + 8b + 4h + r.  Exchange with the other half so that every
    // lane owns 8 consecutive output columns 32cb + 16a + 8h + (0..7): one 16-byte store each.
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        uint32_t x[2], y[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const uint32_t tx = pack_bf16(oacc[qb][cb][(2 * a) * 4 + 2 * r] * inv, oacc[qb][cb][(2 * a) * 4 + 2 * r + 1] * inv);
          const uint32_t ty = pack_bf16(oacc[qb][cb][(2 * a + 1) * 4 + 2 * r] * inv, oacc[qb][cb][(2 * a + 1) * 4 + 2 * r + 1] * inv);
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

int launch_q64(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_q64_kernel<true>), dim3(grid), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_bf16_q64_kernel<false>), dim3(grid), dim3(256), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_bf16_q64_variants(int* count) {
  static const AttnVariant table[] = {
      {"bf16 d128 64 queries per wave BM256 BN64", 0, 128, 256, 64, 256, 2 * 4 * 64 * 128 * 2, launch_q64},
  };
  *count = 1;
  return table;
}
