// Fused attention forward, bf16, gfx950: the software-pipelined kernel on 16x16x32 MFMA.
//
// Same operation (paper section 6.1 phases, appendix C.3 state and outputs), the same
// transposed products (S^T = K Q^T, O^T += V^T P^T, a lane holds query columns and the
// exponentiated accumulator IS the next operand), the same K/V streaming and the same
// step pipeline as attn_fwd_bf16_sp.hip.  What differs is the matrix instruction: the
// 16x16x32 bf16 MFMA contracts over 32 instead of 16 per instruction, so every product
// term reads and writes half as many accumulator registers.  Under sustained load this
// chip is power-limited (a loop of nothing but 32x32x16 MFMAs on random data holds
// 1.87 GHz, the same loop of 16x16x32 MFMAs 2.2 GHz at the same utilisation), so the
// cheaper instruction buys clock.
//
// Layout (j = lane % 16, g = lane / 16):
//   * A wave owns 32 queries as two halves qh of 16.  Q operand (B of S^T = K Q^T), half qh,
//     k-step kk: lane holds Q[16 qh + j][32 kk + 8 g .. +7].
//   * K operand (A), key group kg of 16, k-step kk: lane holds K[16 kg + j][32 kk + 8 g .. +7],
//     one 128-bit LDS read, used for both query halves.
//   * S^T accumulator (kg, qh), element r: key 16 kg + 4 g + r, query 16 qh + j.  A lane
//     therefore holds 8 keys of each of its two queries per 32-key block; row sums stay
//     per-lane partial sums until the epilogue.
//   * P^T operand (B of O^T += V^T P^T), half qh: the lane's 8 exponentials of that query,
//     k-slot 8 g + 4 kg + r  <->  key 16 kg + 4 g + r.
//   * V^T operand (A), 16-row group dg of the head dimension: two transposing LDS reads
//     (kg = 0, 1) hand the lane V[16 kg + 4 g + (0..3)][16 dg + j]; used for both query halves.
//   * O^T accumulator (dg, qh), element r: column 16 dg + 4 g + r of query 16 qh + j.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kSumLimit = 65536.0f;  // a lane's 8-term partial sum above this redoes the block with a raised reference

template <int V>
using ic = std::integral_constant<int, V>;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

// V tile swizzle for this kernel's transposing reads: a 16-lane group reads 4 consecutive
// rows x 32 bytes and two groups (8 consecutive rows) are served together, so 8 consecutive
// rows must land in 8 different 32-byte bank groups: XOR the 32-byte index with the row.
template <int ROWB>
__device__ __forceinline__ constexpr int swz_v16(int row) {
  constexpr int NCH = ROWB / 16, RP = 256 / ROWB;
  return ((row / RP) & (NCH / 2 - 1)) << 1;
}

// max / sum over the four lanes j, j+16, j+32, j+48 that share a query column (rare paths only)
__device__ __forceinline__ float max_over_g(float x) {
  x = fmaxf(x, __shfl_xor(x, 16, 64));
  return fmaxf(x, __shfl_xor(x, 32, 64));
}
__device__ __forceinline__ float sum_over_g(float x) {
  x += __shfl_xor(x, 16, 64);
  return x + __shfl_xor(x, 32, 64);
}

// Scheduling-group pipeline of one pipelined step (the builtin wants literal constants, hence
// the recursion): after each MFMA its share of the plain vector work, of the 16 exponentials
// and of the NDS LDS reads.
template <int M, int NM, int NVALU, int NDS>
__device__ __forceinline__ void w16_step_pipeline() {
  if constexpr (M < NM) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr ((NVALU * (M + 1)) / NM - (NVALU * M) / NM > 0)
      __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (M + 1)) / NM - (NVALU * M) / NM, 0);
    if constexpr ((16 * (M + 1)) / NM - (16 * M) / NM > 0)
      __builtin_amdgcn_sched_group_barrier(0x400, (16 * (M + 1)) / NM - (16 * M) / NM, 0);
    if constexpr ((NDS * (M + 1)) / NM - (NDS * M) / NM > 0)
      __builtin_amdgcn_sched_group_barrier(0x100, (NDS * (M + 1)) / NM - (NDS * M) / NM, 0);
    w16_step_pipeline<M + 1, NM, NVALU, NDS>();
  }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 2) attn_fwd_bf16_w16_kernel(const AttnParams p) {
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int NK2 = D / 32;       // MFMA k-steps of S^T = K Q^T
  constexpr int NDG = D / 16;       // 16-row groups of O^T
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
  constexpr int NOP = 2 * NK2 + NDG;    // LDS operands of a step: 2*NK2 of K, NDG of V
#ifndef ATTN_W16_RA
#define ATTN_W16_RA 4
#endif
  constexpr int RA = ATTN_W16_RA;       // operands are read from LDS this many operands ahead
  static_assert(BN * NCH % NT == 0 && NLD >= 1, "tile must divide evenly over the workgroup");
  static_assert(NDG == 2 * NK2 && RA >= 2 && RA <= NOP && RA % 2 == 0, "operand order assumes D/16 = 2 * D/32");
  static_assert((NSLOT - 1) * TILEB + SUBB + 16 * ROWB < 65536 && (NSLOT == 3 || NSLOT == 4), "ring offsets must fit the 16-bit LDS immediate");

  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int j = lane & 15;  // query column within a half / key row within a group / column within a d-group
  const int g = lane >> 4;  // k-slot group of the operands, row group of the accumulators

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
    ld_voff[it] = r * ROWB + ((c ^ swz_v16<ROWB>(r)) << 4);
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
  // bundle b = key tile b+1 (the last tile again if there is none) and value tile b
  auto issue_bundle = [&](int b, int slot) __attribute__((always_inline)) {
    issue_tile(khead, min(b + 1, nt - 1), ld_koff, lds_wave + slot * TILEB);
    issue_tile(vhead, b, ld_voff, lds_wave + VBASE + slot * TILEB);
  };

  issue_tile(khead, 0, ld_koff, lds_wave + (NSLOT - 1) * TILEB);  // key tile 0 borrows the K part of the last slot
  issue_bundle(0, 0);

  // ---- Q operand ---------------------------------------------------------------------------------
  bf16x8 qf[2][NK2];
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    const int row = min(wq0 + 16 * qh + j, N - 1);
    const char* src = qhead + (size_t)row * ROWB + g * 16;
#pragma unroll
    for (int kk = 0; kk < NK2; ++kk) qf[qh][kk] = *(const bf16x8*)(src + kk * 64);
  }
  if (nt > 1) issue_bundle(1, 1);
  if (NSLOT > 3 && nt > 2) issue_bundle(2, 2);

  // ---- LDS read addresses (slot 0, first 32-key block) -----------------------------------------
  uint32_t kaddr[NK2];  // key row j (+16 kg as an immediate: the swizzle has period 16), chunk 4 kk + g
#pragma unroll
  for (int kk = 0; kk < NK2; ++kk) kaddr[kk] = j * ROWB + (((4 * kk + g) ^ attn_swz_k<ROWB>(j)) << 4);
  // V through the transposing load: in a group of 16 lanes, lane s reads the four columns
  // 4*(s%4).. of key row s/4 and the hardware hands lane t the four keys of column t.
  uint32_t vaddr[NDG];  // key row 4 g + s/4 (+16 kg as an immediate), columns 16 dg + 4 (s%4) .. +3
  {
    const int key = 4 * g + (j >> 2);
#pragma unroll
    for (int dg = 0; dg < NDG; ++dg) {
      const int chunk = 2 * dg + ((j & 3) >> 1);
      vaddr[dg] = VBASE + key * ROWB + ((chunk ^ swz_v16<ROWB>(key)) << 4) + ((j & 1) << 3);
    }
  }
  auto k_operand = [&](auto koff, int kg, int kk) __attribute__((always_inline)) {
    return __builtin_bit_cast(u32x4, *(LDS_AS bf16x8*)(smem + kaddr[kk] + koff + kg * 16 * ROWB));
  };
  auto v_operand = [&](auto voff, int dg) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[dg] + voff));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[dg] + voff + 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return __builtin_bit_cast(u32x4, av);
  };
  auto mfma = [&](const u32x4& a, const bf16x8& b, const f32x4& acc) __attribute__((always_inline)) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), b, acc, 0, 0, 0);
  };

  // ---- streaming-softmax state (per query half) ---------------------------------------------------
  f32x4 oacc[NDG][2];
#pragma unroll
  for (int dg = 0; dg < NDG; ++dg)
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) oacc[dg][qh] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_ref[2] = {-INFINITY, -INFINITY};  // reference maxima, scaled log2 units
  float l_run[2] = {0.f, 0.f};              // this lane's share of the row sums
  const float c = p.scale_log2;
  int limit[2];                             // last visible key of each of this lane's two queries
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) limit[qh] = CAUSAL ? min(wq0 + 16 * qh + j, N - 1) : (N - 1);
  const int wlast = wq0 + 31;

  // S^T and packed P^T of two consecutive blocks, indexed [kg][qh] and [qh]
  f32x4 s_a[2][2], s_b[2][2];
  u32x4 p_a[2], p_b[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) p_a[i] = p_b[i] = u32x4{0, 0, 0, 0};

  // P^T = exp2(c S^T - m) of one block against the current references; returns the two partial sums
  auto exp_block = [&](const f32x4 (&s)[2][2], u32x4 (&pk)[2], float (&ls)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      float e[2][4];
#pragma unroll
      for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int r = 0; r < 4; ++r) e[kg][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kg][qh][r], c, -m_ref[qh]));
#pragma unroll
      for (int kg = 0; kg < 2; ++kg) {
        pk[qh][2 * kg] = pack_bf16(e[kg][0], e[kg][1]);
        pk[qh][2 * kg + 1] = pack_bf16(e[kg][2], e[kg][3]);
      }
      ls[qh] = ((e[0][0] + e[0][1]) + (e[0][2] + e[0][3])) + ((e[1][0] + e[1][1]) + (e[1][2] + e[1][3]));
    }
  };
  // slow pass: true block maxima, raise the references, rescale, redo the block
  auto redo_block = [&](const f32x4 (&s)[2][2], u32x4 (&pk)[2], float (&ls)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      float mx = fmaxf(s[0][qh][0], s[1][qh][0]);
#pragma unroll
      for (int r = 1; r < 4; ++r) mx = fmaxf(mx, fmaxf(s[0][qh][r], s[1][qh][r]));
      mx = max_over_g(mx) * c;
      const float m_new = fmaxf(m_ref[qh], mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref[qh] - m_new);  // exp2(-inf) = 0 on the first block
      m_ref[qh] = m_new;
      l_run[qh] *= alpha;
#pragma unroll
      for (int dg = 0; dg < NDG; ++dg) oacc[dg][qh] *= alpha;
    }
    exp_block(s, pk, ls);
  };
  auto finish_block = [&](const f32x4 (&s)[2][2], u32x4 (&pk)[2], float (&ls)[2]) __attribute__((always_inline)) {
    if (__builtin_amdgcn_ballot_w64(!(ls[0] <= kSumLimit) || !(ls[1] <= kSumLimit)) != 0) redo_block(s, pk, ls);
    l_run[0] += ls[0];
    l_run[1] += ls[1];
  };

  // ---- boundary-case building blocks (compiler-scheduled, not overlapped) ----------------------
  auto qk_block = [&](f32x4 (&s)[2][2], auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) s[kg][qh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < NK2; ++kk)
#pragma unroll
      for (int kg = 0; kg < 2; ++kg) {
        const u32x4 a = k_operand(koff, kg, kk);
        s[kg][0] = mfma(a, qf[0][kk], s[kg][0]);
        s[kg][1] = mfma(a, qf[1][kk], s[kg][1]);
      }
  };
  auto pv_block = [&](const u32x4 (&pk)[2], auto voff) __attribute__((always_inline)) {
#pragma unroll
    for (int dg = 0; dg < NDG; ++dg) {
      const u32x4 a = v_operand(voff, dg);
      oacc[dg][0] = mfma(a, __builtin_bit_cast(bf16x8, pk[0]), oacc[dg][0]);
      oacc[dg][1] = mfma(a, __builtin_bit_cast(bf16x8, pk[1]), oacc[dg][1]);
    }
  };
  auto softmax_block = [&](f32x4 (&s)[2][2], u32x4 (&pk)[2], int key0, bool need_mask) __attribute__((always_inline)) {
    if (need_mask) {
#pragma unroll
      for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (key0 + 16 * kg + 4 * g + r > limit[qh]) s[kg][qh][r] = -INFINITY;
    }
    float ls[2];
    exp_block(s, pk, ls);
    finish_block(s, pk, ls);
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
  // LDS operands in the order they are consumed: t even -> K operand (kk, kg) = (t/4, (t/2)%2),
  // t odd -> V operand dg = t/2; each serves two MFMAs (the two query halves):
  //   MFMA 4u: S(kg, 0)  4u+1: O(dg, 0)  4u+2: S(kg, 1)  4u+3: O(dg, 1)     with K operand 2u, V operand 2u+1
  // so consecutive MFMAs never share an accumulator.  Operands are read RA operands ahead; the
  // first RA of a step are requested by the previous step (offnext = where the next step reads).
  // Source order inside the step does not matter: the scheduling-group pipeline at its end tells
  // the scheduler how to interleave MFMAs, vector work, exponentials and LDS reads.
  u32x4 pre[RA];
  auto step_operand = [&](auto off, int t) __attribute__((always_inline)) {
    const int u = t >> 1;
    return (t & 1) ? v_operand(off, u) : k_operand(off, u % 2, u / 2);
  };
  auto step_hot = [&](f32x4 (&s_in)[2][2], f32x4 (&s_out)[2][2], u32x4 (&p_out)[2], u32x4 (&p_pv)[2], auto off, auto offnext)
      __attribute__((always_inline)) {
    u32x4 op[NOP];
#pragma unroll
    for (int t = 0; t < RA; ++t) op[t] = pre[t];
#pragma unroll
    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) s_out[kg][qh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < NDG; ++u) {
      const int kg = u % 2, kk = u / 2;
      s_out[kg][0] = mfma(op[2 * u], qf[0][kk], s_out[kg][0]);
      oacc[u][0] = mfma(op[2 * u + 1], __builtin_bit_cast(bf16x8, p_pv[0]), oacc[u][0]);
      s_out[kg][1] = mfma(op[2 * u], qf[1][kk], s_out[kg][1]);
      oacc[u][1] = mfma(op[2 * u + 1], __builtin_bit_cast(bf16x8, p_pv[1]), oacc[u][1]);
#pragma unroll
      for (int t = 2 * u + RA; t < 2 * u + RA + 2; ++t) {
        if (t < NOP) op[t] = step_operand(off, t);
        else pre[t - NOP] = step_operand(offnext, t - NOP);
      }
    }
    float ls[2];
    exp_block(s_in, p_out, ls);
    // the packs belong to this step: keep the compiler from sinking them past the branch below
#pragma unroll
    for (int qh = 0; qh < 2; ++qh)
#pragma unroll
      for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(p_out[qh][i]));
    // vector work of a block: 16 multiply-adds, 14 adds, 8 packs, compare
    w16_step_pipeline<0, 4 * NDG, 16 + 14 + 8 + 2, NK2 * 2 + NDG * 2>();
    finish_block(s_in, p_out, ls);
  };

  // the same step for blocks that may be masked or not visible to this wave (run-time offsets):
  // O += V P of the previous block first (still relative to the old references), then the
  // softmax of this block (which may rescale O), then the scores of the next block
  auto step_any = [&](bool do_sm, int key0, bool do_mm, f32x4 (&s_in)[2][2], f32x4 (&s_out)[2][2], u32x4 (&p_out)[2], u32x4 (&p_pv)[2],
                      int koff, int voff) __attribute__((always_inline)) {
    if (do_mm) pv_block(p_pv, voff);
    if (do_sm) softmax_block(s_in, p_out, key0, needs_mask(key0));
    if (do_mm) qk_block(s_out, koff);
  };

  // ---- prologue: block 0 ---------------------------------------------------------------------------
  // key tile 0 (and Q) have landed once only the bundle loads issued after them are outstanding
  if (NSLOT > 3 && nt > 2) ATTN_WAIT_VMCNT(6 * NLD);
  else if (nt > 1) ATTN_WAIT_VMCNT(4 * NLD);
  else ATTN_WAIT_VMCNT(2 * NLD);
#pragma unroll
  for (int qh = 0; qh < 2; ++qh)
#pragma unroll
    for (int kk = 0; kk < NK2; ++kk) asm volatile("" ::"v"(qf[qh][kk]));  // Q is in registers from here on
  attn_wg_barrier();
  if (wave_valid) {
    qk_block(s_b, (NSLOT - 1) * TILEB);                   // S(0)
    softmax_block(s_b, p_b, 0, needs_mask(0));  // P(0) -> p_b
    qk_block(s_a, (NSLOT - 1) * TILEB + SUBB);            // S(1); ignored if block 1 is not visible
  }
  if (NSLOT > 3 && nt > 2) ATTN_WAIT_VMCNT(4 * NLD);
  else if (nt > 1) ATTN_WAIT_VMCNT(2 * NLD);
  else ATTN_WAIT_VMCNT(0);
  attn_wg_barrier();  // bundle 0 is full; the K part of the last slot is empty again
#pragma unroll
  for (int t = 0; t < RA; ++t) pre[t] = step_operand(ic<0>{}, t);  // first operands of the first pipelined step

  // ---- main loop over bundles ------------------------------------------------------------------------
  // iteration b: exponentiate blocks 2b+1 and 2b+2, compute the scores of blocks 2b+2 and 2b+3
  // (key tile b+1), accumulate blocks 2b and 2b+1 (value tile b).  Between the two steps of
  // iteration b, bundle b+1 (requested one iteration ago, the only loads in flight) is published,
  // and the slot of bundle b-1, which every wave has finished reading, is handed to bundle b+2.
  auto bundle_mid = [&](int b, int free_slot) __attribute__((always_inline)) {
    if (NSLOT > 3 && b + 2 < nt) ATTN_WAIT_VMCNT(2 * NLD);  // bundle b+2 may stay in flight
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
    if (b + NSLOT - 1 < nt) issue_bundle(b + NSLOT - 1, free_slot);
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
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    const int qrow = wq0 + 16 * qh + j;
    const float l = sum_over_g(l_run[qh]);
    const float inv = p.out_scale / l;
    if (qrow < N && g == 0) lsehead[qrow] = (m_ref[qh] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    // the lane holds columns 16 dg + 4 g + (0..3): one 8-byte store per column group
    if (qrow < N) {
#pragma unroll
      for (int dg = 0; dg < NDG; ++dg) {
        u32x2 out = {pack_bf16(oacc[dg][qh][0] * inv, oacc[dg][qh][1] * inv), pack_bf16(oacc[dg][qh][2] * inv, oacc[dg][qh][3] * inv)};
        *(u32x2*)(ohead + (size_t)qrow * ROWB + (16 * dg + 4 * g) * 2) = out;
      }
    }
  }
}

template <int D>
int launch_w16(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_bf16_w16_kernel<D, true>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_bf16_w16_kernel<D, false>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_bf16_w16_variants(int* count) {
  static const AttnVariant table[] = {
      {"bf16 d128 pipelined 16x16x32 BM256 BN64", 0, 128, 256, 64, 512, 2 * 3 * 64 * 128 * 2, launch_w16<128>},
      {"bf16 d64 pipelined 16x16x32 BM256 BN64", 0, 64, 256, 64, 512, 2 * 3 * 64 * 64 * 2, launch_w16<64>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
