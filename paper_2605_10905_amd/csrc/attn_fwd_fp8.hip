// Fused attention forward, fp8 (OCP e4m3) inputs, fp32 accumulate, bf16 output, gfx950.
//
// Same operation as the bf16 kernels (paper section 6.1 phases, appendix C.3 outputs) on
// per-tensor-scaled e4m3 Q, K, V; the probabilities are re-quantised to e4m3 before the
// second product.  Both products run on the 32x32x64 f8f6f4 MFMA (16 passes, twice the bf16
// rate), again transposed (S^T = K Q^T, O^T += V^T P^T) so that a lane holds one query.
//
//  * q_descale * k_descale is folded into the exponent constant, v_descale into the final
//    normalisation: no extra pass over memory.
//  * P is stored as e4m3 of 2^6 * exp2(c s - m).  The exponentials of a tile are taken against
//    the current reference maximum without looking at the tile's own maximum; the tile is redone
//    with a raised reference only if a lane's partial row sum exceeds 448 (the e4m3 conversion
//    does not saturate: it returns NaN above 464; a sum of non-negative terms below 448 bounds
//    every term).  Values down to 2^-12 keep a normal encoding.  The factor 2^6 cancels in
//    O = acc / l.
//  * P enters the second product as the SUM OF TWO e4m3 TERMS: the e4m3 rounding of P and the
//    e4m3 rounding of what that rounding lost (converted back with v_cvt_pk_f32_fp8 and
//    subtracted in fp32).  One term alone carries 3 mantissa bits, a relative error of 2.6 %
//    rms per weight, and measured 2.0 - 2.6 % relative Frobenius error on O, above the 2 %
//    bound; two terms bring it to the level of the bf16 path.  The second term doubles the PV
//    MFMAs (which have slack here) and adds two VALU operations per score.
//  * The row sum l is taken in fp32 from the unrounded exponentials (lse to 1e-3) and also
//    normalises O: the two-term weights sum to l within 2^-8.
//  * V^T operands come from the 8-bit transposing LDS load (ds_read_b64_tr_b8): a lane reads
//    8 bytes of one key row and receives 8 keys of one column.
//
// Orchestration: all 8 waves symmetric, one workgroup barrier per 64-key tile, three-slot
// LDS ring fed by direct-to-LDS loads two tiles ahead.  The path is bound by the softmax
// VALU work (the matrix pipe needs half the time it needs in bf16), so the MFMA phases are
// left to the compiler's scheduler.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) int i32x2;

constexpr float kSumLimit = 448.0f;  // largest finite e4m3 value: a 32-term partial sum below it bounds every term
constexpr float kPShift = 6.0f;  // P is stored as 2^6 * exp2(.)

// 16-byte-chunk swizzle of the V tile for the 8-bit transposing load.  A 16-lane group reads
// 16 bytes of each of the rows r .. r+3 and r+8 .. r+11 (r a multiple of 4) and two groups
// that read neighbouring chunks of the same rows are served together.  With 128-byte rows two
// consecutive rows already sit in different halves of the 64 banks; bits 1 and 3 of the row
// move the chunk PAIR, so the four rows of a bank half and the two chunks of a pair cover all
// eight 16-byte groups of that half.
__device__ __forceinline__ constexpr int swz_v8(int row) { return (((row >> 1) & 1) | (((row >> 3) & 1) << 1)) << 1; }

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 2) attn_fwd_fp8_kernel(const AttnParams p) {
  static_assert(D == 128, "fp8 path is built for head dimension 128");
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int ROWB = D;           // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row (8)
  constexpr int NKK = D / 64;       // MFMA k-steps of S^T = K Q^T (2)
  constexpr int NCB = D / 32;       // 32-row blocks of O^T (4)
  constexpr int TILEB = BN * ROWB;  // 8 KB
  constexpr int NSLOT = 3;
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

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;
  const int nt = (kv_end + BN - 1) / BN;

  // ---- producer role: one direct-to-LDS 16-byte load per thread per tile and tensor --------
  const int ld_row = tid / NCH, ld_c = tid % NCH;
  const uint32_t ld_koff = ld_row * ROWB + ((ld_c ^ attn_swz_k<ROWB>(ld_row)) << 4);
  const uint32_t ld_voff = ld_row * ROWB + ((ld_c ^ swz_v8(ld_row)) << 4);
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_tile_loads = [&](int j, int slot) __attribute__((always_inline)) {
    const uint32_t over = (uint32_t)max(0, j * BN + ld_row - (N - 1)) * ROWB;  // rows past N-1 re-read row N-1
    attn_lds_dma16(khead + (size_t)j * TILEB, ld_koff - over, lds_wave + slot * TILEB);
    attn_lds_dma16(vhead + (size_t)j * TILEB, ld_voff - over, lds_wave + VBASE + slot * TILEB);
  };
  issue_tile_loads(0, 0);

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
  if (nt > 1) issue_tile_loads(1, 1);

  // ---- LDS read addresses (slot 0) ------------------------------------------------------------
  // K operand: lane (qi,h) reads key row qi, bytes 64kk + 32h .. +31 = chunks 4kk + 2h, +1
  uint32_t kaddr[NKK][2];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
    for (int e = 0; e < 2; ++e) kaddr[kk][e] = qi * ROWB + (((4 * kk + 2 * h + e) ^ attn_swz_k<ROWB>(qi)) << 4);
  // V operand through the 8-bit transposing load.  In a group of 16 lanes, lane s reads the 8
  // columns 8*(s%2).. of "row" s/2 and the hardware hands lane t the 8 rows of column t.  The
  // k-slots of the PV product follow the S^T accumulator layout: dword wd of the operand holds
  // keys 32*(wd/4) + 8*(wd%4) + 4h + (0..3), so read pr (dwords 2pr, 2pr+1) takes rows
  // base + 4h + (0..3) and base + 8 + 4h + (0..3) with base = 32*(pr/2) + 16*(pr%2).
  uint32_t vaddr[NCB][4];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
    const int e = s >> 1;  // row slot 0..7 of the read
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const int key = 32 * (pr >> 1) + 16 * (pr & 1) + 8 * (e >> 2) + 4 * h + (e & 3);
        const int chunk = cb * 2 + chalf;
        vaddr[cb][pr] = VBASE + key * ROWB + ((chunk ^ swz_v8(key)) << 4) + ((s & 1) << 3);
      }
  }

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

  if (nt > 1) ATTN_WAIT_VMCNT(2);
  else ATTN_WAIT_VMCNT(0);
  // Q is in registers from here on (touched one dword at a time: a 256-bit asm operand has no
  // host-side equivalent and silently drops the kernel's launch stub)
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(qf[kk][i]));
  __syncthreads();

  auto consume_tile = [&](int j, int slot, bool masked) __attribute__((always_inline)) {
    const int sb = slot * TILEB;
    // S^T = K Q^T for the two 32-key blocks of the tile
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const u32x4 lo = *(LDS_AS u32x4*)(smem + kaddr[kk][0] + sb + kb * 32 * ROWB);
        const u32x4 hi = *(LDS_AS u32x4*)(smem + kaddr[kk][1] + sb + kb * 32 * ROWB);
        const i32x8 a = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        s[kb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, qf[kk], s[kb], 0, 0, 0, unit_scale, 0, unit_scale);
      }
    }
    if (masked) {
      const int kbase = j * BN + 4 * h;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kbase + kb * 32 + 8 * (r >> 2) + (r & 3) > limit) s[kb][r] = -INFINITY;
    }
    // P^T = 2^6 exp2(c S^T - m) as two e4m3 terms, packed four keys to a dword in accumulator
    // order.  Optimistic pass against the current reference maximum; if a lane's partial row
    // sum exceeds the largest e4m3 value (only then could a term leave the e4m3 range) or is
    // not a number (first tile), the true tile maximum is taken, the reference raised, the
    // accumulator rescaled and the tile redone.
    i32x8 phi, plo;
    auto exp_tile = [&]() __attribute__((always_inline)) {
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
          ls0 += e0 + e2;
          ls1 += e1 + e3;
        }
      return ls0 + ls1;
    };
    float ls = exp_tile();
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) {
      float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
      mx = attn_max_halves(mx) * c;
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
      ls = exp_tile();
    }
    l_run += ls;
    // O^T += V^T (P_hi + P_lo)^T
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      i32x8 a;
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const i32x2 t = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(smem + vaddr[cb][pr] + sb));
        a[2 * pr] = t[0];
        a[2 * pr + 1] = t[1];
      }
      oacc[cb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, phi, oacc[cb], 0, 0, 0, unit_scale, 0, unit_scale);
      oacc[cb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, plo, oacc[cb], 0, 0, 0, unit_scale, 0, unit_scale);
    }
  };

  int slot = 0;
  for (int j = 0; j < nt; ++j) {
    const int pslot = slot == 0 ? NSLOT - 1 : slot - 1;  // slot of tile j+2 = slot of tile j-1
    if (j + 2 < nt) issue_tile_loads(j + 2, pslot);
    const int key_lo = j * BN, key_hi = key_lo + BN - 1;
    const bool skip = !wave_valid || (CAUSAL && key_lo > wq0 + 31);
    if (!skip) {
      if ((CAUSAL && key_hi > wq0) || key_hi >= N) consume_tile(j, slot, true);
      else consume_tile(j, slot, false);
    }
    if (j + 2 < nt) ATTN_WAIT_VMCNT(2);  // tile j+1 has landed; the two loads of tile j+2 stay in flight
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();  // tile j+1 full for everyone, tile j's slot empty
    slot = slot == NSLOT - 1 ? 0 : slot + 1;
  }

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
int launch_fp8(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.causal) hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, true>), dim3(grid), dim3(512), 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, false>), dim3(grid), dim3(512), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const AttnVariant* attn_fp8_variants(int* count) {
  static const AttnVariant table[] = {
      {"fp8 d128 BM256 BN64", 1, 128, 256, 64, 512, 2 * 3 * 64 * 128, launch_fp8<128>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
