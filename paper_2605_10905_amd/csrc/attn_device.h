// Device-side helpers shared by the gfx950 attention kernels: vector types, the LDS tile
// swizzles, the direct-to-LDS load, and the two-lane exchange used by the row reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

__device__ __forceinline__ constexpr int attn_ilog2(int x) { return x <= 1 ? 0 : 1 + attn_ilog2(x >> 1); }

// K and V tiles live in LDS row-major (one key per row, ROWB bytes) with the index of each
// 16-byte chunk XORed with a function of the row.
//  * K is read as MFMA A operands: 16 consecutive lanes read the same chunk of 16 consecutive
//    rows, so the XOR term must differ over 16 consecutive rows (and, counting the two lane
//    halves that differ in the lowest chunk bit, over 8 rows in the upper bits): a rotate-left
//    of the row bits.
//  * V is read with the transposing load: 16 lanes cover 4 consecutive rows x 32 bytes, so
//    consecutive rows must land in different 64-byte groups.
template <int ROWB>
__device__ __forceinline__ constexpr int attn_swz_k(int row) {
  constexpr int NCH = ROWB / 16, BITS = attn_ilog2(NCH), RP = 256 / ROWB;
  const int a = (row / RP) & (NCH - 1);
  return ((a << 1) | (a >> (BITS - 1))) & (NCH - 1);
}
template <int ROWB>
__device__ __forceinline__ constexpr int attn_swz_v(int row) {
  constexpr int NCH = ROWB / 16, RP = 256 / ROWB;
  return ((row / RP) & (NCH / 4 - 1)) << 2;
}

// max / sum over lane l and lane l^32 (the two lanes that hold the same query column)
__device__ __forceinline__ float attn_max_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float attn_sum_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// two floats -> two bf16 (round to nearest even) in one word, the first in the low half
__device__ __forceinline__ uint32_t attn_pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

// Epilogue of the transposed accumulator layout shared by the forward kernels: lane (qi, h) of a
// wave holds, for its query row, the O^T rows 32cb + 8b + 4h + r (b = 0..3, r = 0..3) of every
// 32-row block cb.  attn_pack_o_rows scales by `inv` (1 / row sum, times any output scale), rounds
// to bf16 and lets the two lanes of a query exchange halves, so that each owns 8 consecutive
// output columns 32cb + 16a + 8h + (0..7) in out[2cb + a]; attn_store_packed_o writes them with
// one 16-byte store each, `dst` pointing at column 8h of the lane's output row.
template <int NCB>
__device__ __forceinline__ void attn_pack_o_rows(const f32x16 (&oacc)[NCB], float inv, u32x4 (&out)[2 * NCB]) {
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      uint32_t x[2], y[2];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const uint32_t tx = attn_pack_bf16(oacc[cb][(2 * a) * 4 + 2 * r] * inv, oacc[cb][(2 * a) * 4 + 2 * r + 1] * inv);
        const uint32_t ty = attn_pack_bf16(oacc[cb][(2 * a + 1) * 4 + 2 * r] * inv, oacc[cb][(2 * a + 1) * 4 + 2 * r + 1] * inv);
        auto sw = __builtin_amdgcn_permlane32_swap(tx, ty, false, false);
        x[r] = sw[0];
        y[r] = sw[1];
      }
      out[2 * cb + a] = u32x4{x[0], x[1], y[0], y[1]};
    }
}
template <int NCB>
__device__ __forceinline__ void attn_store_packed_o(const u32x4 (&out)[2 * NCB], char* dst) {
#pragma unroll
  for (int i = 0; i < 2 * NCB; ++i) *(u32x4*)(dst + i * 32) = out[i];
}

// Direct-to-LDS 128-bit load: lane i of the wave copies 16 bytes from sbase + voff to LDS
// address lds_base + 16*i.  Inline assembly (uniform 64-bit base in SGPRs plus a per-lane
// 32-bit offset, no VALU address arithmetic), so that the compiler does not serialise later
// LDS reads of OTHER ring slots behind it; completion is tracked by hand with s_waitcnt
// vmcnt before the barrier that publishes the slot.  The statement overwrites m0 and says so.
__device__ __forceinline__ void attn_lds_dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "m0");
}

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left alone)
#define ATTN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))

// workgroup barrier that the instruction scheduler may not move code across
__device__ __forceinline__ void attn_wg_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}
