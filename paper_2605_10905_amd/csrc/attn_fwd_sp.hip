// Fused attention forward for gfx950: the software-pipelined kernel, for bf16 inputs and for
// fp8 (e4m3) inputs.
//
// Mathematics (paper section 6.1 for the phases, appendix C.3 for the streaming-softmax state and
// the overlap of one block's QK^T product with the previous block's PV product): both products
// are taken transposed, S^T = K Q^T and O^T += V^T P^T, on the 32x32 MFMA shapes, so that a lane
// holds ONE query column and many keys: row sums are per-lane partial sums, the rescale factor
// is one scalar per lane, and the exponentiated, packed S^T accumulator IS the B operand of the
// second product (no shuffle, no LDS round trip).
//
// Orchestration.  All 8 waves of a workgroup run the same instruction stream, and that stream
// is pipelined over 32-key blocks so that the matrix pipe and the vector pipe are fed from the
// SAME wave at the same time (measured on gfx950: a wave that issues only MFMAs and a sibling
// that issues only VALU work delay each other at the shared issue port; one MFMA followed by
// three to five independent VALU instructions from the same wave is nearly free).  In the step
// that handles block u a wave
//     * exponentiates block u            (VALU:  P(u)   = exp2(c S(u) - m))
//     * computes the scores of block u+1 (MFMA:  S(u+1) = K(u+1) Q^T)
//     * accumulates block u-1            (MFMA:  O^T   += V(u-1)^T P(u-1)^T)
// The three streams are independent inside a step; a scheduling-group pipeline at the end of
// each scheduling region tells the compiler's scheduler the interleave: per MFMA its share of the
// exponentials and of the plain vector instructions, and the LDS reads of the operand a few
// MFMAs ahead.
//
// K/V streaming (the producer role).  Block u+1 of K and block u-1 of V travel together:
// "bundle" b holds key tile b+1 and value tile b (64 keys each) and is consumed by exactly one
// loop iteration, so a three-slot LDS ring with direct-to-LDS loads issued two bundles ahead
// needs one workgroup barrier per 64 keys: it is both the "full" signal of bundle b+1 and the
// "empty" signal of bundle b-1 (stage = b mod 3).  The barrier sits between the two 32-key steps
// of an iteration so that the first K operands of the next iteration can be read one step
// early; the loads into the slot it frees are issued one at a time at the region cuts of the
// iteration's second step, never in a burst that keeps every wave off the matrix pipe at once.
//
// No block maximum is taken on the common path: exponentials are computed against the current
// reference maximum, and only when a lane's partial row sum comes out large (or not a number,
// as on the very first block) is the true block maximum taken, the reference raised, the
// accumulator rescaled and the block redone (exact: any reference is valid for the streaming
// softmax as long as nothing overflows).
//
// fp8 inputs (FP8 = true).  S^T = K Q^T is taken directly on the e4m3 bytes with the 32x32x64
// f8f6f4 MFMA (two MFMAs per 32-key block instead of eight bf16 ones; K tiles of half the size go
// straight from memory into the ring).  P loses too much when it is rounded to e4m3 (a single
// term measures above the 2 % Frobenius bound), so P stays bf16 and V is converted e4m3 -> bf16,
// exactly, once per tile on arrival: the fp8 value tile lands in a two-slot staging area one
// bundle early, and every thread converts the 16 bytes it staged itself with the packed
// conversion and writes them, swizzled, into the ring slot the barrier has just freed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;

constexpr float kTau = 8.0f;
constexpr float kSumLimit = 65536.0f;  // a lane's 16-term partial sum above this redoes the block with a raised reference

template <int V>
using ic = std::integral_constant<int, V>;

// Scheduling-group pipeline of the MFMAs [M, M1) of a step (the builtin wants literal constants,
// hence the recursion).  The region [M0, M1) holds NVALU plain vector instructions and NEXP
// exponentials, spread evenly over its MFMAs; behind each MFMA come the LDS reads of the operand
// RA MFMAs ahead: QKR reads for a K fragment, two transposing reads for a V fragment.  MFMA m of a
// step is a score product iff m % STRIDE == 0.
template <int M, int M1, int NM, int RA, int NVALU, int NEXP, int STRIDE, int QKR, int M0 = M>
__device__ __forceinline__ void step_pipeline() {
  if constexpr (M < M1) {
    constexpr int NS = M1 - M0, J = M - M0;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                        // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, (NVALU * (J + 1)) / NS - (NVALU * J) / NS, 0);  // VALU
    __builtin_amdgcn_sched_group_barrier(0x400, (NEXP * (J + 1)) / NS - (NEXP * J) / NS, 0);    // transcendental
    __builtin_amdgcn_sched_group_barrier(0x100, ((M + RA) % NM) % STRIDE == 0 ? QKR : 2, 0);    // LDS read
    step_pipeline<M + 1, M1, NM, RA, NVALU, NEXP, STRIDE, QKR, M0>();
  }
}

// MODE says where a workgroup's query tiles come from.
//   0: one tile per workgroup (the tile the workgroup id maps to).
//   1: the launch has one workgroup per CU, and each takes tiles from a queue in device memory until
//      it is drained.  The queue is 8 counters, one per XCD list of the static tile order (a tile
//      index wg belongs to list wg % 8, the XCD the static launch would run it on, and lists are
//      consumed heaviest tile first); a workgroup serves the list of the XCD it was dispatched to
//      and, when that is empty, the lists after it, so every tile is taken exactly once whatever
//      the dispatch order was.  This is the software stand-in for the paper's cluster launch
//      control (section 4.2): dynamic assignment of tiles to resident workgroups.
//   2: one workgroup per CU again, but each walks a list fixed by arithmetic: the tiles of its XCD's
//      list are dealt to the XCD's workgroups in boustrophedon order (first to last, then last to
//      first, ...), which balances lists sorted by weight (causal inputs) without a queue, without
//      atomics and without any memory the library would have to own.
// In modes 1 and 2 consecutive tiles of a workgroup overlap at the seam: the next tile's first
// loads are requested as soon as every wave has left the ring, before the finished tile's output
// is packed, and the packed output is stored only when the next tile's loads have been waited
// for (loads and stores share one counter per wave, so a store in between would be waited for
// as well).
template <int D, bool CAUSAL, int MODE, bool FP8>
__global__ void __launch_bounds__(512, 2) attn_fwd_sp_kernel(const AttnParams p) {
  static_assert(!FP8 || (D == 128 && MODE != 1), "fp8 inputs: head dimension 128, no queue launch");
  constexpr int BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  constexpr int NCB = D / 32;                // 32-row blocks of O^T
  constexpr int ROWB = D * 2;                // bytes per bf16 row: V in the ring, O
  constexpr int INB = FP8 ? D : 2 * D;       // bytes per input row (q, k, v in memory; K rows in the ring)
  constexpr int NKQ = FP8 ? D / 64 : D / 16; // MFMA k-steps of S^T = K Q^T
  constexpr int KTILEB = BN * INB;           // bytes per K tile in the ring
  constexpr int KSUBB = 32 * INB;            // bytes per 32-key block of it
  constexpr int TILEB = BN * ROWB;           // bytes per bf16 V tile in the ring
  constexpr int SUBB = 32 * ROWB;            // bytes per 32-key block of it
  constexpr int NSLOT = 3;                   // ring depth: bundles are requested NSLOT-1 ahead
  constexpr int VBASE = NSLOT * KTILEB;      // K parts of the slots first, then the V parts
  constexpr int STGBASE = VBASE + NSLOT * TILEB;  // fp8: two staging slots of one e4m3 V tile each
  constexpr int STGTILE = BN * INB;
  constexpr int LDSB = FP8 ? STGBASE + 2 * STGTILE : STGBASE;
  constexpr int NCHI = INB / 16;             // 16-byte chunks per input row
  constexpr int NLD = BN * NCHI / NT;        // direct-to-LDS loads per thread per tile
  constexpr int QKR = FP8 ? 2 : 1;           // 128-bit LDS reads per K fragment
#ifndef ATTN_RA
#define ATTN_RA 4
#endif
  constexpr int RA = ATTN_RA;                // operands are read from LDS this many MFMAs ahead
  constexpr int NM = NKQ + 2 * NCB;          // MFMAs per 32-key step
  constexpr int STRIDE = NM / NKQ;           // MFMA m is a score product iff m % STRIDE == 0
  static_assert(BN * NCHI % NT == 0 && NLD >= 1 && (!FP8 || NLD == 1), "tile must divide evenly over the workgroup");
  static_assert(NM % NKQ == 0 && RA >= 2 && RA <= NM, "score products evenly spaced; read-ahead within a step");
  static_assert((NSLOT - 1) * TILEB + SUBB + 16 * ROWB < 65536, "ring offsets must fit the 16-bit LDS immediate");

  __shared__ __attribute__((aligned(1024))) char smem_raw[LDSB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;
  __shared__ int next_tile;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31;  // query column within the wave's 32-query block
  const int h = lane >> 5;   // which half of the k-slots / accumulator rows this lane holds

  // ---- the tile this workgroup works on (re-assigned at every seam in modes 1 and 2) ------------
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  int tile_b, tile_hq;              // batch and query head
  int q0, wq0;                      // first query row of the tile / of this wave
  bool wave_valid;
  const char *qhead, *khead, *vhead;
  int kv_end, nt;                   // keys the workgroup visits; 64-key tiles = bundles
  int qrow, limit, wlast;           // this lane's query row, its last visible key, the wave's last row
  auto set_tile = [&](int wg) __attribute__((always_inline)) {
    const AttnTileCoord tc = attn_tile_coord_map(wg, p.map);
    tile_b = tc.b;
    tile_hq = tc.hq;
    const int hk = tc.hq / G;
    q0 = tc.t * BM;
    wq0 = q0 + w * 32;
    wave_valid = wq0 < N;
    qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * INB;
    khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * INB;
    vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * INB;
    kv_end = CAUSAL ? min(N, q0 + BM) : N;
    nt = (kv_end + BN - 1) / BN;
    qrow = wq0 + qi;
    limit = CAUSAL ? min(qrow, N - 1) : (N - 1);
    wlast = wq0 + 31;
  };
  // Next tile index of this workgroup, -1 when there is none.  Every thread calls it; in mode 1
  // it contains the barrier after which no wave reads the ring of the finished tile any more.
  int lists_tried = 0;  // mode 1, thread 0 only
  int round = 0;        // mode 2: how many tiles this workgroup has taken
  auto next_tile_index = [&]() __attribute__((always_inline)) {
    if constexpr (MODE == 1) {
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
      const int wg = __builtin_amdgcn_readfirstlane(next_tile);
      __syncthreads();
      return wg;
    } else {
      // the grid is a multiple of 8 when the tile order has 8 lists (one per XCD), any size otherwise
      const int lists = ((p.B * p.Hkv) & 7) == 0 ? 8 : 1;
      const int per = (int)gridDim.x / lists;             // workgroups per list
      const int x = (int)blockIdx.x % lists, s = (int)blockIdx.x / lists;
      const int rank = round * per + ((round & 1) ? per - 1 - s : s);
      ++round;
      return rank * lists + x < p.total ? rank * lists + x : -1;
    }
  };

  // V rows in the ring (256 bytes, 16 chunks): which physical chunk holds logical chunk `chunk`
  // (columns 8 chunk .. 8 chunk + 7) of row `row`.  bf16: the XOR swizzle of the transposing read
  // (four consecutive rows in different 64-byte groups).  fp8: the conversion pass writes the
  // tile with 128-bit stores, which the LDS serves eight lanes (= one row's eight even or eight
  // odd logical chunks) per cycle, without a second pass only if those eight lie in one 128-byte
  // half of a bank line: the even logical chunks therefore fill the first half of a row and the
  // odd ones the second, and rows are told apart inside the halves (bits 1-2), which keeps the
  // transposing read's 32 lanes (4 rows x 64 bytes) on distinct banks as well.
  auto v_chunk = [](int row, int chunk) __attribute__((always_inline)) {
    if constexpr (FP8) return ((chunk >> 1) + 8 * (chunk & 1)) ^ ((row & 3) << 1);
    else return chunk ^ attn_swz_v<ROWB>(row);
  };

  // ---- producer role: direct-to-LDS tile loads ---------------------------------------------
  // Thread tid moves chunks tid, tid + NT, ... of a tile (16 bytes each).  K goes into the ring
  // (LDS chunk c of a row holds the row's chunk c ^ swizzle; the swizzle is applied on the
  // global-address side).  V: bf16 the same; fp8 into the staging area, unswizzled.
  // The "_r" offsets are those inside the ragged last tile, where rows past N-1 re-read row N-1
  // (finite data; masked out later): a load is then one select away from the regular one.
  uint32_t ld_koff[NLD], ld_voff[NLD], ld_koff_r[NLD], ld_voff_r[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCHI, c = s % NCHI;
    ld_koff[it] = r * INB + ((c ^ attn_swz_k<INB>(r)) << 4);
    ld_voff[it] = r * INB + ((FP8 ? c : v_chunk(r, c)) << 4);
    const uint32_t over = (uint32_t)max(0, (N - 1) / BN * BN + r - (N - 1)) * INB;
    ld_koff_r[it] = ld_koff[it] - over;
    ld_voff_r[it] = ld_voff[it] - over;
  }
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  // one load of key tile t into ring slot `slot` / of value tile t into ring slot (bf16) or
  // staging slot (fp8) `slot`; only the last tile of a ragged length takes the "_r" offsets
  auto load_k = [&](int t, int slot, int it) __attribute__((always_inline)) {
    attn_lds_dma16(khead + (size_t)t * KTILEB, (t + 1) * BN > N ? ld_koff_r[it] : ld_koff[it], lds_wave + slot * KTILEB + it * NT * 16);
  };
  auto load_v = [&](int t, int slot, int it) __attribute__((always_inline)) {
    attn_lds_dma16(vhead + (size_t)t * KTILEB, (t + 1) * BN > N ? ld_voff_r[it] : ld_voff[it],
                   lds_wave + (FP8 ? STGBASE + slot * STGTILE : VBASE + slot * TILEB) + it * NT * 16);
  };
  auto issue_k = [&](int t, int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < NLD; ++it) load_k(t, slot, it);
  };
  auto issue_v = [&](int t, int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < NLD; ++it) load_v(t, slot, it);
  };
  // fp8: where this thread's 16 staged values (row tid / 8, bytes 16 (tid % 8) ..) go in a bf16
  // value tile: chunks 2 (tid % 8) and 2 (tid % 8) + 1 of that row
  const int st_row = tid >> 3, st_c = tid & 7;
  const uint32_t cv_v0 = VBASE + st_row * ROWB + (v_chunk(st_row, 2 * st_c) << 4);
  const uint32_t cv_v1 = VBASE + st_row * ROWB + (v_chunk(st_row, 2 * st_c + 1) << 4);
  const uint32_t st_self = STGBASE + tid * 16;  // this thread's chunk inside a staged tile
  auto staged_chunk = [&](int stg) __attribute__((always_inline)) { return *(const LDS_AS u32x4*)(smem + st_self + stg * STGTILE); };
  auto convert_store = [&](const u32x4 in, int slot) __attribute__((always_inline)) {
    // 16 e4m3 bytes -> 16 bf16 (two 16-byte chunks), exact
    uint32_t o[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(in[i], 1.0f, false));
      o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(in[i], 1.0f, true));
    }
    *(LDS_AS u32x4*)(smem + cv_v0 + slot * TILEB) = u32x4{o[0], o[1], o[2], o[3]};
    *(LDS_AS u32x4*)(smem + cv_v1 + slot * TILEB) = u32x4{o[4], o[5], o[6], o[7]};
  };
  auto lds_ops_done = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };  // lgkmcnt(0)

  // ---- first requests of a tile: key tile 0, bundle 0 and the Q operand ---------------------------
  // bundle b = key tile b+1 (the last tile again if there is none) and value tile b.
  // Q is the B operand of S^T = K Q^T: bf16: lane (qi,h) holds Q[row][16kk + 8h .. +7];
  // fp8: Q[row][64kk + 32h .. +31].
  using QFrag = std::conditional_t<FP8, i32x8, bf16x8>;
  QFrag qf[NKQ];
  auto issue_prologue = [&]() __attribute__((always_inline)) {
    issue_k(0, NSLOT - 1);  // key tile 0 borrows the K part of the last slot
    issue_k(min(1, nt - 1), 0);
    issue_v(0, 0);
    const int row = min(wq0 + qi, N - 1);
    const char* src = qhead + (size_t)row * INB + h * (FP8 ? 32 : 16);
#pragma unroll
    for (int kk = 0; kk < NKQ; ++kk) {
      if constexpr (FP8) {
        const u32x4 lo = *(const u32x4*)(src + kk * 64), hi = *(const u32x4*)(src + kk * 64 + 16);
        qf[kk] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
      } else {
        qf[kk] = *(const bf16x8*)(src + kk * 32);
      }
    }
  };

  // ---- LDS read addresses (slot 0, first 32-key block) -----------------------------------------
  // K fragment of k-step kk: lane (qi,h) reads key row qi, chunk 2kk + h (bf16) or chunks
  // 4kk + 2h, + 1 (fp8)
  uint32_t kaddr[NKQ][QKR];
#pragma unroll
  for (int kk = 0; kk < NKQ; ++kk)
#pragma unroll
    for (int e = 0; e < QKR; ++e) kaddr[kk][e] = qi * INB + (((QKR * (2 * kk + h) + e) ^ attn_swz_k<INB>(qi)) << 4);
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
        vaddr[cb][e] = VBASE + key * ROWB + (v_chunk(key, chunk) << 4) + ((s & 1) << 3);
      }
  }
  // A block id names a 32-key block of the ring: 2 * slot + (which half of the slot's tiles)
  struct Operand {
    u32x4 x, y;  // K: the fragment (fp8: its low and high half); V: the fragment in x
  };
  auto k_operand = [&](auto koff, int kk) __attribute__((always_inline)) {
    Operand o;
    o.x = *(LDS_AS u32x4*)(smem + kaddr[kk][0] + koff);
    o.y = QKR > 1 ? *(LDS_AS u32x4*)(smem + kaddr[kk][QKR - 1] + koff) : o.x;
    return o;
  };
  auto v_operand = [&](auto voff, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][0] + voff + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + vaddr[cb][1] + voff + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    Operand o;
    o.x = __builtin_bit_cast(u32x4, av);
    o.y = o.x;
    return o;
  };
  auto qk_mfma = [&](const Operand& a, int kk, const f32x16& acc) __attribute__((always_inline)) {
    if constexpr (FP8) {
      const i32x8 av = i32x8{(int)a.x[0], (int)a.x[1], (int)a.x[2], (int)a.x[3], (int)a.y[0], (int)a.y[1], (int)a.y[2], (int)a.y[3]};
      // literal zero scale operands select the instruction without block scales (the scaled form
      // is not recognised as a matrix instruction by the scheduling-group pipeline and would be
      // left outside it, two dependent MFMAs back to back at the end of the step)
      return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, qf[kk], acc, 0, 0, 0, 0, 0, 0);
    } else {
      return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.x), qf[kk], acc, 0, 0, 0);
    }
  };

  // ---- streaming-softmax state ----------------------------------------------------------------
  f32x16 oacc[NCB];
  float m_ref;            // reference maximum, scaled log2 units
  float l_run;            // this lane's share of the row sum (halves are added at the end)
  const float c = p.scale_log2;
  f32x16 s_a, s_b;        // S^T of two consecutive blocks (one consumed, one produced)
  u32x4 p_a[2], p_b[2];   // packed P^T of two consecutive blocks (one produced, one consumed)

  // true maximum of a block in scaled log2 units (both lanes of a query column agree on it)
  auto block_max = [&](const f32x16& s) __attribute__((always_inline)) {
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
    return attn_max_halves(mx) * c;
  };
  // raise the reference maximum to cover mx and rescale what is relative to it: l and O
  auto raise_reference = [&](float mx) __attribute__((always_inline)) {
    const float m_new = fmaxf(m_ref, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // exp2(-inf) = 0 on the first block
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) oacc[cb] *= alpha;
    return alpha;
  };
  // exponentials of a whole block against the current reference, packed; returns the lane's sum
  auto exp_block = [&](const f32x16& s_in, u32x4 (&p_out)[2]) __attribute__((always_inline)) {
    f32x16 e;
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[r], c, -m_ref));
#pragma unroll
    for (int u = 0; u < 8; ++u) p_out[u >> 2][u & 3] = attn_pack_bf16(e[2 * u], e[2 * u + 1]);
    float ls0 = e[0], ls1 = e[1];
#pragma unroll
    for (int u = 1; u < 8; ++u) {
      ls0 += e[2 * u];
      ls1 += e[2 * u + 1];
    }
    return ls0 + ls1;
  };

  // ---- boundary-case building blocks (compiler-scheduled, not overlapped) ----------------------
  auto qk_block = [&](f32x16& s, auto koff) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKQ; ++kk) s = qk_mfma(k_operand(koff, kk), kk, s);
  };
  auto pv_block = [&](const u32x4 (&pk)[2], auto voff) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2 * NCB; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v_operand(voff, cb, kc).x),
                                                         __builtin_bit_cast(bf16x8, pk[kc]), oacc[cb], 0, 0, 0);
    }
  };
  // softmax of a block that may need masking, with the block maximum taken first; `pend` is the
  // packed P^T of the block whose PV product has not been issued yet (rescaled with O)
  auto softmax_block = [&](f32x16& s, u32x4 (&pk)[2], u32x4 (&pend)[2], int key0, bool need_mask) __attribute__((always_inline)) {
    if (need_mask) {
      const int kbase = key0 + 4 * h;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kbase + 8 * (r >> 2) + (r & 3) > limit) s[r] = -INFINITY;
    }
    const float mx = block_max(s);
    if (__builtin_amdgcn_ballot_w64(mx > m_ref + kTau) != 0) {
      const float alpha = raise_reference(mx);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t u = pend[i][r];
          pend[i][r] = attn_pack_bf16(__uint_as_float(u << 16) * alpha, __uint_as_float(u & 0xffff0000u) * alpha);
        }
    }
    l_run += exp_block(s, pk);
  };
  auto is_active = [&](int key0) __attribute__((always_inline)) {
    return wave_valid && key0 < kv_end && (!CAUSAL || key0 <= wlast);
  };
  auto needs_mask = [&](int key0) __attribute__((always_inline)) {
    return (CAUSAL && key0 + 31 > wq0) || key0 + 31 >= N;
  };

  // ---- the pipelined step on fully visible blocks ------------------------------------------------
  //   s_in  : scores of the block exponentiated now                     -> p_out
  //   s_out : scores of the next block        (K operands of block id bid)
  //   p_pv  : probabilities of the previous block, multiplied into O    (V operands of block id bid)
  // Of the NM MFMAs of a step every STRIDE-th is a score product (a dependent chain), the others
  // are PV products (independent accumulators); operands are read from LDS RA MFMAs ahead, and
  // the first RA operands of a step are requested by the previous step (bidnext = the block the
  // next step reads).  The vector work needs no block maximum: exponentials are taken against
  // the current reference and the block is redone, after raising the reference and rescaling,
  // only if a lane's partial sum comes out large or not a number (always on the very first
  // block).  Source order inside a scheduling region does not matter: the scheduling-group
  // pipeline at its end tells the scheduler how to interleave the four instruction classes.
  // NSEG > 1 cuts the step into NSEG regions of NM / NSEG MFMAs (each with its share of the
  // exponentials, sums and packs); between(i) runs in front of region i, which is where the
  // producer role's work goes.
  Operand pre[RA];
  auto koff_of = [](auto bid) __attribute__((always_inline)) { return ic<(decltype(bid)::value >> 1) * KTILEB + (decltype(bid)::value & 1) * KSUBB>{}; };
  auto voff_of = [](auto bid) __attribute__((always_inline)) { return ic<(decltype(bid)::value >> 1) * TILEB + (decltype(bid)::value & 1) * SUBB>{}; };
  auto step_operand = [&](auto bid, int m) __attribute__((always_inline)) {
    const int i = m - m / STRIDE - 1;
    return m % STRIDE == 0 ? k_operand(koff_of(bid), m / STRIDE) : v_operand(voff_of(bid), i % NCB, i / NCB);
  };
  auto step_hot = [&](f32x16& s_in, f32x16& s_out, u32x4 (&p_out)[2], u32x4 (&p_pv)[2], auto bid, auto bidnext, auto nseg_tag, auto between) __attribute__((always_inline)) {
    constexpr int NSEG = decltype(nseg_tag)::value, SEG = NM / NSEG;
    static_assert(NSEG <= 4 && NM % NSEG == 0 && (16 / NSEG) % 2 == 0 && 16 % NSEG == 0, "regions hold whole MFMAs and whole pairs of scores");
    Operand op[NM];
#pragma unroll
    for (int m = 0; m < RA; ++m) op[m] = pre[m];
#pragma unroll
    for (int r = 0; r < 16; ++r) s_out[r] = 0.f;
    float ls0 = 0.f, ls1 = 0.f;
    float e[16];
    auto segment = [&](auto seg_tag) __attribute__((always_inline)) {
      constexpr int SG = decltype(seg_tag)::value, M0 = SG * SEG, M1 = M0 + SEG;
      constexpr int R0 = 16 * SG / NSEG, R1 = 16 * (SG + 1) / NSEG;  // scores exponentiated in this region
      between(SG);
      if constexpr (SG > 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = M0; m < M1; ++m) {
        if (m % STRIDE == 0) {
          s_out = qk_mfma(op[m], m / STRIDE, s_out);
        } else {
          const int i = m - m / STRIDE - 1;
          oacc[i % NCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m].x), __builtin_bit_cast(bf16x8, p_pv[i / NCB]),
                                                                  oacc[i % NCB], 0, 0, 0);
        }
        if (m + RA < NM) op[m + RA] = step_operand(bid, m + RA);
        else pre[m + RA - NM] = step_operand(bidnext, m + RA - NM);
      }
#pragma unroll
      for (int r = R0; r < R1; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[r], c, -m_ref));
#pragma unroll
      for (int u = R0 / 2; u < R1 / 2; ++u) {
        p_out[u >> 2][u & 3] = attn_pack_bf16(e[2 * u], e[2 * u + 1]);
        ls0 = u == 0 ? e[0] : ls0 + e[2 * u];
        ls1 = u == 0 ? e[1] : ls1 + e[2 * u + 1];
      }
      if constexpr (SG == NSEG - 1) ls0 += ls1;
      // multiply-adds, packs and adds of this region (the first pair starts the two sums, the
      // last region adds them and compares)
      constexpr int NVALU = (R1 - R0) + 3 * ((R1 - R0) / 2) - (SG == 0 ? 2 : 0) + (SG == NSEG - 1 ? 2 : 0);
      step_pipeline<M0, M1, NM, RA, NVALU, R1 - R0, STRIDE, QKR>();
      if constexpr (SG + 1 < NSEG) __builtin_amdgcn_sched_barrier(0);
    };
    segment(ic<0>{});
    if constexpr (NSEG > 1) segment(ic<1>{});
    if constexpr (NSEG > 2) segment(ic<2>{});
    if constexpr (NSEG > 3) segment(ic<3>{});
    float ls = ls0;
    if (__builtin_amdgcn_ballot_w64(!(ls <= kSumLimit)) != 0) {
      // the redo path "reads" the optimistic packs, so that they are computed inside the
      // pipelined region above and not sunk below this branch into the common path's tail
      asm volatile("" ::"v"(p_out[0]), "v"(p_out[1]));
      raise_reference(block_max(s_in));
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

  // ---- main loop over bundles ------------------------------------------------------------------------
  // Iteration b: exponentiate blocks 2b+1 and 2b+2, compute the scores of blocks 2b+2 and 2b+3
  // (key tile b+1), accumulate blocks 2b and 2b+1 (value tile b).  Between its two steps bundle
  // b+1 (requested one iteration ago) is published and the slot of bundle b-1, which every wave
  // has finished reading, is handed to bundle b+2: bf16 requests its key and value tiles into it;
  // fp8 requests its key tile into it, converts its staged value tile (staging slot b mod 2) into
  // it, and stages the value tile of bundle b+3 where that of bundle b+1 was converted from.
  // A wave's LDS writes must have completed before it signals the barrier that publishes them.
  auto publish_and_free = [&](bool drain_lds) __attribute__((always_inline)) {
    ATTN_WAIT_VMCNT(0);
    if (FP8 && drain_lds) lds_ops_done();
    attn_wg_barrier();
  };
  // burst form, for the iterations that are not pipelined
  auto bundle_mid = [&](int b, int free_slot) __attribute__((always_inline)) {
    publish_and_free(true);
    if (b + 2 < nt) {
      issue_k(min(b + 3, nt - 1), free_slot);
      if constexpr (FP8) convert_store(staged_chunk(b & 1), free_slot);
      else issue_v(b + 2, free_slot);
    }
    if constexpr (FP8)
      if (b + 3 < nt) issue_v(b + 3, (b + 1) & 1);
  };
  auto nothing = [](int) __attribute__((always_inline)) {};
  // Pipelined form: the same work is handed out over the region cuts of the iteration's second
  // step, one piece in front of each region, between the operand reads.  A bundle index past the
  // end re-requests the last tiles into the free slot, which is never read again (and converts
  // whatever the staging slot holds): the loads in flight per wave are then the same in every
  // iteration.
  auto bundle_hot = [&](int b, auto slot_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    constexpr int FREE = (SLOT + NSLOT - 1) % NSLOT;
    constexpr int NSEG = FP8 ? 2 : (2 * NLD < 2 ? 2 : 2 * NLD);
    step_hot(s_a, s_b, p_a, p_b, ic<2 * SLOT>{}, ic<2 * SLOT + 1>{}, ic<NSEG>{}, nothing);
    const int kt = min(b + 3, nt - 1), vt = min(b + 2, nt - 1);  // key and value tile of bundle b+2
    u32x4 staged;
    auto producer = [&](int sg) __attribute__((always_inline)) {
      // (the conversion's LDS writes of the previous iteration have retired: LDS operations
      // complete in order, and this wave has since waited for dozens of later operand reads)
      if (sg == 0) publish_and_free(false);
      if constexpr (FP8) {
        if (sg == 0) {
          load_k(kt, FREE, 0);
          staged = staged_chunk(b & 1);
        } else {
          convert_store(staged, FREE);
          load_v(min(b + 3, nt - 1), (b + 1) & 1, 0);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 2 * NLD; ++j) {
          if ((j < NSEG ? j : NSEG - 1) != sg) continue;
          if (j < NLD) load_k(kt, FREE, j);
          else load_v(vt, FREE, j - NLD);
        }
      }
    };
    step_hot(s_b, s_a, p_b, p_a, ic<2 * SLOT + 1>{}, ic<2 * ((SLOT + 1) % NSLOT)>{}, ic<NSEG>{}, producer);
  };
  auto bundle_any = [&](int b, int slot) __attribute__((always_inline)) {
    const int k1 = (2 * b + 1) * 32, k2 = k1 + 32;
    step_any(is_active(k1), k1, is_active(k1 - 32), s_a, s_b, p_a, p_b, slot * KTILEB, slot * TILEB);
    bundle_mid(b, slot >= 1 ? slot - 1 : NSLOT - 1);
    step_any(is_active(k2), k2, is_active(k1), s_b, s_a, p_b, p_a, slot * KTILEB + KSUBB, slot * TILEB + SUBB);
  };

  // ---- the tiles of this workgroup -----------------------------------------------------------------
  int wg = (int)blockIdx.x;
  if constexpr (MODE != 0) {
    wg = next_tile_index();
    if (wg < 0) return;
  }
  set_tile(wg);
  issue_prologue();
  // output of the previous tile, packed, waiting to be stored (modes 1 and 2)
  u32x4 pend_o[2 * NCB];
  float pend_lse = 0.f;
  char* pend_o_ptr = nullptr;   // this lane's output row (null: row past the end)
  float* pend_lse_ptr = nullptr;  // this lane's lse element (null: not this lane's to write)
  bool pending = false;
  for (;;) {
    // fresh streaming-softmax state
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
    m_ref = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) p_a[i] = p_b[i] = u32x4{0, 0, 0, 0};

    // ---- prologue: block 0 ---------------------------------------------------------------------------
    if constexpr (FP8) {
      // everything requested so far has landed: convert value tile 0 into slot 0, request key tile 2
      // and stage value tiles 1 and 2
      ATTN_WAIT_VMCNT(0);
  #pragma unroll
      for (int kk = 0; kk < NKQ; ++kk)
  #pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(qf[kk][i]));  // Q is in registers from here on
      convert_store(staged_chunk(0), 0);
      lds_ops_done();
      if (nt > 1) {
        issue_k(min(2, nt - 1), 1);
        issue_v(1, 1);
      }
      if (nt > 2) issue_v(2, 0);
    } else {
      // Q is in registers from here on.  The compiler waits for Q with the counter that the
      // direct-to-LDS loads share and cannot see them, so this is a wait for every load issued
      // so far: bundle 1 is therefore requested only behind the barrier.
      ATTN_WAIT_VMCNT(0);
  #pragma unroll
      for (int kk = 0; kk < NKQ; ++kk) asm volatile("" ::"v"(qf[kk]));
    }
    attn_wg_barrier();
    if constexpr (!FP8) {
      if (nt > 1) {
        issue_k(min(2, nt - 1), 1);
        issue_v(1, 1);
      }
    }
    if (wave_valid) {
      qk_block(s_b, (NSLOT - 1) * KTILEB);             // S(0)
      softmax_block(s_b, p_b, p_a, 0, needs_mask(0));  // P(0) -> p_b (nothing pending yet)
      qk_block(s_a, (NSLOT - 1) * KTILEB + KSUBB);     // S(1); ignored if block 1 is not visible
    }
    if constexpr (FP8) {
      // bundle 1 has arrived once only value tile 2's load is outstanding: convert its value tile into slot 1
      if (nt > 1) {
        if (nt > 2) ATTN_WAIT_VMCNT(1);
        else ATTN_WAIT_VMCNT(0);
        convert_store(staged_chunk(1), 1);
        lds_ops_done();
      }
    } else {
      if (nt > 1) ATTN_WAIT_VMCNT(2 * NLD);
      else ATTN_WAIT_VMCNT(0);
    }
    attn_wg_barrier();  // bundle 0 is full; the K part of the last slot is empty again
    if constexpr (MODE != 0) {
      // every load of this tile's prologue has been waited for: the previous tile's output may go
      if (pending) {
        if (pend_lse_ptr) *pend_lse_ptr = pend_lse;
        if (pend_o_ptr) attn_store_packed_o<NCB>(pend_o, pend_o_ptr);
      }
    }
  #pragma unroll
    for (int m = 0; m < RA; ++m) pre[m] = step_operand(ic<0>{}, m);  // first operands of the first pipelined step (block id 0)


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


    // ---- epilogue: O = acc / l (bf16), lse = (m + log2 l) * ln 2 ----------------------------------
    const float l = attn_sum_halves(l_run);
    const float lse_val = (m_ref + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    float* const lse_ptr = (qrow < N && h == 0) ? p.lse + (size_t)(tile_b * p.Hq + tile_hq) * N + qrow : nullptr;
    char* const o_ptr = qrow < N ? (char*)p.o + ((size_t)(tile_b * p.Hq + tile_hq) * N + qrow) * ROWB : nullptr;
    if constexpr (MODE == 0) {
      if (lse_ptr) *lse_ptr = lse_val;
      attn_pack_o_rows<NCB>(oacc, p.out_scale / l, pend_o);
      if (o_ptr) attn_store_packed_o<NCB>(pend_o, o_ptr + h * 16);
      break;
    } else {
      // seam: once no wave reads the ring any more, request the next tile's first loads, then
      // pack this tile's output; it is stored when those loads have been waited for
      if constexpr (MODE == 2) attn_wg_barrier();
      const int nwg = next_tile_index();
      if (nwg >= 0) {
        set_tile(nwg);
        issue_prologue();
      }
      attn_pack_o_rows<NCB>(oacc, p.out_scale / l, pend_o);
      pend_lse = lse_val;
      pend_lse_ptr = lse_ptr;
      pend_o_ptr = o_ptr ? o_ptr + h * 16 : nullptr;
      pending = true;
      if (nwg < 0) {
        if (pend_lse_ptr) *pend_lse_ptr = pend_lse;
        if (pend_o_ptr) attn_store_packed_o<NCB>(pend_o, pend_o_ptr);
        break;
      }
    }
  }  // tile loop
}

// resident workgroups of the list-walking launch: one per CU, rounded down to whole XCD shares
int resident_workgroups() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return cus - cus % 8;
}

// Causal launches with at least three tiles per CU walk static tile lists (mode 2): the seams
// between a workgroup's tiles hide part of what a workgroup pays per tile outside its main loop
// (measured: +0.5 .. +4.5 %; with two tiles per CU the plain launch is 1 % faster).  Non-causal
// launches run one tile per workgroup: in the list-walking instantiation the compiler's greedy
// scheduling-group solver interleaves the pipelined step less well (5 % more cycles).
template <int D, bool FP8>
int launch_sp(const AttnParams& p, int grid, hipStream_t stream) {
  const int resident = p.causal ? resident_workgroups() : 0;
  if (p.causal && resident >= 8 && grid >= 3 * resident) {
    AttnParams q = p;
    q.total = grid;
    hipLaunchKernelGGL((attn_fwd_sp_kernel<D, true, 2, FP8>), dim3(resident), dim3(512), 0, stream, q);
  } else if (p.causal) {
    hipLaunchKernelGGL((attn_fwd_sp_kernel<D, true, 0, FP8>), dim3(grid), dim3(512), 0, stream, p);
  } else {
    hipLaunchKernelGGL((attn_fwd_sp_kernel<D, false, 0, FP8>), dim3(grid), dim3(512), 0, stream, p);
  }
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
    if (p.causal) hipLaunchKernelGGL((attn_fwd_sp_kernel<128, true, 1, false>), grid, dim3(512), 0, stream, p);
    else hipLaunchKernelGGL((attn_fwd_sp_kernel<128, false, 1, false>), grid, dim3(512), 0, stream, p);
  } else if (d == 64) {
    if (p.causal) hipLaunchKernelGGL((attn_fwd_sp_kernel<64, true, 1, false>), grid, dim3(512), 0, stream, p);
    else hipLaunchKernelGGL((attn_fwd_sp_kernel<64, false, 1, false>), grid, dim3(512), 0, stream, p);
  } else {
    return -1;
  }
  return (int)hipGetLastError();
}

const AttnVariant* attn_sp_variants(int* count) {
  static const AttnVariant table[] = {
      {"bf16 d128 pipelined BM256 BN64", 0, 128, 256, 64, 512, 2 * 3 * 64 * 128 * 2, launch_sp<128, false>},
      {"bf16 d64 pipelined BM256 BN64", 0, 64, 256, 64, 512, 2 * 3 * 64 * 64 * 2, launch_sp<64, false>},
      {"fp8 d128 fp8-QK bf16-PV pipelined BM256 BN64", 1, 128, 256, 64, 512, 3 * 64 * 128 + 3 * 64 * 256 + 2 * 64 * 128, launch_sp<128, true>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
