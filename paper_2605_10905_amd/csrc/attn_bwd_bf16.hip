// Attention backward, bf16, gfx950 (head dimension 128 or 64).
//
// The paper lists the backward pass beside the forward among its attention kernels (section
// 6.1; appendix A, attention shape table, backward rows).  Given Q, K, V, the forward output O
// with its per-row logsumexp, and the output gradient dO:
//
//     P  = exp(scale Q K^T - lse)             (rebuilt from the stored statistic, no maximum needed)
//     dV = P^T dO        dP = dO V^T        delta_i = sum_d dO_id O_id
//     dS = P * (dP - delta)                 dQ = scale dS K        dK = scale dS^T Q
//
// Two kernels, neither of which uses atomics or a reduction across workgroups, so the result is
// deterministic and no gradient needs an fp32 accumulation buffer in memory:
//
//   * attn_bwd_dq_kernel: a workgroup owns 256 query rows (Q and dO rows stationary in registers
//     as MFMA B operands, one query per lane, exactly the forward layout) and streams K/V tiles:
//     S^T = K Q^T, dP^T = V dO^T, dS^T in registers, dQ^T += K^T dS^T.  It also writes the two
//     per-row vectors the other kernel needs, delta and lse * log2(e), into the workspace.
//   * attn_bwd_dkv_pipe_kernel: a workgroup owns 128 keys (K and V rows stationary, one key per
//     lane) and streams Q/dO tiles of every query head of its group: S = Q K^T, dP = dO V^T, P,
//     dS = P * (dP - delta), dV^T += dO^T P, dK^T += Q^T dS.
//   S and dP are therefore computed twice, 7 matrix products per tile pair instead of the minimal
//   5: the price of keeping every accumulator in registers without atomics.
//
// Both share the forward kernels' machinery: 64-row tiles streamed HBM/L2 -> LDS by
// direct-to-LDS loads into a ring of slots two tiles ahead (one workgroup barrier per tile),
// transposed products on the 32x32x16 MFMA so that the exponentiated accumulator is the next
// B operand in place, and the transposing LDS read for the operand that must be contracted
// over its row index.  Streamed tiles are read both row-wise and transposed, so their 16-byte
// chunks are swizzled with a bit-swap of the row (conflict-free for both patterns).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int V>
using ic = std::integral_constant<int, V>;

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

// Chunk swizzle of a streamed tile.  256-byte rows (16 chunks): XOR with the bit-swapped low four
// row bits.  Row-wise operand reads (16 lanes, one chunk of 16 consecutive rows) see 16 different
// values; transposing reads (16 lanes over 4 consecutive rows x 32 bytes, two such groups on
// neighbouring chunk pairs served together) see the rows in different 64-byte groups.
// 128-byte rows (8 chunks, two rows per 256-byte bank line): rows of equal parity share a half
// line, so the XOR value is built from row bits 1-3: bit 1 selects the 64-byte group (rows r and
// r + 2, which a transposing read takes together, fall into different groups), bits 2-3 the chunk
// inside it; 16 consecutive rows then see every (half line, chunk) pair once.
template <int ROWB>
__device__ __forceinline__ constexpr int swz_rt(int row) {
  static_assert(ROWB == 256 || ROWB == 128, "row of 128 or 64 bf16");
  return ROWB == 256 ? ((row & 3) << 2) | ((row >> 2) & 3) : (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}

template <int D_>
struct BwdCommon {
  static constexpr int D = D_, BN = 64, NWAVES = 8, BM = NWAVES * 32, NT = NWAVES * 64;
  static constexpr int NKK = D / 16, NCB = D / 32, ROWB = D * 2, NCH = ROWB / 16;
  static constexpr int TILEB = BN * ROWB, SUBB = 32 * ROWB, NSLOT = 3;
  static constexpr int T2BASE = NSLOT * TILEB;       // second streamed tensor's slots
  static constexpr int AUXBASE = 2 * NSLOT * TILEB;  // per-slot 512 bytes: lse*log2e and delta of the tile's 64 rows
  static constexpr int NLD = BN * NCH / NT;
  static constexpr int LDS_BYTES = AUXBASE + NSLOT * 512;
};

// store a transposed accumulator (lane (ci,h) holds rows 32cb + 8a + 4h + r of column ci) as
// row `row` of a [.., D] bf16 matrix, scaled; the two lane halves exchange so that every lane
// writes 8 consecutive columns with one 16-byte store
template <int NCB>
__device__ __forceinline__ void store_transposed(const f32x16 (&acc)[NCB], float mul, char* rowptr, int h, bool valid) {
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      uint32_t x[2], y[2];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const uint32_t tx = pack_bf16(acc[cb][(2 * a) * 4 + 2 * r] * mul, acc[cb][(2 * a) * 4 + 2 * r + 1] * mul);
        const uint32_t ty = pack_bf16(acc[cb][(2 * a + 1) * 4 + 2 * r] * mul, acc[cb][(2 * a + 1) * 4 + 2 * r + 1] * mul);
        auto sw = __builtin_amdgcn_permlane32_swap(tx, ty, false, false);
        x[r] = sw[0];
        y[r] = sw[1];
      }
      if (valid) {
        u32x4 out = {x[0], x[1], y[0], y[1]};
        *(u32x4*)(rowptr + (cb * 32 + a * 16 + h * 8) * 2) = out;
      }
    }
}

// =====================================================================================================
// dQ (and the workspace vectors)
// =====================================================================================================
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 2) attn_bwd_dq_kernel(const AttnBwdParams p) {
  using C = BwdCommon<D>;
  constexpr int NKK = C::NKK, NCB = C::NCB, ROWB = C::ROWB, NCH = C::NCH, TILEB = C::TILEB, SUBB = C::SUBB, NSLOT = C::NSLOT;
  constexpr int NLD = C::NLD, NT = C::NT, BN = C::BN, BM = C::BM;

  __shared__ __attribute__((aligned(1024))) char smem_raw[2 * NSLOT * TILEB];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int qi = lane & 31, h = lane >> 5;

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int hk = tc.hq / (p.Hq / p.Hkv);
  const int q0 = tc.t * BM;
  const int wq0 = q0 + w * 32;
  const bool wave_valid = wq0 < N;
  const int qrow = wq0 + qi;

  const size_t qoff = ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;

  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;
  const int nt = (kv_end + BN - 1) / BN;

  // ---- producer role ------------------------------------------------------------------------------
  int ld_row[NLD];
  uint32_t ld_off[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCH, c = s % NCH;
    ld_row[it] = r;
    ld_off[it] = r * ROWB + ((c ^ swz_rt<ROWB>(r)) << 4);
  }
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_tile = [&](int j, int slot) __attribute__((always_inline)) {
    const char* const kb = khead + (size_t)j * TILEB;
    const char* const vb = vhead + (size_t)j * TILEB;
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      const uint32_t over = (uint32_t)max(0, j * BN + ld_row[it] - (N - 1)) * ROWB;  // rows past N-1 re-read row N-1
      attn_lds_dma16(kb, ld_off[it] - over, lds_wave + slot * TILEB + it * NT * 16);
      attn_lds_dma16(vb, ld_off[it] - over, lds_wave + C::T2BASE + slot * TILEB + it * NT * 16);
    }
  };
  issue_tile(0, 0);

  // ---- stationary operands: Q and dO rows of this lane's query; delta from dO and O ---------------
  bf16x8 qf[NKK], dof[NKK];
  float delta;
  {
    const int row = min(qrow, N - 1);
    const char* qs = (const char*)p.q + qoff + (size_t)row * ROWB + h * 16;
    const char* ds = (const char*)p.dout + qoff + (size_t)row * ROWB + h * 16;
    const char* os = (const char*)p.o + qoff + (size_t)row * ROWB + h * 16;
    float acc = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      qf[kk] = *(const bf16x8*)(qs + kk * 32);
      dof[kk] = *(const bf16x8*)(ds + kk * 32);
      const bf16x8 ov = *(const bf16x8*)(os + kk * 32);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc += (float)dof[kk][e] * (float)ov[e];
    }
    delta = attn_sum_halves(acc);
  }
  const float lse2 = p.lse[(size_t)(tc.b * p.Hq + tc.hq) * N + min(qrow, N - 1)] * kLog2e;
  // workspace for the key-side kernels, padded to whole 64-row tiles: rows past N get a
  // statistic of +inf (their probabilities come out as zero) and delta = 0
  if (h == 0 && qrow < p.Npad) {
    float* const wsrow = p.ws + (size_t)(tc.b * p.Hq + tc.hq) * 2 * p.Npad;
    wsrow[qrow] = qrow < N ? lse2 : INFINITY;
    wsrow[p.Npad + qrow] = qrow < N ? delta : 0.f;
  }
  if (nt > 1) issue_tile(1, 1);

  // ---- LDS read addresses (slot 0, first 32-row block) --------------------------------------------
  uint32_t raddr[NKK];  // row-wise operand: row qi, chunk 2kk + h
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) raddr[kk] = qi * ROWB + (((2 * kk + h) ^ swz_rt<ROWB>(qi)) << 4);
  uint32_t taddr[NCB][2];  // transposed operand through the transposing load
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int key = 8 * e + 4 * h + (s >> 2);
        const int chunk = cb * 4 + chalf * 2 + ((s & 3) >> 1);
        taddr[cb][e] = key * ROWB + ((chunk ^ swz_rt<ROWB>(key)) << 4) + ((s & 1) << 3);
      }
  }
  auto row_operand = [&](int base, int kk) __attribute__((always_inline)) { return *(LDS_AS bf16x8*)(smem + raddr[kk] + base); };
  auto tr_operand = [&](int base, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + taddr[cb][0] + base + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + taddr[cb][1] + base + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return __builtin_bit_cast(bf16x8, av);
  };

  f32x16 acc[NCB];  // dQ^T
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  const float c = p.scale_log2;
  const int limit = CAUSAL ? min(qrow, N - 1) : (N - 1);
  const int wlast = wq0 + 31;

  // one 32-key block: `base` = byte offset of the block inside the K slots (V: + T2BASE)
  auto block = [&](int key0, int base) __attribute__((always_inline)) {
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_operand(base, kk), qf[kk], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_operand(base + C::T2BASE, kk), dof[kk], dp, 0, 0, 0);
    }
    // invisible keys (causal diagonal, ragged tail): a score of -inf gives P = 0 and dS = 0.  The
    // compare / select work sits behind a wave-uniform branch, the common case carries none of it.
    if ((CAUSAL && key0 + 31 > wq0) || key0 + 31 >= N) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (key0 + 4 * h + 8 * (r >> 2) + (r & 3) > limit) s[r] = -INFINITY;
    }
    u32x4 dsk[2];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      float e[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int r = 2 * u + t;
        const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse2));
        e[t] = pr * (dp[r] - delta);
      }
      dsk[u >> 2][u & 3] = pack_bf16(e[0], e[1]);
    }
#pragma unroll
    for (int i = 0; i < 2 * NCB; ++i) {
      const int cb = i % NCB, kc = i / NCB;
      acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_operand(base, cb, kc), __builtin_bit_cast(bf16x8, dsk[kc]), acc[cb], 0, 0, 0);
    }
  };

  if (nt > 1) ATTN_WAIT_VMCNT(2 * NLD);
  else ATTN_WAIT_VMCNT(0);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) asm volatile("" ::"v"(qf[kk]), "v"(dof[kk]));  // stationary operands are in registers
  attn_wg_barrier();

  int slot = 0;
  for (int j = 0; j < nt; ++j) {
    const int pslot = slot == 0 ? NSLOT - 1 : slot - 1;  // slot of tile j+2 = slot of tile j-1
    if (j + 2 < nt) issue_tile(j + 2, pslot);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int key0 = j * BN + kb * 32;
      if (wave_valid && key0 < kv_end && (!CAUSAL || key0 <= wlast)) block(key0, slot * TILEB + kb * SUBB);
    }
    if (j + 2 < nt) ATTN_WAIT_VMCNT(2 * NLD);  // tile j+1 has landed; the loads of tile j+2 stay in flight
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
    slot = slot == NSLOT - 1 ? 0 : slot + 1;
  }

  store_transposed<NCB>(acc, p.scale, (char*)p.dq + qoff + (size_t)min(qrow, N - 1) * ROWB, h, qrow < N);
}

// =====================================================================================================
// dK and dV in one kernel (S and dP computed once for both).  The accumulators of both gradients
// (128 registers per 32 keys) beside the stationary K and V rows (64) leave no room for two waves
// per SIMD, so this kernel runs four waves of 32 keys, one per SIMD, with the whole register file;
// a workgroup owns 128 keys.
// With one wave per SIMD nothing else hides the vector work of a block behind matrix work, so the
// wave is software-pipelined: a step works on three 32-query blocks at once, the score products of
// block i+1, the exponentials and dS of block i, and the gradient products of block i-1.  The 32
// MFMAs of a step depend on none of its vector work.  Instruction order inside a step is fixed by
// hand (one MFMA per slot, operands requested two groups of four slots ahead, the vector work of
// one row per slot) and fenced slot by slot.  The ring has four slots because a step touches three
// tiles, and the loop is unrolled over them so that every LDS offset is an immediate.
// Every block of every tile is computed by every wave: a block that is invisible to the wave's keys
// (causal) or past the end (ragged) contributes exact zeros through the -inf scores and the +inf
// statistic of the padded workspace rows, and the slowest wave of the workgroup computes it anyway.
// =====================================================================================================
#ifndef ATTN_BWD_RA
#define ATTN_BWD_RA 8
#endif
template <int D_>
struct BwdPipe {
  static constexpr int D = D_, BN = 64, NWAVES = 4, BM = NWAVES * 32, NT = NWAVES * 64;
  static constexpr int NKK = D / 16, NCB = D / 32, ROWB = D * 2, NCH = ROWB / 16;
  static constexpr int TILEB = BN * ROWB, SUBB = 32 * ROWB, NSLOT = 4;
  static constexpr int T2BASE = NSLOT * TILEB;
  static constexpr int AUXBASE = 2 * NSLOT * TILEB;
  static constexpr int NLD = BN * NCH / NT;
  static constexpr int LDS_BYTES = AUXBASE + NSLOT * 512;
  static constexpr int NS = 2 * NKK;         // score products of a block: S and dP, NKK k-steps each
  static constexpr int NG = 4 * NCB;         // gradient products of a block: dV and dK, NCB column blocks x 2 k-steps
  static constexpr int NM = NS + NG;         // 32 (d = 128) or 16 (d = 64)
  static constexpr int RA = D == 128 ? ATTN_BWD_RA : 4;
  static_assert(NS == NG && RA % 4 == 0 && RA <= NS && NM % 4 == 0, "schedule shape");
  // slot p of a step: the first RA MFMAs are gradient products (their operands were requested by
  // the previous step, from a tile that is certainly resident), then score and gradient products
  // alternate, and the last RA are score products
  static constexpr bool is_score(int p) {
    if (p < RA) return false;
    const int q = p - RA, npairs = NS - RA;
    return q < 2 * npairs ? (q & 1) == 0 : true;
  }
  static constexpr int index(int p) {
    if (p < RA) return p;
    const int q = p - RA, npairs = NS - RA;
    if (q < 2 * npairs) return (q & 1) == 0 ? q / 2 : RA + q / 2;
    return npairs + (q - 2 * npairs);
  }
  // slot m requests the operand of slot read_target(m): two groups of four slots ahead, and inside
  // a group in the reverse of the order of use, so that the first product of a group waits for the
  // newest request of its batch and the other three need no wait instruction
  static constexpr int read_target(int m) { return (m / 4 + RA / 4) * 4 + 3 - m % 4; }
  static constexpr int VP0 = 6;                                                       // first slot with vector work
  static constexpr int vslot(int r) { return VP0 + (r * (NM - VP0)) / 16; }            // slot of row r's vector work
  static constexpr int aslot(int a) { return vslot(4 * a) - 6 > 0 ? vslot(4 * a) - 6 : 0; }  // slot that reads the statistics of rows 4a..4a+3
};

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, 1) attn_bwd_dkv_pipe_kernel(const AttnBwdParams p) {
  using C = BwdPipe<D>;
  constexpr int NKK = C::NKK, NCB = C::NCB, ROWB = C::ROWB, NCH = C::NCH, TILEB = C::TILEB, SUBB = C::SUBB, NSLOT = C::NSLOT;
  constexpr int NLD = C::NLD, NT = C::NT, BN = C::BN, BM = C::BM, NM = C::NM, RA = C::RA;

  __shared__ __attribute__((aligned(1024))) char smem_raw[C::LDS_BYTES];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int ki = lane & 31, h = lane >> 5;

  const int T128 = (p.N + BM - 1) / BM;
  AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hkv, p.Hkv, T128, CAUSAL ? 1 : 0);
  if (CAUSAL) tc.t = T128 - 1 - tc.t;  // key tile 0 is the heaviest: first
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  const int g = tc.hq;
  const int k0 = tc.t * BM;
  const int wk0 = k0 + w * 32;  // first key of this wave
  const int krow = wk0 + ki;

  const size_t koff = ((size_t)(tc.b * p.Hkv + g) * N) * ROWB;
  const int nqt_all = (N + BN - 1) / BN;
  const int qt0 = CAUSAL ? k0 / BN : 0;
  const int nt = G * (nqt_all - qt0);

  int ld_row[NLD];
  uint32_t ld_off[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCH, c = s % NCH;
    ld_row[it] = r;
    ld_off[it] = r * ROWB + ((c ^ swz_rt<ROWB>(r)) << 4);
  }
  const uint32_t lds_base = (uint32_t)(uintptr_t)smem;
  const uint32_t lds_wave = lds_base + w * 1024;
  // the next tile to request: query tile iss_qt of the current query head, whose Q, dO and
  // workspace rows start at iss_q, iss_do, iss_ws; after the last tile the next head begins
  int iss_qt = qt0;
  const size_t head_bytes = (size_t)N * ROWB;
  const char* iss_q = (const char*)p.q + (size_t)(tc.b * p.Hq + g * G) * head_bytes + (size_t)qt0 * TILEB;
  const char* iss_do = (const char*)p.dout + (size_t)(tc.b * p.Hq + g * G) * head_bytes + (size_t)qt0 * TILEB;
  const float* iss_ws = p.ws + (size_t)(tc.b * p.Hq + g * G) * 2 * p.Npad + (size_t)qt0 * BN;
  const uint32_t aoff = (uint32_t)(((lane & 15) * 4 + ((lane >> 4) & 1) * p.Npad) * 4);
  const bool ragged = (N % BN) != 0;
  auto issue_next = [&](int slot) __attribute__((always_inline)) {
    if (ragged && iss_qt == nqt_all - 1) {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const uint32_t over = (uint32_t)max(0, iss_qt * BN + ld_row[it] - (N - 1)) * ROWB;  // rows past N-1 re-read row N-1
        attn_lds_dma16(iss_q, ld_off[it] - over, lds_wave + slot * TILEB + it * NT * 16);
        attn_lds_dma16(iss_do, ld_off[it] - over, lds_wave + C::T2BASE + slot * TILEB + it * NT * 16);
      }
    } else {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        attn_lds_dma16(iss_q, ld_off[it], lds_wave + slot * TILEB + it * NT * 16);
        attn_lds_dma16(iss_do, ld_off[it], lds_wave + C::T2BASE + slot * TILEB + it * NT * 16);
      }
    }
    if (lane < 32) attn_lds_dma16(iss_ws, aoff, lds_base + C::AUXBASE + slot * 512);
    if (++iss_qt == nqt_all) {  // on to the next query head of the group
      iss_qt = qt0;
      iss_q += head_bytes - (size_t)(nqt_all - 1 - qt0) * TILEB;
      iss_do += head_bytes - (size_t)(nqt_all - 1 - qt0) * TILEB;
      iss_ws += 2 * (size_t)p.Npad - (size_t)(nqt_all - 1 - qt0) * BN;
    } else {
      iss_q += TILEB;
      iss_do += TILEB;
      iss_ws += BN;
    }
  };
  constexpr int LPT = 2 * NLD + 1;  // loads per thread and tile
  issue_next(0);

  bf16x8 kf[NKK], vf[NKK];
  {
    const int row = min(krow, N - 1);
    const char* ks = (const char*)p.k + koff + (size_t)row * ROWB + h * 16;
    const char* vs = (const char*)p.v + koff + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      kf[kk] = *(const bf16x8*)(ks + kk * 32);
      vf[kk] = *(const bf16x8*)(vs + kk * 32);
    }
  }
  if (nt > 1) issue_next(1);
  if (nt > 2) issue_next(2);

  f32x16 acc_dv[NCB], acc_dk[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_dv[cb][r] = acc_dk[cb][r] = 0.f;

  // LDS read addresses.  Inside the ring every offset (slot, 32-row half, 16-row group) is a
  // compile-time immediate of the read instruction; the second tensor's slots lie beyond the
  // immediate's range and get address registers of their own.
  uint32_t raddr[2][NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    raddr[0][kk] = ki * ROWB + (((2 * kk + h) ^ swz_rt<ROWB>(ki)) << 4);
    raddr[1][kk] = raddr[0][kk] + C::T2BASE;
  }
  uint32_t taddr[2][NCB][2];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int row = 8 * e + 4 * h + (s >> 2);
        const int chunk = cb * 4 + chalf * 2 + ((s & 3) >> 1);
        taddr[0][cb][e] = row * ROWB + ((chunk ^ swz_rt<ROWB>(row)) << 4) + ((s & 1) << 3);
        taddr[1][cb][e] = taddr[0][cb][e] + C::T2BASE;
      }
  }
  const uint32_t auxaddr = C::AUXBASE + 16 * h;
  // `t2` selects the tensor (0: Q slots, 1: dO slots), `off` is the block's offset inside them
  auto row_operand = [&](int t2, int off, int kk) __attribute__((always_inline)) { return *(LDS_AS u32x4*)(smem + raddr[t2][kk] + off); };
  auto tr_operand = [&](int t2, int off, int cb, int kc) __attribute__((always_inline)) {
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + taddr[t2][cb][0] + off + kc * 16 * ROWB));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + taddr[t2][cb][1] + off + kc * 16 * ROWB));
    s16x8 av;
    av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
    av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
    return __builtin_bit_cast(u32x4, av);
  };
  // operand of gradient product i of the block at `off`: dV^T += dO^T P (even i), dK^T += Q^T dS (odd i)
  auto grad_operand = [&](int off, int i) __attribute__((always_inline)) { return tr_operand((i & 1) ? 0 : 1, off, (i >> 1) % NCB, (i >> 1) / NCB); };
  // operand of score product i of the block at `off`: S += Q K^T (even i), dP += dO V^T (odd i)
  auto score_operand = [&](int off, int i) __attribute__((always_inline)) { return row_operand(i & 1, off, i >> 1); };
  auto grad_mfma = [&](int i, u32x4 o, const u32x4 (&pp)[2], const u32x4 (&pd)[2]) __attribute__((always_inline)) {
    const int cb = (i >> 1) % NCB, kc = (i >> 1) / NCB;
    if (i & 1) acc_dk[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o), __builtin_bit_cast(bf16x8, pd[kc]), acc_dk[cb], 0, 0, 0);
    else acc_dv[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o), __builtin_bit_cast(bf16x8, pp[kc]), acc_dv[cb], 0, 0, 0);
  };

  const float c = p.scale_log2;

  u32x4 pre[RA];  // operands of the next step's first RA MFMAs
  // One step.  (s_in, dp_in): finished scores of the block at CUR whose first query row is q0b;
  // (s_out, dp_out) <- scores of the block at NEXT; (pp_out, pd_out) <- P and dS of the block at
  // CUR; (pp_acc, pd_acc): P and dS of the block at PREV, multiplied into dV and dK.  PREV, CUR,
  // NEXT are compile-time offsets inside the ring, AUX the offset of CUR's statistics.
  auto step = [&](f32x16& s_in, f32x16& dp_in, f32x16& s_out, f32x16& dp_out, u32x4 (&pp_out)[2], u32x4 (&pd_out)[2],
                  const u32x4 (&pp_acc)[2], const u32x4 (&pd_acc)[2], auto PREV, auto CUR, auto NEXT, auto AUX,
                  int q0b) __attribute__((always_inline)) {
    constexpr int prev = decltype(PREV)::value, cur = decltype(CUR)::value, next = decltype(NEXT)::value, auxo = decltype(AUX)::value;
    u32x4 op[NM];
#pragma unroll
    for (int m = 0; m < RA; ++m) op[m] = pre[m];
    f32x4 l4[4], d4[4];
    float e_even = 0.f, f_even = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      // LDS reads: the operand of slot m + RA, and the statistics of the rows handled six slots on
      {
        const int t = C::read_target(m);
        if (t < NM) op[t] = C::is_score(t) ? score_operand(next, C::index(t)) : grad_operand(prev, C::index(t));
        else pre[t - NM] = grad_operand(cur, t - NM);
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
        if (C::aslot(a) == m) {
          l4[a] = *(const LDS_AS f32x4*)(smem + auxaddr + auxo + 32 * a);
          d4[a] = *(const LDS_AS f32x4*)(smem + auxaddr + auxo + 256 + 32 * a);
        }
      // the matrix product of this slot
      const int i = C::index(m);
      if (C::is_score(m)) {
        if (i == 0 || i == 1) {
#pragma unroll
          for (int r = 0; r < 16; ++r) (i ? dp_out : s_out)[r] = 0.f;
        }
        if (i & 1) dp_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), vf[i >> 1], dp_out, 0, 0, 0);
        else s_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, op[m]), kf[i >> 1], s_out, 0, 0, 0);
      } else {
        grad_mfma(i, op[m], pp_acc, pd_acc);
      }
      // causal diagonal: -inf scores for the queries before this lane's key (wave-uniform branch)
      if (CAUSAL && m == C::VP0 - 1 && q0b < wk0 + 31) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (q0b + 8 * (r >> 2) + 4 * h + (r & 3) < krow) s_in[r] = -INFINITY;
      }
      // vector work: P = exp2(s c - lse2), dS = P (dP - delta) for the rows of this slot
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (C::vslot(r) == m) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[r], c, -l4[r >> 2][r & 3]));
          const float f = e * (dp_in[r] - d4[r >> 2][r & 3]);
          if (r & 1) {
            pp_out[r >> 3][(r >> 1) & 3] = pack_bf16(e_even, e);
            pd_out[r >> 3][(r >> 1) & 3] = pack_bf16(f_even, f);
          } else {
            e_even = e;
            f_even = f;
          }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // the block "before the first" lives in the last half of slot 3: zeros, so that its gradient
  // products (with P = dS = 0) add exact zeros
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < SUBB / (NT * 16); ++i) {
      *(LDS_AS u32x4*)(smem + 3 * TILEB + SUBB + (i * NT + tid) * 16) = z;
      *(LDS_AS u32x4*)(smem + C::T2BASE + 3 * TILEB + SUBB + (i * NT + tid) * 16) = z;
    }
  }
  if (nt > 2) ATTN_WAIT_VMCNT(2 * LPT);
  else if (nt > 1) ATTN_WAIT_VMCNT(LPT);
  else ATTN_WAIT_VMCNT(0);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) asm volatile("" ::"v"(kf[kk]), "v"(vf[kk]));
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the zero fill is written
  attn_wg_barrier();

  // prologue: scores of block 0
  f32x16 sa, dpa, sb, dpb;
  u32x4 ppa[2], pda[2], ppb[2], pdb[2];
#pragma unroll
  for (int r = 0; r < 16; ++r) sa[r] = dpa[r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, row_operand(0, 0, kk)), kf[kk], sa, 0, 0, 0);
    dpa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, row_operand(1, 0, kk)), vf[kk], dpa, 0, 0, 0);
  }
#pragma unroll
  for (int t = 0; t < 2; ++t) ppb[t] = pdb[t] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int m = 0; m < RA; ++m) pre[m] = grad_operand(3 * TILEB + SUBB, m);

  int qt = qt0;
  // tile j lives in slot j % 4 = S
  auto tile = [&](auto S, int j) __attribute__((always_inline)) {
    constexpr int s = decltype(S)::value;
    constexpr int b0 = s * TILEB, b1 = b0 + SUBB, bp = ((s + 3) & 3) * TILEB + SUBB, bn = ((s + 1) & 3) * TILEB;
    const int q0b = qt * BN;
    step(sa, dpa, sb, dpb, ppa, pda, ppb, pdb, ic<bp>{}, ic<b0>{}, ic<b1>{}, ic<s * 512>{}, q0b);
    // tile j+1 has landed (the loads of tile j+2 stay in flight); every wave is done with tile j-1
    if (j + 2 < nt) ATTN_WAIT_VMCNT(LPT);
    else ATTN_WAIT_VMCNT(0);
    attn_wg_barrier();
    if (j + 3 < nt) issue_next((s + 3) & 3);
    step(sb, dpb, sa, dpa, ppb, pdb, ppa, pda, ic<b0>{}, ic<b1>{}, ic<bn>{}, ic<s * 512 + 128>{}, q0b + 32);
    if (++qt == nqt_all) qt = qt0;
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
  // epilogue: the gradient products of the last block (its first RA operands are already here)
  {
    const int last = ((nt - 1) & 3) * TILEB + SUBB;
#pragma unroll
    for (int i = RA; i < C::NG; ++i) grad_mfma(i, grad_operand(last, i), ppb, pdb);
#pragma unroll
    for (int i = 0; i < RA; ++i) grad_mfma(i, pre[i], ppb, pdb);
  }


  const size_t roff = koff + (size_t)min(krow, N - 1) * ROWB;
  store_transposed<NCB>(acc_dv, 1.0f, (char*)p.dv + roff, h, krow < N);
  store_transposed<NCB>(acc_dk, p.scale, (char*)p.dk + roff, h, krow < N);
}

}  // namespace

int attn_bwd_launch_bf16(const AttnBwdParams& p, int d, hipStream_t stream) {
  const int grid_q = p.B * p.Hq * p.T;
  const int grid_f = p.B * p.Hkv * ((p.N + 127) / 128);
  auto launch = [&](auto dtag) {
    constexpr int D = decltype(dtag)::value;
    if (p.causal) {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<D, true>), dim3(grid_q), dim3(512), 0, stream, p);
      hipLaunchKernelGGL((attn_bwd_dkv_pipe_kernel<D, true>), dim3(grid_f), dim3(256), 0, stream, p);
    } else {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<D, false>), dim3(grid_q), dim3(512), 0, stream, p);
      hipLaunchKernelGGL((attn_bwd_dkv_pipe_kernel<D, false>), dim3(grid_f), dim3(256), 0, stream, p);
    }
  };
  if (d == 128) launch(ic<128>{});
  else if (d == 64) launch(ic<64>{});
  else return -1;
  return (int)hipGetLastError();
}
