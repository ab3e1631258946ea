// Fused attention forward, bf16 inputs, fp32 accumulate, for gfx950 (MI355X).
//
// What is computed: paper section 6.1 (score computation, masking,
// normalisation, output accumulation) with the streaming-softmax state and the
// two outputs of appendix C.3 (acc / l and m + log l).
//
// How it maps to CDNA4 (this is not the paper's NVIDIA design):
//   * One workgroup owns one query tile of BM = NWAVES*QB*32 rows; each wave owns
//     QB blocks of 32 query rows for the whole kernel and keeps their Q operand,
//     their running max / sum and their fp32 output accumulator in registers.
//   * The products are computed TRANSPOSED on 32x32x16 bf16 MFMA:
//         S^T[key][query] = K . Q^T          O^T[c][query] += V^T . P^T
//     so a lane holds ONE query (column) and many keys (rows).  Row max and row
//     sum are then in-lane reductions plus a single exchange between lane l and
//     lane l^32, the rescale factor is one scalar per lane, and the fp32 S^T
//     accumulator registers, once exponentiated and packed to bf16, ARE the
//     P^T operand of the second MFMA: no cross-lane shuffle, no LDS round trip.
//   * K and V tiles stream HBM/L2 -> LDS with direct-to-LDS 128-bit loads (no
//     register staging) into a two-stage ring; the load of tile j+1 is issued
//     before tile j is consumed (the producer role), and one workgroup barrier per
//     tile is both the "full" signal of stage j+1 and the "empty" signal of
//     stage j (paper sections 3.2 and 4.1: producer/consumer hand-off through
//     full/empty barriers with stage = j mod 2).
//   * K rows are read from LDS as 128-bit MFMA operands; V is read with the
//     gfx950 transposing LDS load (ds_read_b64_tr_b16), which delivers the
//     key-contiguous operand the second MFMA needs from a row-major V tile.
//     Both tiles are XOR-swizzled at 16-byte granularity against bank conflicts;
//     the swizzle is applied on the global-address side of the direct-to-LDS load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_kernels.h"
#include "tile_map.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

__device__ __forceinline__ constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x >> 1); }

// Swizzles: 16-byte chunk index within a row is XORed with a function of the row.
// K (read as 16 keys x one 16-byte chunk per 16 lanes): the XOR term must take 16
// (or 8) different values over 16 consecutive rows -> rotate-left of the row bits.
template <int ROWB>
__device__ __forceinline__ constexpr int swz_k(int row) {
  constexpr int NCH = ROWB / 16, BITS = ilog2(NCH), RP = 256 / ROWB;
  const int a = (row / RP) & (NCH - 1);
  return ((a << 1) | (a >> (BITS - 1))) & (NCH - 1);
}
// V (transposing read: 16 lanes cover 4 consecutive rows x 32 bytes): consecutive
// rows must land in different 64-byte groups.
template <int ROWB>
__device__ __forceinline__ constexpr int swz_v(int row) {
  constexpr int NCH = ROWB / 16, RP = 256 / ROWB;
  return ((row / RP) & (NCH / 4 - 1)) << 2;
}

// max over lane l and lane l^32 (the two lanes that hold the same query)
__device__ __forceinline__ float max_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, int BN, int NWAVES, int QB, bool CAUSAL>
__global__ void __launch_bounds__(NWAVES * 64, NWAVES / 4) attn_fwd_bf16_kernel(const AttnParams p) {
  constexpr int BM = NWAVES * QB * 32;
  constexpr int NT = NWAVES * 64;
  constexpr int NKB = BN / 32;      // 32-key blocks per K/V tile (S^T row blocks)
  constexpr int NKK = D / 16;       // MFMA k-steps over the head dimension
  constexpr int NKC = BN / 16;      // 16-key chunks (k-steps of the second product)
  constexpr int NCB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;       // bytes per K/V row
  constexpr int NCH = ROWB / 16;    // 16-byte chunks per row
  constexpr int TILEB = BN * ROWB;  // bytes per K (or V) tile
  constexpr int STAGEB = 2 * TILEB; // K tile then V tile
  constexpr int NLD = BN * NCH / NT;  // direct-to-LDS loads per thread per tile per tensor
  static_assert(BN * NCH % NT == 0, "tile must divide evenly over the workgroup");
  static_assert(STAGEB + (NKB - 1) * 32 * ROWB < 65536, "LDS immediates must fit 16 bits");

  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63;
  const int qi = lane & 31;  // query column within a 32-query block
  const int h = lane >> 5;   // which half of the k-slots / accumulator rows this lane holds

  const AttnTileCoord tc = attn_tile_coord_impl(blockIdx.x, p.B, p.Hq, p.Hkv, p.T, CAUSAL ? 1 : 0);
  const int N = p.N;
  const int G = p.Hq / p.Hkv;
  const int hk = tc.hq / G;
  const int q0 = tc.t * BM;                 // first query row of the workgroup
  const int wq0 = q0 + w * QB * 32;         // first query row of this wave

  const char* const qhead = (const char*)p.q + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  const char* const khead = (const char*)p.k + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;
  const char* const vhead = (const char*)p.v + ((size_t)(tc.b * p.Hkv + hk) * N) * ROWB;

  // number of K/V tiles this workgroup visits
  const int kv_end = CAUSAL ? min(N, q0 + BM) : N;
  const int nt = (kv_end + BN - 1) / BN;

  // ---- producer role: per-thread constants of the direct-to-LDS tile loads ----------
  // LDS slot s (16-byte units) of a tile holds row s/NCH, chunk (s%NCH)^swizzle(row).
  int ld_row[NLD];
  uint32_t ld_koff[NLD], ld_voff[NLD];  // byte offsets inside an (unclamped) tile
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * NT + tid;
    const int r = s / NCH, c = s % NCH;
    ld_row[it] = r;
    ld_koff[it] = r * ROWB + ((c ^ swz_k<ROWB>(r)) << 4);
    ld_voff[it] = r * ROWB + ((c ^ swz_v<ROWB>(r)) << 4);
  }
  auto issue_tile_loads = [&](int j, int st) __attribute__((always_inline)) {
    LDS_AS char* const kdst = smem + st * STAGEB + w * 1024;
    LDS_AS char* const vdst = kdst + TILEB;
    const char* const kt = khead + (size_t)j * TILEB;
    const char* const vt = vhead + (size_t)j * TILEB;
    if ((j + 1) * BN <= N) {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(kt + ld_koff[it]), (LDS_AS void*)(kdst + it * NT * 16), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(vt + ld_voff[it]), (LDS_AS void*)(vdst + it * NT * 16), 16, 0, 0);
      }
    } else {
      // ragged last tile: rows past N-1 re-read row N-1 (finite data; masked out later)
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const int over = max(0, j * BN + ld_row[it] - (N - 1));
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(kt + ld_koff[it] - (size_t)over * ROWB), (LDS_AS void*)(kdst + it * NT * 16), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(vt + ld_voff[it] - (size_t)over * ROWB), (LDS_AS void*)(vdst + it * NT * 16), 16, 0, 0);
      }
    }
  };

  issue_tile_loads(0, 0);

  // ---- Q operand (B operand of S^T = K Q^T): lane (qi,h) holds Q[row][16kk+8h .. +7] ----
  bf16x8 qf[QB][NKK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = min(wq0 + qb * 32 + qi, N - 1);
    const char* src = qhead + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[qb][kk] = *(const bf16x8*)(src + kk * 32);
  }

  // ---- LDS read addresses (per lane, stage 0, key block 0) ------------------------
  // K operand: lane (qi,h) reads key row qi, chunk 2kk+h of each 32-key block.
  uint32_t kaddr[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = qi * ROWB + (((2 * kk + h) ^ swz_k<ROWB>(qi)) << 4);
  // V operand through the transposing load: in a group of 16 lanes, lane s reads the
  // four columns 4*(s%4).. of key row s/4; the hardware hands lane t the four keys
  // of column t.  Lane l therefore addresses key 4h + (l%16)/4 (+8 for the second
  // half of the k-slots) and columns 32cb + 16*((l/16)%2) + 4*(l%4).
  uint32_t vaddr[NCB][2];
  {
    const int s = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int key = 8 * e + 4 * h + (s >> 2);
        const int chunk = cb * 4 + chalf * 2 + ((s & 3) >> 1);
        vaddr[cb][e] = TILEB + key * ROWB + ((chunk ^ swz_v<ROWB>(key)) << 4) + ((s & 1) << 3);
      }
  }

  // ---- streaming-softmax state (appendix C.3: m = -inf, acc = 0; l starts at 0 here,
  //      which is equivalent because the first rescale factor is exp(-inf) = 0) -------
  f32x16 oacc[QB][NCB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qb][cb][r] = 0.f;
  }
  const float c = p.scale_log2;

  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): tile 0 and Q have landed
  __syncthreads();

  // ---- one K/V tile: scores, mask, streaming softmax, output accumulation ----------
  auto consume_tile = [&](int j, int st, bool masked) __attribute__((always_inline)) {
    LDS_AS char* const sb = smem + st * STAGEB;
    // S^T = K Q^T
    f32x16 s[QB][NKB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8 a = *(LDS_AS bf16x8*)(sb + kaddr[kk] + kb * 32 * ROWB);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][kk], s[qb][kb], 0, 0, 0);
      }

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (masked) {
        // key visible iff key <= limit; limit folds the causal rule and the ragged end of K
        const int qrow = wq0 + qb * 32 + qi;
        const int limit = CAUSAL ? min(qrow, N - 1) : (N - 1);
        const int key0 = j * BN + 4 * h;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kb * 32 + 8 * (r >> 2) + (r & 3);
            if (key > limit) s[qb][kb][r] = -INFINITY;
          }
      }
      // row max over this tile (in-lane, then across the two lanes of the query)
      float mx = s[qb][0][0];
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qb][kb][r]);
      mx = max_halves(mx);
      const float m_new = fmaxf(m_run[qb], mx * c);
      const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
      m_run[qb] = m_new;
      // P^T = exp2(c*S^T - m): packed to bf16 in place
      float lsum = 0.f;
      bf16x2 pk[NKB][8];
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][kb][2 * r], c, -m_new));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][kb][2 * r + 1], c, -m_new));
          bf16x2 t;
          t[0] = (__bf16)p0;
          t[1] = (__bf16)p1;
          pk[kb][r] = t;
          // the row sum is taken in fp32 from the unrounded values: summing the bf16-rounded
          // ones (one dot2 per pair) is cheaper but moves lse by up to ~1e-3 on rows whose
          // weight sits on two or three keys
          lsum += p0 + p1;
        }
      l_run[qb] = l_run[qb] * alpha + lsum;
      // rescale the accumulator only if some row's max moved
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) oacc[qb][cb] *= alpha;
      }
      // O^T += V^T P^T
#pragma unroll
      for (int kc = 0; kc < NKC; ++kc) {
        u32x4 bu;
#pragma unroll
        for (int r = 0; r < 4; ++r) bu[r] = __builtin_bit_cast(uint32_t, pk[kc >> 1][(kc & 1) * 4 + r]);
        const bf16x8 bop = __builtin_bit_cast(bf16x8, bu);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(sb + vaddr[cb][0] + kc * 16 * ROWB));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(sb + vaddr[cb][1] + kc * 16 * ROWB));
          s16x8 av;
          av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
          av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
          oacc[qb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), bop, oacc[qb][cb], 0, 0, 0);
        }
      }
    }
  };

  auto tile_step = [&](int j, int st) __attribute__((always_inline)) {
    if (j + 1 < nt) issue_tile_loads(j + 1, st ^ 1);
    const int key_lo = j * BN, key_hi = j * BN + BN - 1;
    const bool skip = CAUSAL && key_lo > wq0 + QB * 32 - 1;  // every key of the tile is masked for this wave
    if (!skip) {
      const bool masked = (CAUSAL && key_hi > wq0) || key_hi >= N;
      if (masked) consume_tile(j, st, true);
      else consume_tile(j, st, false);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's share of tile j+1 has landed
    __syncthreads();                     // stage st^1 full for everyone, stage st empty
  };

  for (int j = 0; j < nt; j += 2) {
    tile_step(j, 0);
    if (j + 1 < nt) tile_step(j + 1, 1);
  }

  // ---- epilogue: O = acc / l (bf16), lse = (m + log2 l) * ln 2 -----------------------
  char* const ohead = (char*)p.o + ((size_t)(tc.b * p.Hq + tc.hq) * N) * ROWB;
  float* const lsehead = p.lse + (size_t)(tc.b * p.Hq + tc.hq) * N;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = wq0 + qb * 32 + qi;
    const float l = sum_halves(l_run[qb]);
    const float inv = p.out_scale / l;
    if (row < N && h == 0) lsehead[row] = (m_run[qb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    // lane (qi,h) holds O^T rows c = 32cb + 8b + 4h + r (b=0..3, r=0..3).  Exchange with the
    // other half so that every lane owns 8 consecutive c: 32cb + 16a + 8h + (0..7).
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        uint32_t x[2], y[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          bf16x2 tx, ty;
          tx[0] = (__bf16)(oacc[qb][cb][(2 * a) * 4 + 2 * r] * inv);
          tx[1] = (__bf16)(oacc[qb][cb][(2 * a) * 4 + 2 * r + 1] * inv);
          ty[0] = (__bf16)(oacc[qb][cb][(2 * a + 1) * 4 + 2 * r] * inv);
          ty[1] = (__bf16)(oacc[qb][cb][(2 * a + 1) * 4 + 2 * r + 1] * inv);
          auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, tx), __builtin_bit_cast(uint32_t, ty), false, false);
          x[r] = sw[0];
          y[r] = sw[1];
        }
        if (row < N) {
          u32x4 out = {x[0], x[1], y[0], y[1]};
          *(u32x4*)(ohead + (size_t)row * ROWB + (cb * 32 + a * 16 + h * 8) * 2) = out;
        }
      }
  }
}

template <int D, int BN, int NWAVES, int QB>
int launch_bf16(const AttnParams& p, int grid, hipStream_t stream) {
  constexpr int lds = 2 * 2 * BN * D * 2;
  auto kc = attn_fwd_bf16_kernel<D, BN, NWAVES, QB, true>;
  auto kn = attn_fwd_bf16_kernel<D, BN, NWAVES, QB, false>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kc, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)kn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  if (p.causal) hipLaunchKernelGGL(kc, dim3(grid), dim3(NWAVES * 64), lds, stream, p);
  else hipLaunchKernelGGL(kn, dim3(grid), dim3(NWAVES * 64), lds, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

#define VARIANT(D, BN, NW, QB) \
  { "bf16 d" #D " BM" #NW "x" #QB "x32 BN" #BN, 0, D, NW * QB * 32, BN, NW * 64, 2 * 2 * BN * D * 2, launch_bf16<D, BN, NW, QB> }

const AttnVariant* attn_bf16_variants(int* count) {
  static const AttnVariant table[] = {
      VARIANT(128, 64, 8, 1),
      VARIANT(128, 64, 4, 2),
      VARIANT(128, 64, 4, 1),
      VARIANT(64, 64, 8, 1),
      VARIANT(64, 64, 4, 1),
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
