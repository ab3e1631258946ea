// bf16 GEMM for gfx950:  C[M,N] = A[M,K] * B[N,K]^T, fp32 accumulation, bf16 output.
//
// The paper's GEMM (section 6.1, GEMM paragraph; section 6.3 and appendix A for the MI350
// shapes) is a producer/consumer pipeline: loader roles stage operand tiles in swizzled shared
// memory through a ring of buffers, tensor-core roles consume them.  The gfx950 form kept here:
//
//   * a workgroup of 4 waves owns a 256 x 256 tile of C, each wave a 128 x 128 quarter: 16
//     accumulators of the 32x32x16 MFMA = 256 registers, which the MFMA reads and writes in
//     place (one wave per SIMD, the whole 512-register file).  Every operand fragment read from
//     LDS feeds four MFMAs, half the LDS bytes per MFMA of a 2-waves-per-SIMD tiling;
//   * operand tiles (256 rows x BK of A and of B) travel HBM/L2 -> LDS by direct-to-LDS loads
//     into a ring of NSTAGE slots, NSTAGE-1 stages ahead, one workgroup barrier per stage.  Every
//     wave issues its share of the loads itself: on CDNA a wave that only loads would idle a
//     SIMD, and the loads cost one issue slot each;
//   * the product is taken transposed (MFMA A operand = rows of B, B operand = rows of A), so a
//     lane owns one row m of C and, after one exchange between the lane halves, writes 8
//     consecutive n with one 16-byte store;
//   * 16-byte chunks of a tile row are XOR-swizzled so that the 16 lanes the LDS serves together
//     hit 16 different bank groups;
//   * tiles are ordered for L2 reuse inside an XCD (gemm_map.h).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_device.h"
#include "gemm_kernels.h"
#include "gemm_map.h"

// One 16-byte piece of C: plain, or non-temporal when the launch streams C (GemmParams::stream_c).
// (Written as an assembly statement: the compiler merges a plain and a non-temporal store behind a
// run-time condition into one plain store.  It is the kernel's last memory operation.)
#define GEMM_STORE_C(val, ptr)                                                                          \
  do {                                                                                                  \
    if (p.stream_c) asm volatile("global_store_dwordx4 %0, %1, off nt" ::"v"(ptr), "v"(val) : "memory"); \
    else *(ptr) = (val);                                                                                \
  } while (0)

namespace {

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

// WM x WN 32x32 blocks per wave, 2 x 2 waves: the workgroup tile is 64 WM x 64 WN.
template <int WM, int WN, int BK, int NSTAGE>
struct GemmCfg {
  static constexpr int BM = 64 * WM, BN = 64 * WN, NT = 256;
  static constexpr int ROWB = BK * 2, NCH = ROWB / 16;
  static constexpr int TILEA = BM * ROWB, TILEB_ = BN * ROWB;
  static constexpr int STAGEB = TILEA + TILEB_;  // A tile then B tile
  static constexpr int NLDA = BM * NCH / NT, NLDB = BN * NCH / NT;  // direct-to-LDS loads per thread and stage
  static constexpr int LPS = NLDA + NLDB;
  static constexpr int NKK = BK / 16;
  static constexpr int LPP = LPS / NKK;  // loads issued per k-step
  static constexpr int LDS_BYTES = NSTAGE * STAGEB;
  static_assert(LDS_BYTES <= 160 * 1024, "ring does not fit the LDS");
  static_assert((NSTAGE - 1) * LPS <= 63, "vmcnt field");
  static_assert(NSTAGE >= 2 && NKK % 2 == 0 && LPS % NKK == 0 && NLDA >= 1 && NLDB >= 1, "pipeline shape");
};

// BKN: the second operand is stored [K, N] (row-major, N contiguous) instead of [N, K].  Its tile is
// then BK rows of BN columns in LDS, and the MFMA operand that needs 8 consecutive k per lane is
// gathered with the transposing LDS read, exactly as the attention kernels read V.
template <int WM, int WN, int BK, int NSTAGE, int MINW, bool BKN>
__global__ void __launch_bounds__(256, MINW) gemm_bf16_kernel(const GemmParams p) {
  using C = GemmCfg<WM, WN, BK, NSTAGE>;
  constexpr int ROWBB = C::BN * 2, NCHB = ROWBB / 16;  // [K,N] layout: bytes and 16-byte chunks per tile row
  constexpr int ROWB = C::ROWB, NCH = C::NCH, TILEA = C::TILEA, STAGEB = C::STAGEB, NKK = C::NKK;
  constexpr int NLDA = C::NLDA, NLDB = C::NLDB, LPS = C::LPS, LPP = C::LPP;

  __shared__ __attribute__((aligned(1024))) char smem_raw[C::LDS_BYTES];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int li = lane & 31, h = lane >> 5;
  const int wm = w >> 1, wn = w & 1;

  const GemmTileCoord tc = gemm_tile_coord_impl(blockIdx.x, p.tiles_m, p.tiles_n);
  const int m0 = tc.tm * C::BM, n0 = tc.tn * C::BN;
  const int M = p.M, N = p.N, K = p.K;
  const size_t rowbytes = (size_t)K * 2;

  // ---- producer role: chunk s = it * 256 + tid of a tile is (row s / NCH, LDS chunk s % NCH) and
  // holds the row's chunk (s % NCH) ^ swizzle(row); rows past the matrix re-read its last row
  uint32_t g_off[LPS];
#pragma unroll
  for (int it = 0; it < LPS; ++it) {
    const bool is_a = it < NLDA;
    const int s = (is_a ? it : it - NLDA) * C::NT + tid;
    if (is_a || !BKN) {
      const int r = s / NCH, c = (s % NCH) ^ attn_swz_k<ROWB>(r);
      const int row = is_a ? min(m0 + r, M - 1) - m0 : min(n0 + r, N - 1) - n0;
      g_off[it] = (uint32_t)row * (uint32_t)rowbytes + c * 16;
    } else {
      // [K,N] tile: k row r, LDS chunk s % NCHB holds the row's chunk XOR ((r & 3) << 2) (rows that the
      // transposing read takes together land in different 64-byte groups); columns past N re-read
      // the row's last 8 (N is a multiple of 8)
      const int r = s / NCHB, c = (s % NCHB) ^ ((r & 3) << 2);
      const int col = min(n0 + c * 8, N - 8) - n0;
      g_off[it] = (uint32_t)r * (uint32_t)(N * 2) + col * 2;
    }
  }
  const char* const a_tile = (const char*)p.a + (size_t)m0 * rowbytes;
  const char* const b_tile = BKN ? (const char*)p.b + (size_t)n0 * 2 : (const char*)p.b + (size_t)n0 * rowbytes;
  const size_t b_step = BKN ? (size_t)BK * N * 2 : (size_t)ROWB;  // bytes between consecutive k-stages of the second operand
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  // load `it` (0 .. LPS-1) of k-stage ks into ring slot `slot`
  auto issue_load = [&](int ks, int slot, int it) __attribute__((always_inline)) {
    if (it < NLDA) attn_lds_dma16(a_tile + (size_t)ks * ROWB, g_off[it], lds_wave + slot * STAGEB + it * C::NT * 16);
    else attn_lds_dma16(b_tile + (size_t)ks * b_step, g_off[it], lds_wave + slot * STAGEB + TILEA + (it - NLDA) * C::NT * 16);
  };

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s)
    if (s < nk) {
#pragma unroll
      for (int it = 0; it < LPS; ++it) issue_load(s, s, it);
    }

  // ---- consumer role: fragment addresses inside a stage (row block 0 of this wave's quarter)
  uint32_t ra[NKK], rb[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    const int rowa = wm * 32 * WM + li, rowb = wn * 32 * WN + li;
    ra[kk] = rowa * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(rowa)) << 4);
    rb[kk] = TILEA + rowb * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(rowb)) << 4);
  }
  // [K,N] layout: in a group of 16 lanes, lane s reads four columns of k row s / 4 and the hardware
  // hands lane t the four k of column t; read e of a fragment takes k = 8 h + 4 e + (0..3) of the k-step
  uint32_t tb[WN][2];
  {
    const int s16 = lane & 15, chalf = (lane >> 4) & 1;
#pragma unroll
    for (int nb = 0; nb < WN; ++nb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int krow = 8 * h + 4 * e + (s16 >> 2);
        const int chunk = (wn * 32 * WN + nb * 32) / 8 + chalf * 2 + ((s16 & 3) >> 1);
        tb[nb][e] = TILEA + krow * ROWBB + ((chunk ^ ((krow & 3) << 2)) << 4) + ((s16 & 1) << 3);
      }
  }

  f32x16 acc[WN][WM];  // [n block][m block]: rows of the accumulator are n, its column is m
#pragma unroll
  for (int nb = 0; nb < WN; ++nb)
#pragma unroll
    for (int mb = 0; mb < WM; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][mb][r] = 0.f;

  // Software pipeline inside the wave: the fragments of k-step kk+1 are read while the MFMAs of
  // k-step kk run.  The stage boundary (all fragments of stage ks are in registers: wait for
  // stage ks+1, barrier, first fragments of stage ks+1) sits in front of the MFMAs of a stage's
  // last k-step, so the matrix pipe has work queued across it; the slot of stage ks is free from
  // that barrier on and is refilled with stage ks+NSTAGE, LPP loads per k-step, over the k-steps
  // up to the next barrier.
  bf16x8 fa[2][WM], fb[2][WN];
  auto read_frags = [&](int buf, int base, int kk) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < WM; ++i) fa[buf][i] = *(LDS_AS bf16x8*)(smem + ra[kk] + base + i * 32 * ROWB);
    if constexpr (!BKN) {
#pragma unroll
      for (int i = 0; i < WN; ++i) fb[buf][i] = *(LDS_AS bf16x8*)(smem + rb[kk] + base + i * 32 * ROWB);
    } else {
#pragma unroll
      for (int i = 0; i < WN; ++i) {
        const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + tb[i][0] + base + kk * 16 * ROWBB));
        const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + tb[i][1] + base + kk * 16 * ROWBB));
        s16x8 av;
        av[0] = v0[0]; av[1] = v0[1]; av[2] = v0[2]; av[3] = v0[3];
        av[4] = v1[0]; av[5] = v1[1]; av[6] = v1[2]; av[7] = v1[3];
        fb[buf][i] = __builtin_bit_cast(bf16x8, av);
      }
    }
  };
  auto mfmas = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < WN; ++nb)
#pragma unroll
      for (int mb = 0; mb < WM; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][nb], fa[buf][mb], acc[nb][mb], 0, 0, 0);
  };
  // spread the WM + WN LDS reads of a k-step over its WM * WN MFMAs
  auto interleave = [&]() __attribute__((always_inline)) {
    constexpr int NR = WM + (BKN ? 2 * WN : WN), NM = WM * WN;
    constexpr int PER = NM / NR > 0 ? NM / NR : 1;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
    }
  };

  if (NSTAGE <= nk) ATTN_WAIT_VMCNT((NSTAGE - 1) * LPS);
  else ATTN_WAIT_VMCNT(0);
  attn_wg_barrier();
  read_frags(0, 0, 0);

  // one k-stage; STEADY: every load and the next stage exist (no checks)
  auto stage = [&](int ks, int slot, auto steady) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady)::value;
    const int base = slot * STAGEB;
    const int nslot = slot == NSTAGE - 1 ? 0 : slot + 1;
    const int pslot = slot == 0 ? NSTAGE - 1 : slot - 1;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < NKK) {
        read_frags(nxt, base, kk + 1);
        if (STEADY || (ks >= 1 && ks - 1 + NSTAGE < nk)) {
#pragma unroll
          for (int i = 0; i < LPP; ++i) issue_load(ks - 1 + NSTAGE, pslot, (kk + 1) * LPP + i);
        }
      } else if (STEADY || ks + 1 < nk) {
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's reads of the slot about to be refilled are done
        if (STEADY || ks + NSTAGE - 1 < nk) ATTN_WAIT_VMCNT((NSTAGE - 2) * LPS);
        else ATTN_WAIT_VMCNT(0);
        attn_wg_barrier();
        read_frags(nxt, nslot * STAGEB, 0);
        if (STEADY || ks + NSTAGE < nk) {
#pragma unroll
          for (int i = 0; i < LPP; ++i) issue_load(ks + NSTAGE, slot, i);
        }
      }
      mfmas(cur);
      interleave();
    }
  };

  int slot = 0, ks = 0;
  if (nk > 0) {
    stage(0, 0, std::false_type{});
    ks = 1;
    slot = NSTAGE > 1 ? 1 : 0;
  }
  for (; ks + NSTAGE < nk; ++ks) {
    stage(ks, slot, std::true_type{});
    slot = slot == NSTAGE - 1 ? 0 : slot + 1;
  }
  for (; ks < nk; ++ks) {
    stage(ks, slot, std::false_type{});
    slot = slot == NSTAGE - 1 ? 0 : slot + 1;
  }

  // ---- epilogue: lane (li, h) holds, for row m, the columns n = 32 nb + 8 a + 4 h + (0..3) ---------
  const bool vec_ok = (N & 7) == 0;
#pragma unroll
  for (int mb = 0; mb < WM; ++mb) {
    const int m = m0 + wm * 32 * WM + mb * 32 + li;
    __bf16* const crow = (__bf16*)p.c + (size_t)min(m, M - 1) * N;
#pragma unroll
    for (int nb = 0; nb < WN; ++nb)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        uint32_t x[2], y[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const uint32_t tx = pack_bf16(acc[nb][mb][(2 * a) * 4 + 2 * r], acc[nb][mb][(2 * a) * 4 + 2 * r + 1]);
          const uint32_t ty = pack_bf16(acc[nb][mb][(2 * a + 1) * 4 + 2 * r], acc[nb][mb][(2 * a + 1) * 4 + 2 * r + 1]);
          auto sw = __builtin_amdgcn_permlane32_swap(tx, ty, false, false);
          x[r] = sw[0];
          y[r] = sw[1];
        }
        const int n = n0 + wn * 32 * WN + nb * 32 + a * 16 + h * 8;  // this lane's 8 consecutive columns
        if (m < M) {
          if (vec_ok && n + 8 <= N) {
            u32x4 out = {x[0], x[1], y[0], y[1]};
            GEMM_STORE_C(out, (u32x4*)(crow + n));
          } else {
            const uint32_t v[4] = {x[0], x[1], y[0], y[1]};
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n + e < N) ((uint16_t*)crow)[n + e] = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
          }
        }
      }
  }
}


// The 256 x 256 tile on the 16x16x32 MFMA: each wave's 128 x 128 quarter is 8 x 8 blocks of 16 x 16
// (64 accumulators of 4 registers), a k-step is 32 wide, a fragment (16 rows x 32 k: 16 bytes per
// lane, lane (j, g) = row j, k 8g .. 8g+7) feeds eight MFMAs.  Same ring, same barrier placement.
typedef __attribute__((ext_vector_type(4))) float f32x4;

// SPLITK: the grid holds p.splits workgroups per tile; workgroup (split, tile) contracts its slice
// of k and stores the fp32 accumulators to p.partial instead of rounding them into c.
template <int BK, int NSTAGE, bool SPLITK>
__global__ void __launch_bounds__(256, 1) gemm_bf16_nt_m16_kernel(const GemmParams p) {
  using C = GemmCfg<4, 4, BK, NSTAGE>;
  constexpr int ROWB = C::ROWB, NCH = C::NCH, TILEA = C::TILEA, STAGEB = C::STAGEB;
  constexpr int NLDA = C::NLDA, LPS = C::LPS;
  constexpr int NPH = BK / 32;       // k-steps per stage
  constexpr int LPP = LPS / NPH;     // loads issued per k-step
  static_assert(BK % 32 == 0 && LPS % NPH == 0, "k-step of 32");

  __shared__ __attribute__((aligned(1024))) char smem_raw[C::LDS_BYTES];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int lj = lane & 15, g = lane >> 4;
  const int wm = w >> 1, wn = w & 1;

  const int ntile = p.tiles_m * p.tiles_n;
  const int split = SPLITK ? (int)blockIdx.x / ntile : 0;
  const GemmTileCoord tc = gemm_tile_coord_impl(SPLITK ? (int)blockIdx.x - split * ntile : (int)blockIdx.x, p.tiles_m, p.tiles_n);
  const int m0 = tc.tm * C::BM, n0 = tc.tn * C::BN;
  const int M = p.M, N = p.N, K = p.K;
  const size_t rowbytes = (size_t)K * 2;
  const int kbeg = SPLITK ? split * p.klen : 0;            // this workgroup's slice of k
  const int kcnt = SPLITK ? min(p.klen, K - kbeg) : K;

  uint32_t g_off[LPS];
#pragma unroll
  for (int it = 0; it < LPS; ++it) {
    const bool is_a = it < NLDA;
    const int s = (is_a ? it : it - NLDA) * C::NT + tid;
    const int r = s / NCH, c = (s % NCH) ^ attn_swz_k<ROWB>(r);
    const int row = is_a ? min(m0 + r, M - 1) - m0 : min(n0 + r, N - 1) - n0;
    g_off[it] = (uint32_t)row * (uint32_t)rowbytes + c * 16;
  }
  const char* const a_tile = (const char*)p.a + (size_t)m0 * rowbytes + (size_t)kbeg * 2;
  const char* const b_tile = (const char*)p.b + (size_t)n0 * rowbytes + (size_t)kbeg * 2;
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_load = [&](int ks, int slot, int it) __attribute__((always_inline)) {
    if (it < NLDA) attn_lds_dma16(a_tile + (size_t)ks * ROWB, g_off[it], lds_wave + slot * STAGEB + it * C::NT * 16);
    else attn_lds_dma16(b_tile + (size_t)ks * ROWB, g_off[it], lds_wave + slot * STAGEB + TILEA + (it - NLDA) * C::NT * 16);
  };

  const int nk = kcnt / BK;
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s)
    if (s < nk) {
#pragma unroll
      for (int it = 0; it < LPS; ++it) issue_load(s, s, it);
    }

  // fragment addresses: row block 0 of this wave's quarter, k-step ph
  uint32_t ra[NPH], rb[NPH];
#pragma unroll
  for (int ph = 0; ph < NPH; ++ph) {
    const int rowa = wm * 128 + lj, rowb = wn * 128 + lj;
    ra[ph] = rowa * ROWB + (((4 * ph + g) ^ attn_swz_k<ROWB>(rowa)) << 4);
    rb[ph] = TILEA + rowb * ROWB + (((4 * ph + g) ^ attn_swz_k<ROWB>(rowb)) << 4);
  }

  f32x4 acc[8][8];  // [n block][m block]: rows of the accumulator are n (4 g + r), its column is m (lj)
#pragma unroll
  for (int nb = 0; nb < 8; ++nb)
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[nb][mb][r] = 0.f;

  bf16x8 fa[2][8], fb[2][8];
  auto read_frags = [&](int buf, int base, int ph) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) fa[buf][i] = *(LDS_AS bf16x8*)(smem + ra[ph] + base + i * 16 * ROWB);
#pragma unroll
    for (int i = 0; i < 8; ++i) fb[buf][i] = *(LDS_AS bf16x8*)(smem + rb[ph] + base + i * 16 * ROWB);
  };
  auto mfmas = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
#pragma unroll
      for (int mb = 0; mb < 8; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[buf][nb], fa[buf][mb], acc[nb][mb], 0, 0, 0);
  };
  auto interleave = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
  };

  if (NSTAGE <= nk) ATTN_WAIT_VMCNT((NSTAGE - 1) * LPS);
  else ATTN_WAIT_VMCNT(0);
  attn_wg_barrier();
  read_frags(0, 0, 0);

  // one k-stage; PAR: which fragment buffer its first k-step uses (stages of one k-step alternate)
  auto stage = [&](int ks, int slot, auto steady, auto par) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady)::value;
    constexpr int PAR = decltype(par)::value;
    const int base = slot * STAGEB;
    const int nslot = slot == NSTAGE - 1 ? 0 : slot + 1;
    const int pslot = slot == 0 ? NSTAGE - 1 : slot - 1;
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph) {
      const int cur = (PAR + ph) & 1, nxt = cur ^ 1;
      if (ph + 1 < NPH) {
        read_frags(nxt, base, ph + 1);
        if (STEADY || (ks >= 1 && ks - 1 + NSTAGE < nk)) {
#pragma unroll
          for (int i = 0; i < LPP; ++i) issue_load(ks - 1 + NSTAGE, pslot, (ph + 1) * LPP + i);
        }
      } else if (STEADY || ks + 1 < nk) {
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's reads of the slot about to be refilled are done
        if (STEADY || ks + NSTAGE - 1 < nk) ATTN_WAIT_VMCNT((NSTAGE - 2) * LPS);
        else ATTN_WAIT_VMCNT(0);
        attn_wg_barrier();
        read_frags(nxt, nslot * STAGEB, 0);
        if (STEADY || ks + NSTAGE < nk) {
#pragma unroll
          for (int i = 0; i < LPP; ++i) issue_load(ks + NSTAGE, slot, i);
        }
      }
      mfmas(cur);
      interleave();
    }
  };

  // stages of one k-step alternate between the two fragment buffers: they are run in pairs (the host
  // only picks this kernel when the number of stages is even)
  int slot = 0, ks = 0;
  auto advance = [&]() __attribute__((always_inline)) {
    slot = slot == NSTAGE - 1 ? 0 : slot + 1;
    ++ks;
  };
  auto step = [&](auto steady) __attribute__((always_inline)) {
    stage(ks, slot, steady, std::integral_constant<int, 0>{});
    advance();
    if (NPH & 1) {
      stage(ks, slot, steady, std::integral_constant<int, 1>{});
      advance();
    }
  };
  constexpr int PER_STEP = (NPH & 1) ? 2 : 1;
  if (nk > 0) step(std::false_type{});
  while (ks + PER_STEP - 1 + NSTAGE < nk) step(std::true_type{});
  while (ks < nk) step(std::false_type{});

  // ---- epilogue: lane (lj, g) holds, for row m, the columns n = 16 nb + 4 g + (0..3); a pair of
  // neighbouring n blocks is exchanged between odd and even lane groups so that every lane owns 8
  // consecutive columns: one 16-byte store each
  if (SPLITK) {
    // fp32 partial tile: every lane owns 4 consecutive columns of row m, one 16-byte store
    const bool vec4 = (N & 3) == 0;
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) {
      const int m = m0 + wm * 128 + mb * 16 + lj;
      float* const prow = p.partial + ((size_t)split * M + (size_t)min(m, M - 1)) * N;
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        const int n = n0 + wn * 128 + nb * 16 + 4 * g;
        if (m < M) {
          if (vec4 && n + 4 <= N) {
            *(f32x4*)(prow + n) = acc[nb][mb];
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < N) prow[n + e] = acc[nb][mb][e];
          }
        }
      }
    }
    return;
  }
  const bool vec_ok = (N & 7) == 0;
#pragma unroll
  for (int mb = 0; mb < 8; ++mb) {
    const int m = m0 + wm * 128 + mb * 16 + lj;
    __bf16* const crow = (__bf16*)p.c + (size_t)min(m, M - 1) * N;
#pragma unroll
    for (int nb = 0; nb < 8; nb += 2) {
      uint32_t x[2], y[2];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const uint32_t tx = pack_bf16(acc[nb][mb][2 * r], acc[nb][mb][2 * r + 1]);
        const uint32_t ty = pack_bf16(acc[nb + 1][mb][2 * r], acc[nb + 1][mb][2 * r + 1]);
        auto sw = __builtin_amdgcn_permlane16_swap(tx, ty, false, false);
        x[r] = sw[0];
        y[r] = sw[1];
      }
      // even lane groups: own block nb, columns 4g .. 4g+7; odd ones: block nb+1, columns 4(g-1) .. 4(g-1)+7
      const int n = n0 + wn * 128 + (nb + (g & 1)) * 16 + 4 * (g & ~1);
      if (m < M) {
        if (vec_ok && n + 8 <= N) {
          u32x4 out = {x[0], x[1], y[0], y[1]};
          GEMM_STORE_C(out, (u32x4*)(crow + n));
        } else {
          const uint32_t v[4] = {x[0], x[1], y[0], y[1]};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (n + e < N) ((uint16_t*)crow)[n + e] = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
        }
      }
    }
  }
}

template <int BK, int NSTAGE>
int launch_m16(const GemmParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_bf16_nt_m16_kernel<BK, NSTAGE, false>), dim3(p.tiles_m * p.tiles_n), dim3(256), 0, stream, p);
  return (int)hipGetLastError();
}

// c[i] = bf16(sum over splits of partial[s][i]), splits added in index order; 8 elements per thread
__global__ void __launch_bounds__(256) gemm_splitk_sum_kernel(const float* __restrict__ partial, void* c, size_t total, int splits) {
  const size_t i8 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i8 >= total) return;
  if ((total & 7) == 0) {
    f32x4 lo = *(const f32x4*)(partial + i8), hi = *(const f32x4*)(partial + i8 + 4);
    for (int s = 1; s < splits; ++s) {
      lo += *(const f32x4*)(partial + (size_t)s * total + i8);
      hi += *(const f32x4*)(partial + (size_t)s * total + i8 + 4);
    }
    u32x4 out = {pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])};
    *(u32x4*)((__bf16*)c + i8) = out;
  } else {
    for (size_t i = i8; i < i8 + 8 && i < total; ++i) {
      float v = partial[i];
      for (int s = 1; s < splits; ++s) v += partial[(size_t)s * total + i];
      ((__bf16*)c)[i] = (__bf16)v;
    }
  }
}

template <int WM, int WN, int BK, int NSTAGE, int MINW, bool BKN = false>
int launch(const GemmParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, BK, NSTAGE, MINW, BKN>), dim3(p.tiles_m * p.tiles_n), dim3(256), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

int gemm_bf16_nt_splitk_launch(const GemmParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_bf16_nt_m16_kernel<32, 4, true>), dim3(p.tiles_m * p.tiles_n * p.splits), dim3(256), 0, stream, p);
  const size_t total = (size_t)p.M * p.N;
  hipLaunchKernelGGL(gemm_splitk_sum_kernel, dim3((unsigned)((total + 2047) / 2048)), dim3(256), 0, stream, p.partial, p.c, total, p.splits);
  return (int)hipGetLastError();
}

const GemmVariant* gemm_bf16_nt_variants(int* count) {
  static const GemmVariant table[] = {
      {"bf16 nt 256x256x32 ring4", 256, 256, 32, 32, launch<4, 4, 32, 4, 1>},
      {"bf16 nt 256x256x64 ring2", 256, 256, 64, 64, launch<4, 4, 64, 2, 1>},
      {"bf16 nt 128x128x64 ring2", 128, 128, 64, 64, launch<2, 2, 64, 2, 2>},
      {"bf16 nt 128x128x64 ring4", 128, 128, 64, 64, launch<2, 2, 64, 4, 1>},
      {"bf16 nt 64x64x64 ring2", 64, 64, 64, 64, launch<1, 1, 64, 2, 4>},
      {"bf16 nt 64x64x32 ring4", 64, 64, 32, 32, launch<1, 1, 32, 4, 4>},
      {"bf16 nt 256x256x32 ring4 mfma16x16x32", 256, 256, 32, 64, launch_m16<32, 4>},
      {"bf16 nt 256x256x64 ring2 mfma16x16x32", 256, 256, 64, 64, launch_m16<64, 2>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}

const GemmVariant* gemm_bf16_nn_variants(int* count) {
  static const GemmVariant table[] = {
      {"bf16 nn 256x256x32 ring4", 256, 256, 32, 32, launch<4, 4, 32, 4, 1, true>},
      {"bf16 nn 128x128x32 ring4", 128, 128, 32, 32, launch<2, 2, 32, 4, 2, true>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
