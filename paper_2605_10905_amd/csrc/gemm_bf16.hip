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

#include "attn_device.h"
#include "gemm_kernels.h"
#include "gemm_map.h"

namespace {

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

template <int BK, int NSTAGE>
struct GemmCfg {
  static constexpr int BM = 256, BN = 256, NT = 256, NWAVES = 4;
  static constexpr int ROWB = BK * 2, NCH = ROWB / 16;
  static constexpr int TILEB = 256 * ROWB;          // one operand tile
  static constexpr int STAGEB = 2 * TILEB;          // A tile then B tile
  static constexpr int NLD = 256 * NCH / NT;        // direct-to-LDS loads per thread, tile and stage
  static constexpr int NKK = BK / 16;
  static constexpr int LDS_BYTES = NSTAGE * STAGEB;
  static_assert(LDS_BYTES <= 160 * 1024, "ring does not fit the LDS");
  static_assert((NSTAGE - 2) * 2 * NLD <= 63, "vmcnt field");
  static_assert(NSTAGE >= 3 && (BK / 16) % 2 == 0, "pipeline shape");
};

template <int BK, int NSTAGE>
__global__ void __launch_bounds__(256, 1) gemm_bf16_nt_kernel(const GemmParams p) {
  using C = GemmCfg<BK, NSTAGE>;
  constexpr int ROWB = C::ROWB, NCH = C::NCH, TILEB = C::TILEB, STAGEB = C::STAGEB, NLD = C::NLD, NKK = C::NKK;

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
  uint32_t a_off[NLD], b_off[NLD];
#pragma unroll
  for (int it = 0; it < NLD; ++it) {
    const int s = it * C::NT + tid;
    const int r = s / NCH, c = (s % NCH) ^ attn_swz_k<ROWB>(r);
    a_off[it] = (uint32_t)(min(m0 + r, M - 1) - m0) * (uint32_t)rowbytes + c * 16;
    b_off[it] = (uint32_t)(min(n0 + r, N - 1) - n0) * (uint32_t)rowbytes + c * 16;
  }
  const char* const a_tile = (const char*)p.a + (size_t)m0 * rowbytes;
  const char* const b_tile = (const char*)p.b + (size_t)n0 * rowbytes;
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + w * 1024;
  auto issue_stage = [&](int ks, int slot) __attribute__((always_inline)) {
    const char* const ab = a_tile + (size_t)ks * ROWB;
    const char* const bb = b_tile + (size_t)ks * ROWB;
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      attn_lds_dma16(ab, a_off[it], lds_wave + slot * STAGEB + it * C::NT * 16);
      attn_lds_dma16(bb, b_off[it], lds_wave + slot * STAGEB + TILEB + it * C::NT * 16);
    }
  };

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nk) issue_stage(s, s);

  // ---- consumer role: fragment addresses inside a stage (row block 0 of this wave's quarter)
  uint32_t ra[NKK], rb[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    const int rowa = wm * 128 + li, rowb = wn * 128 + li;
    ra[kk] = rowa * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(rowa)) << 4);
    rb[kk] = TILEB + rowb * ROWB + (((2 * kk + h) ^ attn_swz_k<ROWB>(rowb)) << 4);
  }

  f32x16 acc[4][4];  // [n block][m block]: rows of the accumulator are n, its column is m
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][mb][r] = 0.f;

  // Software pipeline inside the wave (it is alone on its SIMD): the fragments of k-step kk+1 are
  // read while the 16 MFMAs of k-step kk run; the stage boundary (wait, barrier, refill of the
  // slot that was consumed one stage ago, first fragments of the next stage) sits in front of the
  // MFMAs of a stage's last k-step, so the matrix pipe has 16 MFMAs queued across it.
  bf16x8 fa[2][4], fb[2][4];
  auto read_frags = [&](int buf, int base, int kk) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[buf][i] = *(LDS_AS bf16x8*)(smem + ra[kk] + base + i * 32 * ROWB);
      fb[buf][i] = *(LDS_AS bf16x8*)(smem + rb[kk] + base + i * 32 * ROWB);
    }
  };
  auto mfma16 = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][nb], fa[buf][mb], acc[nb][mb], 0, 0, 0);
  };
  // 8 LDS reads spread over 16 MFMAs
  auto interleave = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
  };

  if (NSTAGE - 2 < nk) ATTN_WAIT_VMCNT((NSTAGE - 2) * 2 * NLD);
  else ATTN_WAIT_VMCNT(0);
  attn_wg_barrier();
  read_frags(0, 0, 0);

  int slot = 0;
  for (int ks = 0; ks < nk; ++ks) {
    const int base = slot * STAGEB;
    const int nslot = slot == NSTAGE - 1 ? 0 : slot + 1;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < NKK) {
        read_frags(nxt, base, kk + 1);
      } else if (ks + 1 < nk) {
        // stage ks+1 has landed once at most the NSTAGE-3 stages after it are outstanding
        if (ks + NSTAGE - 2 < nk) ATTN_WAIT_VMCNT((NSTAGE - 3) * 2 * NLD);
        else ATTN_WAIT_VMCNT(0);
        attn_wg_barrier();
        // every wave has finished stage ks-1: refill its slot
        if (ks + NSTAGE - 1 < nk) issue_stage(ks + NSTAGE - 1, slot == 0 ? NSTAGE - 1 : slot - 1);
        read_frags(nxt, nslot * STAGEB, 0);
      }
      mfma16(cur);
      interleave();
    }
    slot = nslot;
  }

  // ---- epilogue: lane (li, h) holds, for row m, the columns n = 32 nb + 8 a + 4 h + (0..3) ---------
  const bool vec_ok = (N & 7) == 0;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const int m = m0 + wm * 128 + mb * 32 + li;
    __bf16* const crow = (__bf16*)p.c + (size_t)min(m, M - 1) * N;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
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
        const int n = n0 + wn * 128 + nb * 32 + a * 16 + h * 8;  // this lane's 8 consecutive columns
        if (m < M) {
          if (vec_ok && n + 8 <= N) {
            u32x4 out = {x[0], x[1], y[0], y[1]};
            *(u32x4*)(crow + n) = out;
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
int launch(const GemmParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_bf16_nt_kernel<BK, NSTAGE>), dim3(p.tiles_m * p.tiles_n), dim3(256), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

const GemmVariant* gemm_bf16_nt_variants(int* count) {
  static const GemmVariant table[] = {
      {"bf16 nt 256x256x32 ring4", 256, 256, 32, launch<32, 4>},
      {"bf16 nt 256x256x32 ring5", 256, 256, 32, launch<32, 5>},
      {"bf16 nt 256x256x32 ring3", 256, 256, 32, launch<32, 3>},
  };
  *count = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
