// Measurement aid, not part of any attention or GEMM path: a loop of bf16 32x32x16 MFMAs in the
// launch shape of the attention forward kernel (one workgroup of eight waves per CU, two waves per
// SIMD), to which the other ingredients of that kernel can be added one by one, so that the
// benchmark can report what the board sustains under its power limit
//   pattern 0: on zero operands (nothing toggles),
//   pattern 1: on pseudo-random bf16 operands held in registers,
//   pattern 2: with the A operand of every MFMA read from LDS (1 KB per wave and MFMA, half of them
//              through the transposing read): the forward kernel's LDS traffic,
//   pattern 3: with, in addition, one exponential, two multiply-adds, one add and half a bf16 pack
//              per MFMA and lane, the results feeding later B operands: its vector work.
// No global memory traffic inside the loop.  Every wave keeps 8 independent accumulators.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/attn.h"
#include "attn_device.h"

namespace {

constexpr int kProbeWorkgroups = 256, kProbeThreads = 512, kProbeMfmaPerIter = 32;
constexpr int kProbeLds = 65536;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// two bf16 per word: random sign and mantissa, magnitude in [2^-4, 1)
__device__ __forceinline__ uint32_t probe_two_bf16(uint32_t r) {
  const uint32_t lo = ((r & 1) << 15) | ((123 + ((r >> 1) & 3)) << 7) | ((r >> 3) & 127);
  const uint32_t hi = (((r >> 10) & 1) << 15) | ((123 + ((r >> 11) & 3)) << 7) | ((r >> 13) & 127);
  return lo | (hi << 16);
}
__device__ __forceinline__ uint32_t probe_pack(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a;
  t[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, t);
}

template <bool ZERO, bool LDS, bool VALU>
__global__ void __launch_bounds__(kProbeThreads, 2) mfma_probe_kernel(int iters, float* sink) {
  __shared__ __attribute__((aligned(1024))) char smem_raw[kProbeLds];
  LDS_AS char* const smem = (LDS_AS char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63;
  const uint32_t gid = blockIdx.x * kProbeThreads + tid;
  if (LDS) {
    for (int i = tid; i < kProbeLds / 4; i += kProbeThreads) ((LDS_AS uint32_t*)smem)[i] = probe_two_bf16(probe_hash(gid * 977 + i));
    __syncthreads();
  }
  u32x4 a[4], b[8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) a[i][e] = ZERO ? 0u : probe_two_bf16(probe_hash(gid * 64 + i * 8 + e));
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) b[i][e] = ZERO ? 0u : probe_two_bf16(probe_hash(gid * 64 + 1032 + i * 8 + e));
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  float x[16], lsum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) x[r] = (float)(probe_hash(gid + r * 7919) & 1023) * (1.f / 512.f) - 1.f;
  const float c = 1.2f, mref = 0.3f;
  const uint32_t lrow = (uint32_t)lane * 16;  // 1 KB per wave, every bank once
  const uint32_t ltr = (uint32_t)((lane & 15) >> 2) * 256 + (lane >> 4) * 32 + (lane & 3) * 8;
  for (int it = 0; it < iters; ++it) {
    const uint32_t roff = (it & 1) ? 32768u : 0u;
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m) {
      u32x4 av;
      if (LDS) {
        if (m & 1) {
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + roff + ltr + (m >> 1) * 1024));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(smem + roff + ltr + (m >> 1) * 1024 + 16384));
          s16x8 t;
          t[0] = v0[0]; t[1] = v0[1]; t[2] = v0[2]; t[3] = v0[3];
          t[4] = v1[0]; t[5] = v1[1]; t[6] = v1[2]; t[7] = v1[3];
          av = __builtin_bit_cast(u32x4, t);
        } else {
          av = *(LDS_AS u32x4*)(smem + roff + lrow + (m >> 1) * 1024);
        }
      } else {
        av = a[m & 3];
      }
      acc[m & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, b[(m + (m >> 3)) & 7]), acc[m & 7], 0, 0, 0);
      if (VALU) {
        const int r = m & 15;
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x[r], c, -mref));
        lsum += e;
        x[r] = __builtin_fmaf(x[r], 0.999f, 0.0005f);
        if (r & 1) b[(m >> 1) & 7][(m >> 4) & 3] = probe_pack(e, lsum * 1e-3f);
      }
    }
  }
  float s = lsum;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[gid] = s;
}

}  // namespace

extern "C" {

int attn_mfma_probe(int iters, int pattern, float* sink, void* stream) {
  if (!sink) return ATTN_ERR_NULL;
  if (iters < 0 || iters > (1 << 24) || pattern < 0 || pattern > 3) return ATTN_ERR_SHAPE;
  const dim3 grid(kProbeWorkgroups), block(kProbeThreads);
  hipStream_t st = (hipStream_t)stream;
  if (pattern == 0) hipLaunchKernelGGL((mfma_probe_kernel<true, false, false>), grid, block, 0, st, iters, sink);
  else if (pattern == 1) hipLaunchKernelGGL((mfma_probe_kernel<false, false, false>), grid, block, 0, st, iters, sink);
  else if (pattern == 2) hipLaunchKernelGGL((mfma_probe_kernel<false, true, false>), grid, block, 0, st, iters, sink);
  else hipLaunchKernelGGL((mfma_probe_kernel<false, true, true>), grid, block, 0, st, iters, sink);
  return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int attn_mfma_probe_sink_floats(void) { return kProbeWorkgroups * kProbeThreads; }

double attn_mfma_probe_flops(int iters) {
  return (double)iters * kProbeMfmaPerIter * (2.0 * 32 * 32 * 16) * (kProbeWorkgroups * (kProbeThreads / 64));
}
}
