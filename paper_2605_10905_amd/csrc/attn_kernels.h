// Internal interface between the C-ABI entry points and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "tile_map.h"

struct AttnParams {
  const void* q;
  const void* k;
  const void* v;
  void* o;
  float* lse;
  int B, Hq, Hkv, N;
  int T;             // query tiles per head = ceil(N / BM)
  int causal;
  float scale_log2;  // scale * log2(e) (times q_descale*k_descale for fp8)
  float out_scale;   // multiplies O in the epilogue (v_descale and P scaling for fp8; 1 for bf16)
  int* queue = nullptr;  // persistent launch only: 8 tile-list counters, 32 ints apart
  int total = 0;         // persistent launch only: number of query tiles = B * Hq * T
  AttnTileMap map;       // attn_tile_map_make(B, Hq, Hkv, T, causal): workgroup id -> (batch, head, tile)
};

// persistent bf16 forward (d = 64 or 128): `workgroups` resident workgroups drain the tile queue
int attn_fwd_bf16_persistent_launch(const AttnParams& p, int d, int workgroups, hipStream_t stream);

// backward pass (bf16, head dimension 128 or 64)
struct AttnBwdParams {
  const void* q;
  const void* k;
  const void* v;
  const void* o;
  const void* dout;
  const float* lse;
  void* dq;
  void* dk;
  void* dv;
  float* ws;         // [B, Hq, 2, Npad] floats: lse * log2(e) and delta, rows padded to whole 64-row tiles
  int B, Hq, Hkv, N;
  int T;             // 256-row tiles per head = ceil(N / 256)
  int Npad;          // ceil(N / 64) * 64
  int causal;
  float scale_log2;  // scale * log2(e)
  float scale;
};
int attn_bwd_launch_bf16(const AttnBwdParams& p, int d, hipStream_t stream);  // d = 128 or 64

struct AttnVariant {
  const char* name;
  int dtype;   // attn_dtype
  int d;       // head dim
  int bm;      // query rows per workgroup
  int bn;      // keys per streamed K/V tile
  int threads; // workgroup size
  int lds;     // dynamic LDS bytes
  // launches the kernel for `grid` workgroups on `stream`; returns the hipError_t as int
  int (*launch)(const AttnParams& p, int grid, hipStream_t stream);
};

// Variant tables, defined by the kernel translation units (host functions).
const AttnVariant* attn_sp_variants(int* count);   // pipelined kernel: bf16 d = 128 / 64, fp8 d = 128 (the defaults)
const AttnVariant* attn_fp8_variants(int* count);  // all products on the fp8 matrix path, P as two e4m3 terms
