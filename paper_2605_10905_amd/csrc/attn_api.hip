// C-ABI entry points: argument validation, variant choice, launch.  See include/attn.h.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/attn.h"
#include "attn_kernels.h"
#include "tile_map.h"

constexpr long long kScratchBytes = 32ll << 20;
// A plain static device array: the compiler keeps a static device variable that host code names
// and makes it visible to the runtime under its mangled name.  (With __attribute__((used)) added
// the runtime could no longer find it: hipGetSymbolAddress aborted the process.)
static __device__ __align__(256) unsigned char scratch[kScratchBytes];  // see scratch_on_current_device()

namespace {

constexpr int kVersion = 1;
constexpr float kLog2e = 1.4426950408889634f;

// all variant tables, concatenated; the first match for (dtype, d) is the default
typedef const AttnVariant* (*VariantTable)(int*);
const VariantTable kTables[] = {attn_sp_variants, attn_fp8_variants};

const AttnVariant* variant_at(int i) {
  if (i < 0) return nullptr;
  for (VariantTable tab : kTables) {
    int n = 0;
    const AttnVariant* t = tab(&n);
    if (i < n) return &t[i];
    i -= n;
  }
  return nullptr;
}
int total_variants() {
  int total = 0;
  for (VariantTable tab : kTables) {
    int n = 0;
    tab(&n);
    total += n;
  }
  return total;
}

bool misaligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

int validate(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d,
             float scale, int dtype) {
  if (!q || !k || !v || !o || !lse) return ATTN_ERR_NULL;
  if (dtype != ATTN_BF16 && dtype != ATTN_FP8_E4M3) return ATTN_ERR_DTYPE;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || d <= 0) return ATTN_ERR_SHAPE;
  if (Hq % Hkv != 0) return ATTN_ERR_SHAPE;
  if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(o, 16) || misaligned(lse, 4)) return ATTN_ERR_SHAPE;
  if (d != 128 && !(d == 64 && dtype == ATTN_BF16)) return ATTN_ERR_UNSUPPORTED;  // fp8 inputs: d = 128 only
  // the kernels take the row maximum of the raw products and scale it afterwards,
  // which needs a positive factor; NaN and +inf pass through (garbage in, garbage out)
  if (scale <= 0.0f) return ATTN_ERR_UNSUPPORTED;
  // element offsets inside one head are 32-bit in the kernels
  if ((long long)N * d * 2 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  return ATTN_OK;
}

// Default choice: the first listed variant for (dtype, d).  The smaller query tiles of the first
// kernel do not pay even when the launch leaves CUs idle: the pipelined kernel on half the chip
// still beats them (e.g. 128 workgroups at N = 8192: 160 against 228 microseconds).
int choose_variant(int dtype, int B, int Hq, int N, int d) {
  (void)B; (void)Hq; (void)N;
  for (int i = 0; i < total_variants(); ++i) {
    const AttnVariant* a = variant_at(i);
    if (a->dtype == dtype && a->d == d) return i;
  }
  return -1;
}

int run(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d, int causal,
        float scale, int dtype, float qk_descale, float v_descale, int variant, void* stream) {
  int st = validate(q, k, v, o, lse, B, Hq, Hkv, N, d, scale, dtype);
  if (st != ATTN_OK) return st;
  if (variant < 0) variant = choose_variant(dtype, B, Hq, N, d);
  const AttnVariant* a = variant_at(variant);
  if (!a || a->dtype != dtype || a->d != d) return ATTN_ERR_UNSUPPORTED;
  AttnParams p;
  p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N;
  p.T = (N + a->bm - 1) / a->bm;
  p.causal = causal ? 1 : 0;
  p.scale_log2 = scale * qk_descale * kLog2e;
  p.out_scale = v_descale;
  p.map = attn_tile_map_make(B, Hq, Hkv, p.T, p.causal);
  const long long grid = (long long)B * Hq * p.T;
  if (grid <= 0 || grid > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  const int err = a->launch(p, (int)grid, (hipStream_t)stream);
  return err == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int bwd_validate(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse, void* dq, void* dk,
                 void* dv, int B, int Hq, int Hkv, int N, int d, float scale, int dtype) {
  if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv) return ATTN_ERR_NULL;
  if (dtype != ATTN_BF16 && dtype != ATTN_FP8_E4M3) return ATTN_ERR_DTYPE;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || d <= 0 || Hq % Hkv != 0) return ATTN_ERR_SHAPE;
  const void* const ptrs[] = {q, k, v, o, dout, dq, dk, dv};
  for (const void* ptr : ptrs)
    if (misaligned(ptr, 16)) return ATTN_ERR_SHAPE;
  if (misaligned(lse, 4)) return ATTN_ERR_SHAPE;
  if (dtype != ATTN_BF16 || (d != 128 && d != 64)) return ATTN_ERR_UNSUPPORTED;
  if (scale <= 0.0f) return ATTN_ERR_UNSUPPORTED;
  if ((long long)N * d * 2 >= (1ll << 31)) return ATTN_ERR_UNSUPPORTED;
  if ((long long)B * Hq * ((N + 255) / 256) > 0x7fffffffll) return ATTN_ERR_UNSUPPORTED;
  return ATTN_OK;
}

int bwd_run(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse, void* dq, void* dk,
            void* dv, float* workspace, int B, int Hq, int Hkv, int N, int d, int causal, float scale, void* stream) {
  AttnBwdParams p;
  p.q = q; p.k = k; p.v = v; p.o = o; p.dout = dout; p.lse = lse;
  p.dq = dq; p.dk = dk; p.dv = dv; p.ws = workspace;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N;
  p.T = (N + 255) / 256;
  p.Npad = (N + 63) / 64 * 64;
  p.causal = causal ? 1 : 0;
  p.scale_log2 = scale * kLog2e;
  p.scale = scale;
  return attn_bwd_launch_bf16(p, d, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

// Scratch memory of attn_bwd_noalloc: the per-row statistics the backward kernels pass from the
// query-side kernel to the key-side kernel, in a device array that is part of the loaded code
// object (every GPU the library runs on holds its own copy until the process ends).  In host
// code the array's name is only a handle: its device address is looked up once per device with
// that device current, and only that address is ever handed to a kernel.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices];  // zero-initialised: not looked up yet

float* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = (float*)ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

long long attn_bwd_workspace_bytes(int B, int Hq, int N);

int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d, int causal,
             float scale, int dtype, void* stream) {
  return run(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, dtype, 1.0f, 1.0f, -1, stream);
}

int attn_fwd_fp8(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d, int causal,
                 float scale, float q_descale, float k_descale, float v_descale, void* stream) {
  if (!(q_descale > 0.0f) || !(k_descale > 0.0f)) return ATTN_ERR_UNSUPPORTED;
  return run(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, ATTN_FP8_E4M3, q_descale * k_descale, v_descale, -1, stream);
}

int attn_fwd_variant(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d,
                     int causal, float scale, int dtype, int variant, void* stream) {
  if (variant < 0 || variant >= total_variants()) {
    int st = validate(q, k, v, o, lse, B, Hq, Hkv, N, d, scale, dtype);
    return st != ATTN_OK ? st : ATTN_ERR_UNSUPPORTED;
  }
  return run(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, dtype, 1.0f, 1.0f, variant, stream);
}

int attn_fwd_fp8_variant(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d,
                         int causal, float scale, float q_descale, float k_descale, float v_descale, int variant, void* stream) {
  if (!(q_descale > 0.0f) || !(k_descale > 0.0f)) return ATTN_ERR_UNSUPPORTED;
  if (variant < 0 || variant >= total_variants()) {
    int st = validate(q, k, v, o, lse, B, Hq, Hkv, N, d, scale, ATTN_FP8_E4M3);
    return st != ATTN_OK ? st : ATTN_ERR_UNSUPPORTED;
  }
  return run(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, ATTN_FP8_E4M3, q_descale * k_descale, v_descale, variant, stream);
}

int attn_fwd_persistent(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int N, int d,
                        int causal, float scale, int dtype, void* queue, void* stream) {
  int st = validate(q, k, v, o, lse, B, Hq, Hkv, N, d, scale, dtype);
  if (st != ATTN_OK) return st;
  if (!queue) return ATTN_ERR_NULL;
  if (misaligned(queue, 128)) return ATTN_ERR_SHAPE;
  if (dtype != ATTN_BF16) return ATTN_ERR_UNSUPPORTED;
  AttnParams p;
  p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N;
  p.T = (N + 255) / 256;
  p.causal = causal ? 1 : 0;
  p.scale_log2 = scale * kLog2e;
  p.out_scale = 1.0f;
  p.map = attn_tile_map_make(B, Hq, Hkv, p.T, p.causal);
  const long long total = (long long)B * Hq * p.T;
  if (total > 0x0fffffffll) return ATTN_ERR_UNSUPPORTED;
  p.queue = (int*)queue;
  p.total = (int)total;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return ATTN_ERR_LAUNCH;
  return attn_fwd_bf16_persistent_launch(p, d, cus, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int attn_persistent_queue_bytes(void) { return 8 * 32 * (int)sizeof(int); }

int attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse, void* dq, void* dk,
             void* dv, float* workspace, int B, int Hq, int Hkv, int N, int d, int causal, float scale, int dtype, void* stream) {
  const int st = bwd_validate(q, k, v, o, dout, lse, dq, dk, dv, B, Hq, Hkv, N, d, scale, dtype);
  if (st != ATTN_OK) return st;
  if (!workspace) return ATTN_ERR_NULL;
  if (misaligned(workspace, 16)) return ATTN_ERR_SHAPE;
  return bwd_run(q, k, v, o, dout, lse, dq, dk, dv, workspace, B, Hq, Hkv, N, d, causal, scale, stream);
}

int attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse, void* dq,
                     void* dk, void* dv, int B, int Hq, int Hkv, int N, int d, int causal, float scale, int dtype, void* stream) {
  const int st = bwd_validate(q, k, v, o, dout, lse, dq, dk, dv, B, Hq, Hkv, N, d, scale, dtype);
  if (st != ATTN_OK) return st;
  if (attn_bwd_workspace_bytes(B, Hq, N) > kScratchBytes) return ATTN_ERR_TOO_LARGE;
  float* const ws = scratch_on_current_device();
  if (!ws) return ATTN_ERR_LAUNCH;
  return bwd_run(q, k, v, o, dout, lse, dq, dk, dv, ws, B, Hq, Hkv, N, d, causal, scale, stream);
}

long long attn_bwd_noalloc_max_workspace_bytes(void) { return kScratchBytes; }

long long attn_bwd_workspace_bytes(int B, int Hq, int N) {
  if (B <= 0 || Hq <= 0 || N <= 0) return 0;
  return (long long)B * Hq * 2 * ((N + 63) / 64 * 64) * (long long)sizeof(float);
}

int attn_default_variant(int dtype, int B, int Hq, int N, int d) {
  if (B <= 0 || Hq <= 0 || N <= 0) return -1;
  return choose_variant(dtype, B, Hq, N, d);
}

int attn_num_variants(void) { return total_variants(); }

const char* attn_variant_name(int variant) {
  const AttnVariant* a = variant_at(variant);
  return a ? a->name : nullptr;
}

int attn_variant_bm(int variant) {
  const AttnVariant* a = variant_at(variant);
  return a ? a->bm : 0;
}

int attn_num_workgroups(int B, int Hq, int N, int BM) {
  if (B <= 0 || Hq <= 0 || N <= 0 || BM <= 0) return 0;
  const long long g = (long long)B * Hq * ((N + BM - 1) / BM);
  return g > 0x7fffffffll ? 0 : (int)g;
}

int attn_tile_coord(int wg, int B, int Hq, int Hkv, int N, int BM, int causal, int* b, int* hq, int* t) {
  if (!b || !hq || !t) return ATTN_ERR_NULL;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || BM <= 0 || Hq % Hkv != 0) return ATTN_ERR_SHAPE;
  const int T = (N + BM - 1) / BM;
  if (wg < 0 || (long long)wg >= (long long)B * Hq * T) return ATTN_ERR_SHAPE;
  const AttnTileCoord c = attn_tile_coord_impl(wg, B, Hq, Hkv, T, causal ? 1 : 0);
  *b = c.b; *hq = c.hq; *t = c.t;
  return ATTN_OK;
}

const char* attn_status_string(int status) {
  switch (status) {
    case ATTN_OK: return "ok";
    case ATTN_ERR_NULL: return "null pointer";
    case ATTN_ERR_SHAPE: return "bad shape or alignment";
    case ATTN_ERR_DTYPE: return "unknown dtype";
    case ATTN_ERR_UNSUPPORTED: return "unsupported configuration";
    case ATTN_ERR_LAUNCH: return "kernel launch failed";
    case ATTN_ERR_TOO_LARGE: return "size exceeds the library's built-in scratch memory";
    default: return "unknown status";
  }
}

int attn_version(void) { return kVersion; }

}  // extern "C"
