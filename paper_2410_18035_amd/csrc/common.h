// Shared host/device helpers of the routed-LoRA library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/milora.h"

namespace milora {

// ---- host-side error plumbing -------------------------------------------------------------------
extern thread_local int g_last_hip_error;

inline int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return MILORA_EHIP;
}

#define MILORA_HIP(call)                              \
  do {                                                \
    hipError_t e__ = (call);                          \
    if (e__ != hipSuccess) return milora::hip_fail(e__); \
  } while (0)

inline int check_launch() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MILORA_OK : hip_fail(e);
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Input and output width of the linear at `site` (Sec. 3.1 of the paper).
inline void site_dims(int site, int d, int F, int* d1, int* d2) {
  *d1 = (site == 6) ? F : d;
  *d2 = (site == 4 || site == 5) ? F : d;
}

// ---- device-side scalar conversions -------------------------------------------------------------
typedef uint16_t bf16_t;  // raw bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Round-to-nearest-even; NaN stays NaN.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kDtype = MILORA_F32;
  __device__ static __forceinline__ float load(const float* p, size_t i) { return p[i]; }
  __device__ static __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kDtype = MILORA_BF16;
  __device__ static __forceinline__ float load(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
  __device__ static __forceinline__ void store(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
};

inline size_t dtype_size(int dtype) { return dtype == MILORA_BF16 ? 2 : 4; }

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

// Device view of the per-tenant adapter tables of one layer.
struct AdapterView {
  const int32_t* rank;
  const void* const* A;
  const void* const* B;
  int n_tenants;
  int r_max;
};

inline AdapterView view_of(const milora_adapters* a) {
  return AdapterView{a->rank, a->A, a->B, a->n_tenants, a->r_max};
}

// Does a route byte select `site`?  0..6 name one site, 0x80 | mask a set of sites (bit m = site m), 255 none.
__host__ __device__ __forceinline__ bool route_has(uint8_t route, int site) {
  if (route < MILORA_NUM_SITES) return route == site;
  if (route == MILORA_ROUTE_NONE || !(route & 0x80)) return false;
  return ((route >> site) & 1) != 0;
}

// Rank of the LoRA term of request `b` at `site`, or 0 when the request carries none there
// (not routed to the site, or an id out of range).
__device__ __forceinline__ int routed_rank(const AdapterView& ad, const int32_t* tenant_id, const uint8_t* route,
                                           int b, int B, int site, int* tenant) {
  if (b < 0 || b >= B || !route_has(route[b], site)) return 0;
  int t = tenant_id[b];
  if (t < 0 || t >= ad.n_tenants) return 0;
  int r = ad.rank[t];
  if (r < 1 || r > ad.r_max) return 0;
  *tenant = t;
  return r;
}

// Optional per-launch event marks of the packed layer path (measurement only).
struct LaunchMarks {
  hipEvent_t* ev;
  int n;
  long long* trace = nullptr;  // device buffer for the kernels' own time stamps (tracing launch), or null
  int grid = 0, stages = 0;    // filled in by a tracing launch: workgroups and stages it ran
};

// The many-row LoRA shrink cuts its reduction into this many parts (one workgroup each); the workspace holds
// one [M][r_max] fp32 array per part.
constexpr int kPrefillShrinkParts = 4;

// ---- internal entry points shared between translation units ------------------------------------
// LoRA shrink: for every row m whose request is routed to `site`, t[m][0..r) = X[m] . A (fp32).
// t is [M][r_max] floats; rows that carry no LoRA term are left untouched.
int launch_shrink(const void* X, int64_t M, int d1, int dtype, const int32_t* row_to_req, const AdapterView& ad,
                  int site, const int32_t* tenant_id, const uint8_t* route, int B, float* t, hipStream_t stream);

// Any-shape linear with the LoRA expand fused before the single rounding:
// Y[m] = X[m] W + bias + t[m] . B for routed rows.  W row-major [d2][d1].
int launch_linear_generic(const void* X, int64_t M, int d1, int d2, int dtype, const int32_t* row_to_req,
                          const void* W, const void* bias, const AdapterView& ad, int site,
                          const int32_t* tenant_id, const uint8_t* route, int B, const float* t, void* Y,
                          hipStream_t stream);

}  // namespace milora
