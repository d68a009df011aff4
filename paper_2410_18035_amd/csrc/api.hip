// C ABI of the routed-LoRA library: argument validation, workspace carving and dispatch between
// the matrix-core decode path (bf16, packed weights), the matrix-core prefill path (bf16,
// row-major weights, many rows) and the any-shape path (fp32 and everything else).
#include "common.h"

namespace milora {

thread_local int g_last_hip_error = 0;

// decode.hip
size_t decode_packed_workspace_bytes(int M, int d, int F, int r_max);
int layer_decode_packed(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                        const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                        bf16_t* y, bf16_t* qkv_out, void* workspace, hipStream_t st, LaunchMarks* marks);
int routed_linear_packed(const bf16_t* X, int M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                         const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                         const uint8_t* route, int B, bf16_t* Y, void* workspace, hipStream_t st);
size_t routed_linear_packed_workspace_bytes(int M, int d1, int d2, int r_max);
int pack_weight(const void* src, void* dst, int d1, int d2, hipStream_t st);
int set_wait_limit(int polls);
size_t decode_trace_bytes();
int decode_trace_dims(int* stages_max, int* waves, int* slots);
int layer_decode_packed_static(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                               const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                               bf16_t* y, bf16_t* qkv_out, hipStream_t st);
int static_scratch_status(int* status, hipStream_t st);
// prefill.hip
int decode_workspace_status(const void* workspace, int* status, hipStream_t st);
bool prefill_supported(int64_t M, int d1, int d2, const void* X, const void* W, const void* Y);
int launch_shrink_tiles(const bf16_t* X, int64_t M, int d1, const int32_t* row_to_req, const AdapterView& ad, int site,
                        const int32_t* tenant_id, const uint8_t* route, int B, float* t, hipStream_t stream);
int routed_linear_prefill(const bf16_t* X, int64_t M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                          const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                          const uint8_t* route, int B, const float* t, bf16_t* Y, hipStream_t st);

namespace {

constexpr int kThreads = 256;

template <typename T>
__device__ __forceinline__ float block_sum(float v, float* sh) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
  for (int w = 0; w < kThreads / 64; ++w) s += sh[w];
  __syncthreads();
  return s;
}

// out[m] = T(n(in[m])) with n = weightless RMS normalisation (one workgroup per row).
template <typename T>
__global__ void __launch_bounds__(kThreads) rmsnorm_rows_kernel(const T* __restrict__ in, int d, T* __restrict__ out) {
  __shared__ float sh[kThreads / 64];
  const size_t m = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += kThreads) {
    const float v = Elem<T>::load(in, m * d + i);
    ss += v * v;
  }
  const float inv = rsqrtf(block_sum<T>(ss, sh) / (float)d + 1e-5f);
  for (int i = threadIdx.x; i < d; i += kThreads) Elem<T>::store(out, m * d + i, Elem<T>::load(in, m * d + i) * inv);
}

// h = x + o in fp32; hn = T(n(h)) or T(h).
template <typename T>
__global__ void __launch_bounds__(kThreads) resid_norm_kernel(const T* __restrict__ x, const T* __restrict__ o, int d,
                                                              int norm, float* __restrict__ h, T* __restrict__ hn) {
  __shared__ float sh[kThreads / 64];
  const size_t m = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += kThreads) {
    const float v = Elem<T>::load(x, m * d + i) + Elem<T>::load(o, m * d + i);
    h[m * d + i] = v;
    ss += v * v;
  }
  const float tot = block_sum<T>(ss, sh);
  const float inv = norm ? rsqrtf(tot / (float)d + 1e-5f) : 1.f;
  for (int i = threadIdx.x; i < d; i += kThreads) Elem<T>::store(hn, m * d + i, h[m * d + i] * inv);
}

template <typename T>
__global__ void __launch_bounds__(kThreads) silu_mul_kernel(const T* __restrict__ g, const T* __restrict__ u, size_t n,
                                                            T* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) Elem<T>::store(out, i, silu(Elem<T>::load(g, i)) * Elem<T>::load(u, i));
}

template <typename T>
__global__ void __launch_bounds__(kThreads) add_f32_kernel(const float* __restrict__ h, const T* __restrict__ dn, size_t n,
                                                           T* __restrict__ y) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) Elem<T>::store(y, i, h[i] + Elem<T>::load(dn, i));
}

template <typename T>
__global__ void __launch_bounds__(kThreads) interleave_qkv_kernel(const T* __restrict__ qkv3, int B, int d, T* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t n = (size_t)3 * B * d;
  if (i >= n) return;
  const size_t s = i / ((size_t)B * d), rem = i % ((size_t)B * d);
  const size_t b = rem / d, c = rem % d;
  out[(b * 3 + s) * d + c] = qkv3[i];
}

// Workspace of the any-shape layer path.
struct GenericWs {
  float* t;   // [B][r_max]
  float* h;   // [B][d]
  char* xn;   // [B][d]   T
  char* qkv;  // [3][B][d] T
  char* o;    // [B][d]   T
  char* hn;   // [B][d]   T
  char* g;    // [B][F]   T
  char* u;    // [B][F]   T
  char* mm;   // [B][F]   T
  char* dn;   // [B][d]   T
  size_t bytes;
};

GenericWs carve_generic(void* base, int B, int d, int F, int r_max, size_t es) {
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  char* b = (char*)base;
  GenericWs w;
  w.t = (float*)(b + take((size_t)B * r_max * 4));
  w.h = (float*)(b + take((size_t)B * d * 4));
  w.xn = b + take((size_t)B * d * es);
  w.qkv = b + take((size_t)3 * B * d * es);
  w.o = b + take((size_t)B * d * es);
  w.hn = b + take((size_t)B * d * es);
  w.g = b + take((size_t)B * F * es);
  w.u = b + take((size_t)B * F * es);
  w.mm = b + take((size_t)B * F * es);
  w.dn = b + take((size_t)B * d * es);
  w.bytes = off;
  return w;
}

template <typename T>
int layer_decode_generic(const void* x, int B, int d, int F, int dtype, const milora_layer_weights* wts,
                         const AdapterView& ad, const int32_t* tenant_id, const uint8_t* route, uint32_t flags,
                         const void* attn_out, void* y, void* qkv_out, void* workspace, hipStream_t st) {
  GenericWs w = carve_generic(workspace, B, d, F, ad.r_max, sizeof(T));
  const int norm = (flags & MILORA_LAYER_RMSNORM) ? 1 : 0;
  int rc;
  auto lin = [&](const void* in, int site, void* out) -> int {
    int d1, d2;
    site_dims(site, d, F, &d1, &d2);
    int r = launch_shrink(in, B, d1, dtype, nullptr, ad, site, tenant_id, route, B, w.t, st);
    if (r) return r;
    return launch_linear_generic(in, B, d1, d2, dtype, nullptr, wts->W[site], nullptr, ad, site, tenant_id, route, B,
                                 w.t, out, st);
  };
  const void* xin = x;
  if (norm) {
    hipLaunchKernelGGL(rmsnorm_rows_kernel<T>, dim3(B), dim3(kThreads), 0, st, (const T*)x, d, (T*)w.xn);
    if ((rc = check_launch())) return rc;
    xin = w.xn;
  }
  T* q3 = (T*)w.qkv;
  for (int s = 0; s < 3; ++s)
    if ((rc = lin(xin, s, q3 + (size_t)s * B * d))) return rc;
  if (qkv_out) {
    const size_t n = (size_t)3 * B * d;
    hipLaunchKernelGGL(interleave_qkv_kernel<T>, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                       (const T*)q3, B, d, (T*)qkv_out);
    if ((rc = check_launch())) return rc;
  }
  const void* a = attn_out ? attn_out : (const void*)(q3 + (size_t)2 * B * d);
  if ((rc = lin(a, 3, w.o))) return rc;
  hipLaunchKernelGGL(resid_norm_kernel<T>, dim3(B), dim3(kThreads), 0, st, (const T*)x, (const T*)w.o, d, norm, w.h,
                     (T*)w.hn);
  if ((rc = check_launch())) return rc;
  if ((rc = lin(w.hn, 4, w.g))) return rc;
  if ((rc = lin(w.hn, 5, w.u))) return rc;
  const size_t nF = (size_t)B * F, nd = (size_t)B * d;
  hipLaunchKernelGGL(silu_mul_kernel<T>, dim3((unsigned)((nF + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     (const T*)w.g, (const T*)w.u, nF, (T*)w.mm);
  if ((rc = check_launch())) return rc;
  if ((rc = lin(w.mm, 6, w.dn))) return rc;
  hipLaunchKernelGGL(add_f32_kernel<T>, dim3((unsigned)((nd + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, w.h,
                     (const T*)w.dn, nd, (T*)y);
  return check_launch();
}

bool valid_dtype(int dt) { return dt == MILORA_BF16 || dt == MILORA_F32; }

int check_adapters(const milora_adapters* a) {
  if (!a || !a->rank || !a->A || !a->B) return MILORA_EINVAL;
  if (a->n_tenants < 1 || a->r_max < 1) return MILORA_EINVAL;
  if (a->r_max > MILORA_MAX_RANK) return MILORA_ERANGE;
  return MILORA_OK;
}

bool packed_shape_ok(int d1, int d2) { return d1 % 32 == 0 && d2 % 16 == 0; }
bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace
}  // namespace milora

using namespace milora;

extern "C" const char* milora_version(void) { return "milora-mi355x 0.1 (gfx950)"; }

extern "C" const char* milora_status_string(int status) {
  switch (status) {
    case MILORA_OK: return "ok";
    case MILORA_EINVAL: return "invalid argument";
    case MILORA_ERANGE: return "size beyond a documented limit";
    case MILORA_EUNSUPPORTED: return "combination not supported";
    case MILORA_EHIP: return "HIP call failed";
    case MILORA_EWORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

extern "C" int milora_last_hip_error(void) { return g_last_hip_error; }

extern "C" size_t milora_routed_linear_workspace_bytes(int64_t M, int d1, int d2, int r_max) {
  if (M < 1 || d1 < 1 || d2 < 1 || r_max < 1) return 0;
  size_t generic = align_up((size_t)M * r_max * sizeof(float) * kPrefillShrinkParts, 256);
  const int mp = M <= MILORA_MAX_DECODE_BATCH ? (int)M : MILORA_MAX_DECODE_BATCH;
  size_t packed = routed_linear_packed_workspace_bytes(mp, d1, d2, r_max);
  return generic > packed ? generic : packed;
}

extern "C" int milora_routed_linear_kernel(int64_t M, int d1, int d2, int dtype, int w_layout) {
  if (M < 1 || d1 < 1 || d2 < 1 || !valid_dtype(dtype)) return MILORA_EINVAL;
  if (w_layout != MILORA_W_ROWMAJOR && w_layout != MILORA_W_PACKED) return MILORA_EINVAL;
  if (w_layout == MILORA_W_PACKED) {
    if (dtype != MILORA_BF16 || !packed_shape_ok(d1, d2)) return MILORA_EUNSUPPORTED;
    return MILORA_KERNEL_STREAM;
  }
  const void* aligned = (const void*)(uintptr_t)256;
  if (dtype == MILORA_BF16 && prefill_supported(M, d1, d2, aligned, aligned, aligned)) return MILORA_KERNEL_TILES;
  return MILORA_KERNEL_GENERIC;
}

extern "C" int milora_routed_linear(const void* X, int64_t M, int d1, int d2, int dtype, const int32_t* row_to_req,
                                    const void* W, int w_layout, const void* bias, const milora_adapters* adapters,
                                    int site, const int32_t* tenant_id, const uint8_t* route, int B, void* Y,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !W || !Y || !tenant_id || !route) return MILORA_EINVAL;
  if (M < 1 || d1 < 1 || d2 < 1 || B < 1) return MILORA_EINVAL;
  if (!valid_dtype(dtype) || site < 0 || site >= MILORA_NUM_SITES) return MILORA_EINVAL;
  if (w_layout != MILORA_W_ROWMAJOR && w_layout != MILORA_W_PACKED) return MILORA_EINVAL;
  if (!row_to_req && M != B) return MILORA_EINVAL;
  int rc = check_adapters(adapters);
  if (rc) return rc;
  if (M > 0x7fffffffLL) return MILORA_ERANGE;
  if (!workspace || workspace_bytes < milora_routed_linear_workspace_bytes(M, d1, d2, adapters->r_max))
    return MILORA_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const AdapterView ad = view_of(adapters);
  if (w_layout == MILORA_W_PACKED) {
    if (dtype != MILORA_BF16 || !packed_shape_ok(d1, d2) || !aligned16(X) || !aligned16(W) || !aligned16(Y) ||
        (bias && !aligned16(bias)))
      return MILORA_EUNSUPPORTED;
    if (!row_to_req && M > MILORA_MAX_DECODE_BATCH) return MILORA_ERANGE;
    // rows are independent: larger M runs as slices of at most 128 rows (each re-reads W)
    for (int64_t m0 = 0; m0 < M; m0 += MILORA_MAX_DECODE_BATCH) {
      const int mc = (int)(M - m0 < MILORA_MAX_DECODE_BATCH ? M - m0 : MILORA_MAX_DECODE_BATCH);
      rc = routed_linear_packed((const bf16_t*)X + m0 * d1, mc, d1, d2, row_to_req ? row_to_req + m0 : nullptr,
                                (const bf16_t*)W, (const bf16_t*)bias, ad, site, tenant_id, route, B,
                                (bf16_t*)Y + m0 * d2, workspace, st);
      if (rc) return rc;
    }
    return MILORA_OK;
  }
  float* t = (float*)workspace;
  if (dtype == MILORA_BF16 && prefill_supported(M, d1, d2, X, W, Y)) {
    rc = launch_shrink_tiles((const bf16_t*)X, M, d1, row_to_req, ad, site, tenant_id, route, B, t, st);
    if (rc) return rc;
    return routed_linear_prefill((const bf16_t*)X, M, d1, d2, row_to_req, (const bf16_t*)W, (const bf16_t*)bias, ad,
                                 site, tenant_id, route, B, t, (bf16_t*)Y, st);
  }
  rc = launch_shrink(X, M, d1, dtype, row_to_req, ad, site, tenant_id, route, B, t, st);
  if (rc) return rc;
  return launch_linear_generic(X, M, d1, d2, dtype, row_to_req, W, bias, ad, site, tenant_id, route, B, t, Y, st);
}

extern "C" int milora_packed_workspace_status(const void* workspace, int* status, void* stream) {
  if (!status) return MILORA_EINVAL;
  if (!workspace) return static_scratch_status(status, (hipStream_t)stream);
  return decode_workspace_status(workspace, status, (hipStream_t)stream);
}

extern "C" int milora_set_wait_limit(int polls) { return set_wait_limit(polls); }

extern "C" size_t milora_layer_decode_workspace_bytes(int B, int d, int F, int r_max) {
  if (B < 1 || d < 1 || F < 1 || r_max < 1 || B > MILORA_MAX_DECODE_BATCH) return 0;
  size_t a = carve_generic(nullptr, B, d, F, r_max, 4).bytes;
  size_t b = decode_packed_workspace_bytes(B, d, F, r_max);
  return a > b ? a : b;
}

static int layer_decode_impl(const void* x, int B, int d, int F, int dtype, const milora_layer_weights* weights,
                             const milora_adapters* adapters, const int32_t* tenant_id, const uint8_t* route,
                             uint32_t flags, const void* attn_out, void* y, void* qkv_out, void* workspace,
                             size_t workspace_bytes, void* stream, LaunchMarks* marks) {
  if (!x || !y || !weights || !tenant_id || !route) return MILORA_EINVAL;
  if (B < 1 || d < 1 || F < 1 || !valid_dtype(dtype)) return MILORA_EINVAL;
  if (flags & ~MILORA_LAYER_RMSNORM) return MILORA_EINVAL;
  for (int m = 0; m < MILORA_NUM_SITES; ++m)
    if (!weights->W[m]) return MILORA_EINVAL;
  if (weights->layout != MILORA_W_ROWMAJOR && weights->layout != MILORA_W_PACKED) return MILORA_EINVAL;
  int rc = check_adapters(adapters);
  if (rc) return rc;
  if (B > MILORA_MAX_DECODE_BATCH) return MILORA_ERANGE;
  if (!workspace || workspace_bytes < milora_layer_decode_workspace_bytes(B, d, F, adapters->r_max))
    return MILORA_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const AdapterView ad = view_of(adapters);
  if (weights->layout == MILORA_W_PACKED) {
    if (dtype != MILORA_BF16 || d % 32 != 0 || F % 32 != 0) return MILORA_EUNSUPPORTED;
    if (!aligned16(x) || (attn_out && !aligned16(attn_out)) || !aligned16(y) || (qkv_out && !aligned16(qkv_out)))
      return MILORA_EUNSUPPORTED;
    for (int m = 0; m < MILORA_NUM_SITES; ++m)
      if (!aligned16(weights->W[m])) return MILORA_EUNSUPPORTED;
    return layer_decode_packed((const bf16_t*)x, B, d, F, weights, ad, tenant_id, route, flags,
                               (const bf16_t*)attn_out, (bf16_t*)y, (bf16_t*)qkv_out, workspace, st, marks);
  }
  if (marks) return MILORA_EUNSUPPORTED;
  if (dtype == MILORA_BF16)
    return layer_decode_generic<bf16_t>(x, B, d, F, dtype, weights, ad, tenant_id, route, flags, attn_out, y, qkv_out,
                                        workspace, st);
  return layer_decode_generic<float>(x, B, d, F, dtype, weights, ad, tenant_id, route, flags, attn_out, y, qkv_out,
                                     workspace, st);
}

extern "C" int milora_layer_decode(const void* x, int B, int d, int F, int dtype, const milora_layer_weights* weights,
                                   const milora_adapters* adapters, const int32_t* tenant_id, const uint8_t* route,
                                   uint32_t flags, const void* attn_out, void* y, void* qkv_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return layer_decode_impl(x, B, d, F, dtype, weights, adapters, tenant_id, route, flags, attn_out, y, qkv_out,
                           workspace, workspace_bytes, stream, nullptr);
}

extern "C" int milora_layer_decode_noalloc(const void* x, int B, int d, int F, int dtype,
                                           const milora_layer_weights* weights, const milora_adapters* adapters,
                                           const int32_t* tenant_id, const uint8_t* route, uint32_t flags,
                                           const void* attn_out, void* y, void* qkv_out, void* stream) {
  if (!x || !y || !weights || !tenant_id || !route) return MILORA_EINVAL;
  if (B < 1 || d < 1 || F < 1 || !valid_dtype(dtype)) return MILORA_EINVAL;
  if (flags & ~MILORA_LAYER_RMSNORM) return MILORA_EINVAL;
  for (int m = 0; m < MILORA_NUM_SITES; ++m)
    if (!weights->W[m]) return MILORA_EINVAL;
  int rc = check_adapters(adapters);
  if (rc) return rc;
  if (weights->layout != MILORA_W_PACKED || dtype != MILORA_BF16 || d % 32 != 0 || F % 32 != 0) return MILORA_EUNSUPPORTED;
  if (!aligned16(x) || (attn_out && !aligned16(attn_out)) || !aligned16(y) || (qkv_out && !aligned16(qkv_out)))
    return MILORA_EUNSUPPORTED;
  for (int m = 0; m < MILORA_NUM_SITES; ++m)
    if (!aligned16(weights->W[m])) return MILORA_EUNSUPPORTED;
  return layer_decode_packed_static((const bf16_t*)x, B, d, F, weights, view_of(adapters), tenant_id, route, flags,
                                    (const bf16_t*)attn_out, (bf16_t*)y, (bf16_t*)qkv_out, (hipStream_t)stream);
}

extern "C" int milora_layer_decode_profile(const void* x, int B, int d, int F, int dtype,
                                           const milora_layer_weights* weights, const milora_adapters* adapters,
                                           const int32_t* tenant_id, const uint8_t* route, uint32_t flags,
                                           const void* attn_out, void* y, void* qkv_out, void* workspace,
                                           size_t workspace_bytes, void* stream, int reps, float* slot_ms) {
  if (!slot_ms || reps < 1) return MILORA_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t ev[MILORA_PROFILE_SLOTS + 1];
  for (int i = 0; i <= MILORA_PROFILE_SLOTS; ++i) MILORA_HIP(hipEventCreate(&ev[i]));
  for (int i = 0; i < MILORA_PROFILE_SLOTS; ++i) slot_ms[i] = 0.f;
  LaunchMarks marks{ev + 1, MILORA_PROFILE_SLOTS};
  int rc = MILORA_OK;
  for (int r = 0; r < reps && rc == MILORA_OK; ++r) {
    MILORA_HIP(hipEventRecord(ev[0], st));
    rc = layer_decode_impl(x, B, d, F, dtype, weights, adapters, tenant_id, route, flags, attn_out, y, qkv_out,
                           workspace, workspace_bytes, stream, &marks);
    if (rc != MILORA_OK) break;
    MILORA_HIP(hipStreamSynchronize(st));
    for (int i = 0; i < MILORA_PROFILE_SLOTS; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) == hipSuccess) slot_ms[i] += ms / (float)reps;
      else (void)hipGetLastError();
    }
  }
  for (int i = 0; i <= MILORA_PROFILE_SLOTS; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

extern "C" size_t milora_layer_decode_trace_bytes(void) { return decode_trace_bytes(); }

extern "C" int milora_layer_decode_trace(const void* x, int B, int d, int F, int dtype,
                                         const milora_layer_weights* weights, const milora_adapters* adapters,
                                         const int32_t* tenant_id, const uint8_t* route, uint32_t flags,
                                         const void* attn_out, void* y, void* qkv_out, void* workspace,
                                         size_t workspace_bytes, void* stream, void* stamps, size_t stamps_bytes,
                                         int32_t* dims) {
  if (!stamps || !dims) return MILORA_EINVAL;
  if (stamps_bytes < decode_trace_bytes()) return MILORA_EWORKSPACE;
  if (!weights || weights->layout != MILORA_W_PACKED) return MILORA_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  MILORA_HIP(hipMemsetAsync(stamps, 0, decode_trace_bytes(), st));
  LaunchMarks marks{nullptr, 0};
  marks.trace = (long long*)stamps;
  const int rc = layer_decode_impl(x, B, d, F, dtype, weights, adapters, tenant_id, route, flags, attn_out, y, qkv_out,
                                   workspace, workspace_bytes, stream, &marks);
  if (rc != MILORA_OK) return rc;
  MILORA_HIP(hipStreamSynchronize(st));
  int smax = 0, waves = 0, slots = 0;
  decode_trace_dims(&smax, &waves, &slots);
  dims[0] = marks.grid; dims[1] = marks.stages; dims[2] = smax; dims[3] = waves; dims[4] = slots;
  return MILORA_OK;
}

extern "C" int milora_pack_weight(const void* src_rowmajor, void* dst_packed, int d1, int d2, void* stream) {
  if (!src_rowmajor || !dst_packed || d1 < 1 || d2 < 1) return MILORA_EINVAL;
  if (!packed_shape_ok(d1, d2) || !aligned16(src_rowmajor) || !aligned16(dst_packed)) return MILORA_EUNSUPPORTED;
  return pack_weight(src_rowmajor, dst_packed, d1, d2, (hipStream_t)stream);
}
