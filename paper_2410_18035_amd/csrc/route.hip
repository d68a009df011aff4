// Prompt-aware LoRA router of one layer (paper Sec. 3.3): pooler (Eq. 2), activation g,
// router linear and top-1 selection (Eq. 3).  Two kernels: a segmented, token-split partial
// sum over the ragged prompts (one HBM pass over H), then one workgroup per request that
// finishes the pooling, applies g, forms the seven logits and picks the expert.
// Pooled state, activation and logits stay in fp32; every sum runs in a fixed order, so the
// same prompt always yields the same route.
#include "common.h"

namespace milora {

namespace {

constexpr int kThreads = 256;

template <typename T, int VEC> struct VecLoad;
template <> struct VecLoad<bf16_t, 8> {
  __device__ static __forceinline__ void load(const bf16_t* p, float* out) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct VecLoad<float, 4> {
  __device__ static __forceinline__ void load(const float* p, float* out) {
    float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
};
template <typename T> struct VecLoad<T, 1> {
  __device__ static __forceinline__ void load(const T* p, float* out) { out[0] = Elem<T>::load(p, 0); }
};

__device__ __forceinline__ bool span_ok(int64_t start, int64_t n, int64_t M_tok) {
  return n >= 1 && start >= 0 && start + n <= M_tok;
}

// partial[b][s][i] = sum of H[t][i] over the s-th slice of request b's valid tokens.
// cgw = threads across column groups (power of two <= 256), 256/cgw token lanes.
template <typename T, int VEC>
__global__ void __launch_bounds__(kThreads) pool_partial_kernel(const T* __restrict__ H, int64_t M_tok, int d,
                                                                const int32_t* __restrict__ seq_start,
                                                                const int32_t* __restrict__ seq_len, int S, int cgw,
                                                                float* __restrict__ partial) {
  __shared__ float red[kThreads * VEC];
  const int b = blockIdx.y, s = blockIdx.x;
  int64_t start = seq_start[b], n = seq_len[b];
  if (!span_ok(start, n, M_tok)) n = 0;
  const int64_t per = (n + S - 1) / S;
  const int64_t t0 = start + (int64_t)s * per;
  int64_t t1 = t0 + per;
  if (t1 > start + n) t1 = start + n;
  const int ncg = d / VEC;
  const int cg = threadIdx.x % cgw, tr = threadIdx.x / cgw, TR = kThreads / cgw;
  float* out = partial + ((size_t)b * S + s) * d;
  for (int c = cg; c < ncg; c += cgw) {  // more than one pass only when cgw == 256 (then TR == 1)
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    const T* col = H + (size_t)c * VEC;
    int64_t t = t0 + tr;
    for (; t + 3 * TR < t1; t += 4 * TR) {
      float x0[VEC], x1[VEC], x2[VEC], x3[VEC];
      VecLoad<T, VEC>::load(col + (size_t)t * d, x0);
      VecLoad<T, VEC>::load(col + (size_t)(t + TR) * d, x1);
      VecLoad<T, VEC>::load(col + (size_t)(t + 2 * TR) * d, x2);
      VecLoad<T, VEC>::load(col + (size_t)(t + 3 * TR) * d, x3);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += (x0[v] + x1[v]) + (x2[v] + x3[v]);
    }
    for (; t < t1; t += TR) {
      float x0[VEC];
      VecLoad<T, VEC>::load(col + (size_t)t * d, x0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += x0[v];
    }
    if (TR == 1) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) out[(size_t)c * VEC + v] = acc[v];
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) red[threadIdx.x * VEC + v] = acc[v];
    }
  }
  if (TR > 1) {
    __syncthreads();
    if (tr == 0 && cg < ncg) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        float a = 0.f;
        for (int r = 0; r < TR; ++r) a += red[(r * cgw + cg) * VEC + v];
        out[(size_t)cg * VEC + v] = a;
      }
    }
  }
}

__device__ __forceinline__ float activate(float x, int act) {
  switch (act) {
    case MILORA_ACT_TANH: return tanhf(x);
    case MILORA_ACT_RELU: return x > 0.f ? x : 0.f;
    case MILORA_ACT_GELU: return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
    default: return x;
  }
}

// One workgroup of 1024 threads per request: h (mean of the partial sums, or the last valid row), z = g(h),
// logits_j = z . Wr[t][j], route = index of the largest logit (lowest index on equality).  A thread owns four
// neighbouring columns; the S partial sums of a column are added as eight interleaved running sums (slice s
// goes to sum s % 8) that are combined pairwise at the end, so eight loads are in flight and the order is fixed.
constexpr int kFinishThreads = 1024;
constexpr int kFinishWays = 8;

template <typename T>
__global__ void __launch_bounds__(kFinishThreads) route_finish_kernel(const T* __restrict__ H, int64_t M_tok, int d,
                                                                      const int32_t* __restrict__ seq_start,
                                                                      const int32_t* __restrict__ seq_len,
                                                                      const int32_t* __restrict__ tenant_id,
                                                                      int T_tenants, const T* __restrict__ Wr, int pool,
                                                                      int act, int S, const float* __restrict__ partial,
                                                                      uint8_t* __restrict__ route_out,
                                                                      float* __restrict__ logits_out) {
  __shared__ float wsum[kFinishThreads / 64][MILORA_NUM_SITES];
  const int b = blockIdx.x;
  const int64_t start = seq_start[b], n = seq_len[b];
  const int t = tenant_id[b];
  if (!span_ok(start, n, M_tok) || t < 0 || t >= T_tenants) {
    if (threadIdx.x == 0) route_out[b] = MILORA_ROUTE_NONE;
    if (logits_out && threadIdx.x < MILORA_NUM_SITES)
      logits_out[b * MILORA_NUM_SITES + threadIdx.x] = __uint_as_float(0x7fc00000u);
    return;
  }
  float acc[MILORA_NUM_SITES];
#pragma unroll
  for (int j = 0; j < MILORA_NUM_SITES; ++j) acc[j] = 0.f;
  const T* w = Wr + (size_t)t * MILORA_NUM_SITES * d;
  const float inv_n = 1.0f / (float)n;
  const bool vec = (d % 4) == 0;  // rows of `partial` are then 16-byte aligned
  const float* pb = partial + (size_t)b * S * d;
  for (int i0 = threadIdx.x * 4; i0 < d; i0 += kFinishThreads * 4) {
    const int nv = d - i0 < 4 ? d - i0 : 4;
    float h[4] = {0.f, 0.f, 0.f, 0.f};
    if (pool == MILORA_POOL_LAST) {
      for (int v = 0; v < nv; ++v) h[v] = Elem<T>::load(H, (size_t)(start + n - 1) * d + i0 + v);
    } else {
      float run[kFinishWays][4];
#pragma unroll
      for (int u = 0; u < kFinishWays; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) run[u][v] = 0.f;
      for (int s0 = 0; s0 < S; s0 += kFinishWays) {
#pragma unroll
        for (int u = 0; u < kFinishWays; ++u) {
          if (s0 + u < S) {
            const float* q = pb + (size_t)(s0 + u) * d + i0;
            if (vec) {
              const float4 x = *reinterpret_cast<const float4*>(q);
              run[u][0] += x.x; run[u][1] += x.y; run[u][2] += x.z; run[u][3] += x.w;
            } else {
              for (int v = 0; v < nv; ++v) run[u][v] += q[v];
            }
          }
        }
      }
#pragma unroll
      for (int v = 0; v < 4; ++v)
        h[v] = (((run[0][v] + run[1][v]) + (run[2][v] + run[3][v])) +
                ((run[4][v] + run[5][v]) + (run[6][v] + run[7][v]))) * inv_n;
    }
    for (int v = 0; v < nv; ++v) {
      const float z = activate(h[v], act);
#pragma unroll
      for (int j = 0; j < MILORA_NUM_SITES; ++j) acc[j] += z * Elem<T>::load(w, (size_t)j * d + i0 + v);
    }
  }
#pragma unroll
  for (int j = 0; j < MILORA_NUM_SITES; ++j) {
    float v = acc[j];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6][j] = v;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float logit[MILORA_NUM_SITES];
    int best = 0;
    for (int j = 0; j < MILORA_NUM_SITES; ++j) {
      float v = 0.f;
      for (int wv = 0; wv < kFinishThreads / 64; ++wv) v += wsum[wv][j];
      logit[j] = v;
      if (v > logit[best]) best = j;
      if (logits_out) logits_out[b * MILORA_NUM_SITES + j] = v;
    }
    route_out[b] = (uint8_t)best;
  }
}

int pick_splits(int B, int64_t M_tok) {
  int64_t avg = (M_tok + B - 1) / B;
  int64_t s = (4096 + B - 1) / B;  // aim at a few thousand workgroups
  if (s > (avg + 15) / 16) s = (avg + 15) / 16;
  if (s > 128) s = 128;
  if (s < 1) s = 1;
  return (int)s;
}

template <typename T, int VEC>
void launch_pool(const void* H, int64_t M_tok, int d, const int32_t* ss, const int32_t* sl, int B, int S,
                 float* partial, hipStream_t st) {
  int ncg = d / VEC, cgw = 1;
  while (cgw < ncg && cgw < kThreads) cgw <<= 1;
  hipLaunchKernelGGL((pool_partial_kernel<T, VEC>), dim3(S, B), dim3(kThreads), 0, st, (const T*)H, M_tok, d, ss, sl,
                     S, cgw, partial);
}

}  // namespace

}  // namespace milora

using namespace milora;

extern "C" size_t milora_route_workspace_bytes(int B, int d, int64_t M_tok) {
  if (B < 1 || d < 1 || M_tok < 1) return 0;
  return align_up((size_t)B * pick_splits(B, M_tok) * d * sizeof(float), 256);
}

extern "C" int milora_route(const void* H, int64_t M_tok, int d, int dtype, const int32_t* seq_start,
                            const int32_t* seq_len, const int32_t* tenant_id, int B, int n_tenants, const void* Wr,
                            int pool, int act, uint8_t* route_out, float* logits_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  if (!H || !seq_start || !seq_len || !tenant_id || !Wr || !route_out) return MILORA_EINVAL;
  if (M_tok < 1 || d < 1 || B < 1 || n_tenants < 1) return MILORA_EINVAL;
  if (dtype != MILORA_BF16 && dtype != MILORA_F32) return MILORA_EINVAL;
  if (pool != MILORA_POOL_MEAN && pool != MILORA_POOL_LAST) return MILORA_EINVAL;
  if (act < MILORA_ACT_IDENTITY || act > MILORA_ACT_GELU) return MILORA_EINVAL;
  if (B > 65535) return MILORA_ERANGE;
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_splits(B, M_tok);
  float* partial = (float*)workspace;
  if (pool == MILORA_POOL_MEAN) {
    if (!workspace || workspace_bytes < milora_route_workspace_bytes(B, d, M_tok)) return MILORA_EWORKSPACE;
    const bool aligned = ((uintptr_t)H % 16) == 0;
    if (dtype == MILORA_BF16) {
      if (aligned && d % 8 == 0) launch_pool<bf16_t, 8>(H, M_tok, d, seq_start, seq_len, B, S, partial, st);
      else launch_pool<bf16_t, 1>(H, M_tok, d, seq_start, seq_len, B, S, partial, st);
    } else {
      if (aligned && d % 4 == 0) launch_pool<float, 4>(H, M_tok, d, seq_start, seq_len, B, S, partial, st);
      else launch_pool<float, 1>(H, M_tok, d, seq_start, seq_len, B, S, partial, st);
    }
    int rc = check_launch();
    if (rc != MILORA_OK) return rc;
  }
  if (dtype == MILORA_BF16)
    hipLaunchKernelGGL((route_finish_kernel<bf16_t>), dim3(B), dim3(kFinishThreads), 0, st, (const bf16_t*)H, M_tok, d,
                       seq_start, seq_len, tenant_id, n_tenants, (const bf16_t*)Wr, pool, act, S, partial, route_out,
                       logits_out);
  else
    hipLaunchKernelGGL((route_finish_kernel<float>), dim3(B), dim3(kFinishThreads), 0, st, (const float*)H, M_tok, d,
                       seq_start, seq_len, tenant_id, n_tenants, (const float*)Wr, pool, act, S, partial, route_out,
                       logits_out);
  return check_launch();
}
