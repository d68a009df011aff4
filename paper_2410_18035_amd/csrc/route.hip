// Prompt-aware LoRA router of one layer (paper Sec. 3.3): pooler (Eq. 2 and the pooler list of Sec. 3.3:
// last token, average, max, self-attention of App. C), activation g (fixed functions or the rational form of
// Sec. 3.4), router linear and top-1 selection (Eq. 3).  Two kernels: a segmented, token-split partial
// reduction over the ragged prompts (one HBM pass over H), then one workgroup per request that
// finishes the pooling, applies g, forms the seven logits and picks the expert.
// Pooled state, activation and logits stay in fp32; every sum runs in a fixed order, so the
// same prompt always yields the same route.
#include "common.h"

namespace milora {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxSplits = 128;  // token slices per request at most

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
template <typename T, int VEC, bool IS_MAX>
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
    for (int v = 0; v < VEC; ++v) acc[v] = IS_MAX ? -INFINITY : 0.f;
    const T* col = H + (size_t)c * VEC;
    int64_t t = t0 + tr;
    for (; t + 3 * TR < t1; t += 4 * TR) {
      float x0[VEC], x1[VEC], x2[VEC], x3[VEC];
      VecLoad<T, VEC>::load(col + (size_t)t * d, x0);
      VecLoad<T, VEC>::load(col + (size_t)(t + TR) * d, x1);
      VecLoad<T, VEC>::load(col + (size_t)(t + 2 * TR) * d, x2);
      VecLoad<T, VEC>::load(col + (size_t)(t + 3 * TR) * d, x3);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        if (IS_MAX) acc[v] = fmaxf(acc[v], fmaxf(fmaxf(x0[v], x1[v]), fmaxf(x2[v], x3[v])));
        else acc[v] += (x0[v] + x1[v]) + (x2[v] + x3[v]);
      }
    }
    for (; t < t1; t += TR) {
      float x0[VEC];
      VecLoad<T, VEC>::load(col + (size_t)t * d, x0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = IS_MAX ? fmaxf(acc[v], x0[v]) : acc[v] + x0[v];
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
        float a = IS_MAX ? -INFINITY : 0.f;
        for (int r = 0; r < TR; ++r) {
          const float x = red[(r * cgw + cg) * VEC + v];
          a = IS_MAX ? fmaxf(a, x) : a + x;
        }
        out[(size_t)cg * VEC + v] = a;
      }
    }
  }
}

// Self-attention pooling (App. C): u_t = H[t] . w_sa, a = softmax over the request's tokens, p = sum_t a_t H[t].
// A workgroup takes one token slice of one request in blocks of 256 tokens: scores (one wave per token), the
// block's maximum, then the weighted sum with the running maximum as reference (a block that raises the
// maximum rescales what was gathered before it).  Out: the unnormalised weighted sum, and (max, sum of
// weights) per slice; the finishing kernel merges the slices.  d <= 8192.
constexpr int kSelfAttnMaxD = 8192;

template <typename T, int VEC>
__global__ void __launch_bounds__(kThreads) pool_selfattn_kernel(const T* __restrict__ H, int64_t M_tok, int d,
                                                                 const int32_t* __restrict__ seq_start,
                                                                 const int32_t* __restrict__ seq_len,
                                                                 const int32_t* __restrict__ tenant_id, int T_tenants,
                                                                 const T* __restrict__ w_sa, int S, int cgw,
                                                                 float* __restrict__ partial, float* __restrict__ ml) {
  constexpr int MAXP = 32 / VEC;  // column passes of a thread: d / VEC / 256 at most
  __shared__ float sc[kThreads];
  __shared__ float red[kThreads * VEC];
  __shared__ float wred[kThreads / 64];
  const int b = blockIdx.y, s = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t start = seq_start[b], n = seq_len[b];
  const int ten = tenant_id[b];
  if (!span_ok(start, n, M_tok) || ten < 0 || ten >= T_tenants) return;  // the finishing kernel skips it too
  const int64_t per = (n + S - 1) / S;
  const int64_t t0 = start + (int64_t)s * per;
  int64_t t1 = t0 + per;
  if (t1 > start + n) t1 = start + n;
  const int ncg = d / VEC;
  const int cg = threadIdx.x % cgw, tr = threadIdx.x / cgw, TR = kThreads / cgw;
  const T* q = w_sa + (size_t)ten * d;
  float acc[MAXP][VEC];
#pragma unroll
  for (int pss = 0; pss < MAXP; ++pss)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[pss][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  for (int64_t tb = t0; tb < t1; tb += kThreads) {
    const int nb = (int)(t1 - tb < kThreads ? t1 - tb : kThreads);
    for (int tt = wave; tt < nb; tt += kThreads / 64) {
      const T* row = H + (size_t)(tb + tt) * d;
      float u = 0.f;
      for (int c = lane; c < ncg; c += 64) {
        float x[VEC], w[VEC];
        VecLoad<T, VEC>::load(row + (size_t)c * VEC, x);
        VecLoad<T, VEC>::load(q + (size_t)c * VEC, w);
#pragma unroll
        for (int v = 0; v < VEC; ++v) u += x[v] * w[v];
      }
      for (int off = 32; off > 0; off >>= 1) u += __shfl_xor(u, off, 64);
      if (lane == 0) sc[tt] = u;
    }
    __syncthreads();
    float mx = threadIdx.x < nb ? sc[threadIdx.x] : -INFINITY;
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) wred[wave] = mx;
    __syncthreads();
    float m_new = m_run;
    for (int w = 0; w < kThreads / 64; ++w) m_new = fmaxf(m_new, wred[w]);
    const float scale = expf(m_run - m_new);  // 0 for the first block (m_run = -inf)
    const float pw = threadIdx.x < nb ? expf(sc[threadIdx.x] - m_new) : 0.f;
    __syncthreads();
    if (threadIdx.x < nb) sc[threadIdx.x] = pw;
    float ps = pw;
    for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
    if (lane == 0) wred[wave] = ps;
    __syncthreads();
    float lsum = 0.f;
    for (int w = 0; w < kThreads / 64; ++w) lsum += wred[w];
    l_run = l_run * scale + lsum;
    m_run = m_new;
#pragma unroll
    for (int pss = 0; pss < MAXP; ++pss) {
      const int c = cg + pss * cgw;
      if (c < ncg) {
        float a[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) a[v] = 0.f;
        const T* col = H + (size_t)tb * d + (size_t)c * VEC;
        for (int tt = tr; tt < nb; tt += TR) {
          float x[VEC];
          VecLoad<T, VEC>::load(col + (size_t)tt * d, x);
          const float p = sc[tt];
#pragma unroll
          for (int v = 0; v < VEC; ++v) a[v] += p * x[v];
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[pss][v] = acc[pss][v] * scale + a[v];
      }
    }
    __syncthreads();
  }
  float* out = partial + ((size_t)b * S + s) * d;
  if (TR == 1) {
#pragma unroll
    for (int pss = 0; pss < MAXP; ++pss) {
      const int c = cg + pss * cgw;
      if (c < ncg) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[(size_t)c * VEC + v] = acc[pss][v];
      }
    }
  } else {
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[threadIdx.x * VEC + v] = acc[0][v];
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
  if (threadIdx.x == 0) {
    ml[((size_t)b * S + s) * 2] = m_run;
    ml[((size_t)b * S + s) * 2 + 1] = l_run;
  }
}

// Coefficients of the rational activation Ra(x) = (a_0 + a_1 x + ... + a_6 x^6) / (1 + |b_1 x + ... + b_5 x^5|)
// (Sec. 3.4); passed by value.
struct RationalCoef {
  float a[7];
  float b[5];
};

__device__ __forceinline__ float activate(float x, int act, const RationalCoef& rc) {
  switch (act) {
    case MILORA_ACT_TANH: return tanhf(x);
    case MILORA_ACT_RELU: return x > 0.f ? x : 0.f;
    case MILORA_ACT_GELU: return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
    case MILORA_ACT_RATIONAL: {
      float num = rc.a[6], den = rc.b[4];
#pragma unroll
      for (int j = 5; j >= 0; --j) num = num * x + rc.a[j];
#pragma unroll
      for (int j = 3; j >= 0; --j) den = den * x + rc.b[j];
      return num / (1.0f + fabsf(den * x));
    }
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
                                                                      int act, RationalCoef coef, int top_k, int S,
                                                                      const float* __restrict__ partial,
                                                                      const float* __restrict__ ml,
                                                                      uint8_t* __restrict__ route_out,
                                                                      float* __restrict__ logits_out) {
  __shared__ float wsum[kFinishThreads / 64][MILORA_NUM_SITES];
  __shared__ float wts[kMaxSplits];  // weight of each slice's partial result in the pooled state
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
  if (pool == MILORA_POOL_SELFATTN) {
    // slices hold sums weighted by exp(u - m_s): bring them to the common maximum and normalise
    const float* mlb = ml + (size_t)b * S * 2;
    float mx = -INFINITY, z = 0.f;
    for (int s = 0; s < S; ++s) mx = fmaxf(mx, mlb[2 * s]);
    for (int s = 0; s < S; ++s) z += mlb[2 * s + 1] * expf(mlb[2 * s] - mx);
    if (threadIdx.x < S) wts[threadIdx.x] = mlb[2 * threadIdx.x + 1] > 0.f ? expf(mlb[2 * threadIdx.x] - mx) / z : 0.f;
  } else if (threadIdx.x < S) {
    wts[threadIdx.x] = inv_n;
  }
  __syncthreads();
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
        for (int v = 0; v < 4; ++v) run[u][v] = pool == MILORA_POOL_MAX ? -INFINITY : 0.f;
      for (int s0 = 0; s0 < S; s0 += kFinishWays) {
#pragma unroll
        for (int u = 0; u < kFinishWays; ++u) {
          if (s0 + u < S) {
            const float* q = pb + (size_t)(s0 + u) * d + i0;
            float x[4] = {0.f, 0.f, 0.f, 0.f};
            if (vec) {
              const float4 x4 = *reinterpret_cast<const float4*>(q);
              x[0] = x4.x; x[1] = x4.y; x[2] = x4.z; x[3] = x4.w;
            } else {
              for (int v = 0; v < nv; ++v) x[v] = q[v];
            }
            const float wgt = wts[s0 + u];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              if (pool == MILORA_POOL_MAX) run[u][v] = fmaxf(run[u][v], x[v]);
              else if (wgt != 0.f) run[u][v] += wgt * x[v];  // a slice without tokens holds nothing to read
            }
          }
        }
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        if (pool == MILORA_POOL_MAX)
          h[v] = fmaxf(fmaxf(fmaxf(run[0][v], run[1][v]), fmaxf(run[2][v], run[3][v])),
                       fmaxf(fmaxf(run[4][v], run[5][v]), fmaxf(run[6][v], run[7][v])));
        else
          h[v] = ((run[0][v] + run[1][v]) + (run[2][v] + run[3][v])) +
                 ((run[4][v] + run[5][v]) + (run[6][v] + run[7][v]));
      }
    }
    for (int v = 0; v < nv; ++v) {
      const float z = activate(h[v], act, coef);
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
    for (int j = 0; j < MILORA_NUM_SITES; ++j) {
      float v = 0.f;
      for (int wv = 0; wv < kFinishThreads / 64; ++wv) v += wsum[wv][j];
      logit[j] = v;
      if (logits_out) logits_out[b * MILORA_NUM_SITES + j] = v;
    }
    // the top_k largest logits, an exact tie going to the lower index
    unsigned mask = 0;
    int last = 0;
    for (int q = 0; q < top_k; ++q) {
      int best = -1;
      for (int j = 0; j < MILORA_NUM_SITES; ++j)
        if (!((mask >> j) & 1) && (best < 0 || logit[j] > logit[best])) best = j;
      mask |= 1u << best;
      last = best;
    }
    route_out[b] = top_k == 1 ? (uint8_t)last : (uint8_t)(0x80u | mask);
  }
}

int pick_splits(int B, int64_t M_tok) {
  int64_t avg = (M_tok + B - 1) / B;
  int64_t s = (4096 + B - 1) / B;  // aim at a few thousand workgroups
  if (s > (avg + 15) / 16) s = (avg + 15) / 16;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  return (int)s;
}

template <typename T, int VEC>
void launch_pool(const void* H, int64_t M_tok, int d, const int32_t* ss, const int32_t* sl, int B, int S, bool is_max,
                 float* partial, hipStream_t st) {
  int ncg = d / VEC, cgw = 1;
  while (cgw < ncg && cgw < kThreads) cgw <<= 1;
  if (is_max)
    hipLaunchKernelGGL((pool_partial_kernel<T, VEC, true>), dim3(S, B), dim3(kThreads), 0, st, (const T*)H, M_tok, d, ss,
                       sl, S, cgw, partial);
  else
    hipLaunchKernelGGL((pool_partial_kernel<T, VEC, false>), dim3(S, B), dim3(kThreads), 0, st, (const T*)H, M_tok, d, ss,
                       sl, S, cgw, partial);
}

template <typename T, int VEC>
void launch_selfattn(const void* H, int64_t M_tok, int d, const int32_t* ss, const int32_t* sl, const int32_t* tenant_id,
                     int T_tenants, const void* w_sa, int B, int S, float* partial, float* ml, hipStream_t st) {
  int ncg = d / VEC, cgw = 1;
  while (cgw < ncg && cgw < kThreads) cgw <<= 1;
  hipLaunchKernelGGL((pool_selfattn_kernel<T, VEC>), dim3(S, B), dim3(kThreads), 0, st, (const T*)H, M_tok, d, ss, sl,
                     tenant_id, T_tenants, (const T*)w_sa, S, cgw, partial, ml);
}

size_t partial_bytes(int B, int S, int d) { return align_up((size_t)B * S * d * sizeof(float), 256); }

}  // namespace

}  // namespace milora

using namespace milora;

extern "C" size_t milora_route_workspace_bytes(int B, int d, int64_t M_tok) {
  if (B < 1 || d < 1 || M_tok < 1) return 0;
  const int S = pick_splits(B, M_tok);
  return partial_bytes(B, S, d) + align_up((size_t)B * S * 2 * sizeof(float), 256);
}

extern "C" int milora_route(const void* H, int64_t M_tok, int d, int dtype, const int32_t* seq_start,
                            const int32_t* seq_len, const int32_t* tenant_id, int B, int n_tenants, const void* Wr,
                            int pool, int act, const void* w_sa, const float* act_coef, int top_k,
                            uint8_t* route_out, float* logits_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (!H || !seq_start || !seq_len || !tenant_id || !Wr || !route_out) return MILORA_EINVAL;
  if (M_tok < 1 || d < 1 || B < 1 || n_tenants < 1) return MILORA_EINVAL;
  if (dtype != MILORA_BF16 && dtype != MILORA_F32) return MILORA_EINVAL;
  if (pool < MILORA_POOL_MEAN || pool > MILORA_POOL_SELFATTN) return MILORA_EINVAL;
  if (act < MILORA_ACT_IDENTITY || act > MILORA_ACT_RATIONAL) return MILORA_EINVAL;
  if (pool == MILORA_POOL_SELFATTN && !w_sa) return MILORA_EINVAL;
  if (act == MILORA_ACT_RATIONAL && !act_coef) return MILORA_EINVAL;
  if (top_k < 1 || top_k >= MILORA_NUM_SITES) return MILORA_EINVAL;
  if (B > 65535) return MILORA_ERANGE;
  if (pool == MILORA_POOL_SELFATTN && d > kSelfAttnMaxD) return MILORA_ERANGE;
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_splits(B, M_tok);
  float* partial = (float*)workspace;
  float* ml = workspace ? (float*)((char*)workspace + partial_bytes(B, S, d)) : nullptr;
  RationalCoef coef = {};
  if (act == MILORA_ACT_RATIONAL) {
    for (int j = 0; j < 7; ++j) coef.a[j] = act_coef[j];
    for (int j = 0; j < 5; ++j) coef.b[j] = act_coef[7 + j];
  }
  if (pool != MILORA_POOL_LAST) {
    if (!workspace || workspace_bytes < milora_route_workspace_bytes(B, d, M_tok)) return MILORA_EWORKSPACE;
    const bool aligned = ((uintptr_t)H % 16) == 0 && (pool != MILORA_POOL_SELFATTN || ((uintptr_t)w_sa % 16) == 0);
    const bool is_max = pool == MILORA_POOL_MAX;
    if (pool == MILORA_POOL_SELFATTN) {
      if (dtype == MILORA_BF16) {
        if (aligned && d % 8 == 0)
          launch_selfattn<bf16_t, 8>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
        else
          launch_selfattn<bf16_t, 1>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
      } else {
        if (aligned && d % 4 == 0)
          launch_selfattn<float, 4>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
        else
          launch_selfattn<float, 1>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
      }
    } else if (dtype == MILORA_BF16) {
      if (aligned && d % 8 == 0) launch_pool<bf16_t, 8>(H, M_tok, d, seq_start, seq_len, B, S, is_max, partial, st);
      else launch_pool<bf16_t, 1>(H, M_tok, d, seq_start, seq_len, B, S, is_max, partial, st);
    } else {
      if (aligned && d % 4 == 0) launch_pool<float, 4>(H, M_tok, d, seq_start, seq_len, B, S, is_max, partial, st);
      else launch_pool<float, 1>(H, M_tok, d, seq_start, seq_len, B, S, is_max, partial, st);
    }
    int rc = check_launch();
    if (rc != MILORA_OK) return rc;
  }
  if (dtype == MILORA_BF16)
    hipLaunchKernelGGL((route_finish_kernel<bf16_t>), dim3(B), dim3(kFinishThreads), 0, st, (const bf16_t*)H, M_tok, d,
                       seq_start, seq_len, tenant_id, n_tenants, (const bf16_t*)Wr, pool, act, coef, top_k, S, partial, ml,
                       route_out, logits_out);
  else
    hipLaunchKernelGGL((route_finish_kernel<float>), dim3(B), dim3(kFinishThreads), 0, st, (const float*)H, M_tok, d,
                       seq_start, seq_len, tenant_id, n_tenants, (const float*)Wr, pool, act, coef, top_k, S, partial, ml,
                       route_out, logits_out);
  return check_launch();
}
