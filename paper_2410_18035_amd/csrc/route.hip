// Prompt-aware LoRA router of one layer (paper Sec. 3.3): pooler (Eq. 2 and the pooler list of Sec. 3.3:
// last token, average, max, self-attention of App. C), activation g (fixed functions or the rational form of
// Sec. 3.4), router linear and top-k selection (Eq. 3).  Last-token, average and max pooling run with the router
// in one kernel (one HBM pass over H, the finish inside the same launch); the self-attention pooler keeps a
// token-split partial reduction followed by one workgroup per request.
// Pooled state, activation and logits stay in fp32; every sum runs in a fixed order, so the
// same prompt always yields the same route.
#include <atomic>

#include "common.h"

namespace milora {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxSplits = 128;  // token slices per request at most

typedef uint32_t raw_u32x4 __attribute__((ext_vector_type(4)));

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
  // the same for data that is read once (no cache line kept for it)
  __device__ static __forceinline__ void load_once(const bf16_t* p, float* out) {
    const raw_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const raw_u32x4*>(p));
    uint32_t w[4] = {v[0], v[1], v[2], v[3]};
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
  __device__ static __forceinline__ void load_once(const float* p, float* out) {
    const raw_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const raw_u32x4*>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(v[i]);
  }
};
template <typename T> struct VecLoad<T, 1> {
  __device__ static __forceinline__ void load(const T* p, float* out) { out[0] = Elem<T>::load(p, 0); }
  __device__ static __forceinline__ void load_once(const T* p, float* out) { out[0] = Elem<T>::load(p, 0); }
};

__device__ __forceinline__ bool span_ok(int64_t start, int64_t n, int64_t M_tok) {
  return n >= 1 && start >= 0 && start + n <= M_tok;
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

// The top_k largest logits as a route byte, an exact tie going to the lower index.
__device__ __forceinline__ uint8_t select_route(const float (&logit)[MILORA_NUM_SITES], int top_k) {
  unsigned mask = 0;
  int last = 0;
  for (int q = 0; q < top_k; ++q) {
    int best = -1;
    for (int j = 0; j < MILORA_NUM_SITES; ++j)
      if (!((mask >> j) & 1) && (best < 0 || logit[j] > logit[best])) best = j;
    mask |= 1u << best;
    last = best;
  }
  return top_k == 1 ? (uint8_t)last : (uint8_t)(0x80u | mask);
}

// ---- last-token, average and max pooling with the router behind them: one kernel ---------------------------------
// A workgroup of 512 threads pools one slab of 32 * VEC columns over one slice of a request's valid tokens (32
// column lanes by 16 token lanes: half a wave covers 32 * VEC contiguous elements of one row).  Its first wave
// finishes: g and the slab's share of the seven logits, stored as four 16-byte units that each carry the call's
// 64-bit tag; the wave then loads the units of all the request's slabs and, if every tag is there, adds the
// shares in slab order and selects.  The wave whose units reach memory last sees all of them; a second wave that
// sees them too computes the same bytes.  Slices that cut a prompt (few, long prompts) hand their slab sums
// through memory the same way, behind one tagged flag per slice, and the wave that sees all flags adds them in
// slice order.  Every sum has a fixed order, so the same prompt always yields the same route, whichever wave
// finishes.  The workspace needs no preparation: a tag is unique to the call, and the finishing wave wipes the tags
// it has used (a recorded launch that is replayed meets wiped tags again).
// Data another workgroup reads inside the launch is stored through to memory and loaded past the caches (an
// L2 serves one XCD only); a store is acknowledged before anything that tells of it is read.  (A 16-byte store
// reads its data registers for two more cycles after it issues, and the compiler guards only stores it can see:
// the idle cycles are part of the statement.)
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void st_through(f32x4* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_through(u32x4* p, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_through(u32x2* p, u32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
// Loads past the caches, complete when the function returns.
__device__ __forceinline__ u32x4 ld_through(const u32x4* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ u32x2 ld_through(const u32x2* p) {
  u32x2 v;
  asm volatile("global_load_dwordx2 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ void ld_through8(const f32x4* const (&q)[8], f32x4 (&v)[8]) {
  asm volatile(
      "global_load_dwordx4 %0, %8, off sc0 sc1\n\t"
      "global_load_dwordx4 %1, %9, off sc0 sc1\n\t"
      "global_load_dwordx4 %2, %10, off sc0 sc1\n\t"
      "global_load_dwordx4 %3, %11, off sc0 sc1\n\t"
      "global_load_dwordx4 %4, %12, off sc0 sc1\n\t"
      "global_load_dwordx4 %5, %13, off sc0 sc1\n\t"
      "global_load_dwordx4 %6, %14, off sc0 sc1\n\t"
      "global_load_dwordx4 %7, %15, off sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
      : "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]), "v"(q[4]), "v"(q[5]), "v"(q[6]), "v"(q[7])
      : "memory");
}
__device__ __forceinline__ void wait_all_mem() { __builtin_amdgcn_s_waitcnt(0); }

constexpr int kPoolThreads = 512;
constexpr int kColLanes = 32;
constexpr int kTokenLanes = kPoolThreads / kColLanes;

template <typename T>
struct PoolRouteArgs {
  const T* H;
  int64_t M_tok;
  int d;
  const int32_t* seq_start;
  const int32_t* seq_len;
  const int32_t* tenant_id;
  int T_tenants;
  const T* Wr;
  int pool, act, top_k;
  int S, C;            // token slices per request, column slabs
  uint32_t tag_lo, tag_hi;  // this call's tag, tag_lo != 0
  float* partial;      // [B][C][S][32 * VEC]
  u32x2* arrived;      // [B][C][S]: the tag once the slice's slab sums are in `partial`
  u32x4* share;        // [B][C][4]: {logit 2u, logit 2u + 1, tag} of the slab
  uint8_t* route_out;
  float* logits_out;
  RationalCoef coef;
};

template <typename T, int VEC>
__global__ void __launch_bounds__(kPoolThreads) pool_route_kernel(PoolRouteArgs<T> p) {
  constexpr int SW = kColLanes * VEC;  // columns of a slab
  constexpr int FT = SW / 4;           // lanes of the first wave that finish the slab, four columns each
  constexpr int TL = kTokenLanes;
  static_assert(FT <= 64 && TL == 16, "the finish is written for one wave and sixteen token lanes");
  __shared__ __align__(16) float red[TL][SW];
  const int c = blockIdx.x % p.C, s = blockIdx.x / p.C, b = blockIdx.y;
  const int cl = threadIdx.x % kColLanes, tl = threadIdx.x / kColLanes;
  const int d = p.d;
  int64_t start = p.seq_start[b], n = p.seq_len[b];
  const int ten = p.tenant_id[b];
  if (!span_ok(start, n, p.M_tok) || ten < 0 || ten >= p.T_tenants) {
    if (blockIdx.x == 0) {
      if (threadIdx.x == 0) p.route_out[b] = MILORA_ROUTE_NONE;
      if (p.logits_out && threadIdx.x < MILORA_NUM_SITES)
        p.logits_out[b * MILORA_NUM_SITES + threadIdx.x] = __uint_as_float(0x7fc00000u);
    }
    return;
  }
  const bool is_max = p.pool == MILORA_POOL_MAX;
  float scale = is_max ? 1.0f : 1.0f / (float)n;
  if (p.pool == MILORA_POOL_LAST) {  // the average over the last valid row alone
    start += n - 1;
    n = 1;
    scale = 1.0f;
  }
  const int64_t per = (n + p.S - 1) / p.S;
  const int64_t t0 = start + (int64_t)s * per;
  int64_t t1 = t0 + per;
  if (t1 > start + n) t1 = start + n;

  // ---- the finishing lanes ask for their router weights first: the values arrive while the rows stream
  const int f = threadIdx.x;
  const int fcol = c * SW + 4 * f;
  float wr[MILORA_NUM_SITES][4];
#pragma unroll
  for (int j = 0; j < MILORA_NUM_SITES; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) wr[j][v] = 0.f;
  if (f < FT) {
    const T* wt = p.Wr + (size_t)ten * MILORA_NUM_SITES * d;
#pragma unroll
    for (int j = 0; j < MILORA_NUM_SITES; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (fcol + v < d) wr[j][v] = Elem<T>::load(wt, (size_t)j * d + fcol + v);
  }

  // ---- pool the slice: token lane tl takes rows t0 + tl, t0 + tl + 16, ...
  const int col = c * SW + cl * VEC;
  const float ident = is_max ? -INFINITY : 0.f;
  float acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = ident;
  if (col < d) {
    const T* q = p.H + col;
    int64_t t = t0 + tl;
    for (; t + 7 * TL < t1; t += 8 * TL) {
      float x[8][VEC];
#pragma unroll
      for (int u = 0; u < 8; ++u) VecLoad<T, VEC>::load_once(q + (size_t)(t + u * TL) * d, x[u]);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        if (is_max)
          acc[v] = fmaxf(acc[v], fmaxf(fmaxf(fmaxf(x[0][v], x[1][v]), fmaxf(x[2][v], x[3][v])),
                                       fmaxf(fmaxf(x[4][v], x[5][v]), fmaxf(x[6][v], x[7][v]))));
        else
          acc[v] += ((x[0][v] + x[1][v]) + (x[2][v] + x[3][v])) + ((x[4][v] + x[5][v]) + (x[6][v] + x[7][v]));
      }
    }
    for (; t < t1; t += TL) {
      float x0[VEC];
      VecLoad<T, VEC>::load_once(q + (size_t)t * d, x0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = is_max ? fmaxf(acc[v], x0[v]) : acc[v] + x0[v];
    }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) red[tl][cl * VEC + v] = acc[v];
  __syncthreads();
  if (threadIdx.x >= 64) return;  // the first wave finishes
  const int lane = threadIdx.x;

  f32x4 h = {ident, ident, ident, ident};
  if (f < FT) {
    f32x4 r[TL];
#pragma unroll
    for (int i = 0; i < TL; ++i) r[i] = *reinterpret_cast<const f32x4*>(&red[i][4 * f]);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if (is_max)
        h[v] = fmaxf(fmaxf(fmaxf(fmaxf(r[0][v], r[1][v]), fmaxf(r[2][v], r[3][v])),
                           fmaxf(fmaxf(r[4][v], r[5][v]), fmaxf(r[6][v], r[7][v]))),
                     fmaxf(fmaxf(fmaxf(r[8][v], r[9][v]), fmaxf(r[10][v], r[11][v])),
                           fmaxf(fmaxf(r[12][v], r[13][v]), fmaxf(r[14][v], r[15][v]))));
      else
        h[v] = (((r[0][v] + r[1][v]) + (r[2][v] + r[3][v])) + ((r[4][v] + r[5][v]) + (r[6][v] + r[7][v]))) +
               (((r[8][v] + r[9][v]) + (r[10][v] + r[11][v])) + ((r[12][v] + r[13][v]) + (r[14][v] + r[15][v])));
    }
  }
  if (p.S > 1) {
    // slab sums of this slice to memory, then the flag; whoever then finds every slice's flag adds the slices up
    f32x4* mine = reinterpret_cast<f32x4*>(p.partial + (((size_t)b * p.C + c) * p.S + s) * SW);
    if (f < FT) st_through(mine + f, h);
    wait_all_mem();
    u32x2* flags = p.arrived + ((size_t)b * p.C + c) * p.S;
    if (lane == 0) st_through(flags + s, u32x2{p.tag_lo, p.tag_hi});
    wait_all_mem();
    bool all = true;
    for (int i = lane; i < p.S; i += 64) {
      const u32x2 g = ld_through(flags + i);
      all = all && g[0] == p.tag_lo && g[1] == p.tag_hi;
    }
    if (__builtin_amdgcn_readfirstlane(__ballot(all) != ~0ull)) return;
    // Two slices that store their flags at the same time both find every flag.  Only one may go on: the second would
    // store the slab's share again after the request's finishing wave has wiped the shares, and a replay of a
    // recorded launch (same tag) would take that left-over share for the new one.  The one that takes the flag of
    // slice 0 away goes on.
    {
      unsigned long long old = 0ull;
      if (lane == 0)
        old = __hip_atomic_exchange(reinterpret_cast<unsigned long long*>(flags), 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t old_lo = __builtin_amdgcn_readfirstlane((uint32_t)old), old_hi = __builtin_amdgcn_readfirstlane((uint32_t)(old >> 32));
      if (old_lo != p.tag_lo || old_hi != p.tag_hi) return;
    }
    for (int i = lane; i < p.S; i += 64) st_through(flags + i, u32x2{0u, 0u});
    if (f < FT) {
      const f32x4* base = reinterpret_cast<const f32x4*>(p.partial + ((size_t)b * p.C + c) * p.S * SW) + f;
      f32x4 tot = {ident, ident, ident, ident};
      for (int s0 = 0; s0 < p.S; s0 += 8) {
        const f32x4* q8[8];
        f32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) q8[u] = base + (size_t)(s0 + u < p.S ? s0 + u : p.S - 1) * FT;
        ld_through8(q8, x);
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (s0 + u >= p.S) x[u] = f32x4{ident, ident, ident, ident};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          if (is_max)
            tot[v] = fmaxf(tot[v], fmaxf(fmaxf(fmaxf(x[0][v], x[1][v]), fmaxf(x[2][v], x[3][v])),
                                         fmaxf(fmaxf(x[4][v], x[5][v]), fmaxf(x[6][v], x[7][v]))));
          else
            tot[v] += ((x[0][v] + x[1][v]) + (x[2][v] + x[3][v])) + ((x[4][v] + x[5][v]) + (x[6][v] + x[7][v]));
        }
      }
      h = tot;
    }
  }

  // ---- z = g(h); the slab's share of the seven logits, summed over the lanes (every lane ends with the sums)
  float lg[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) lg[j] = 0.f;
  if (f < FT) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if (fcol + v < d) {
        const float z = activate(h[v] * scale, p.act, p.coef);
#pragma unroll
        for (int j = 0; j < MILORA_NUM_SITES; ++j) lg[j] += z * wr[j][v];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < MILORA_NUM_SITES; ++j)
    for (int off = 32; off > 0; off >>= 1) lg[j] += __shfl_xor(lg[j], off, 64);

  if (p.C > 1) {
    // unit u of the slab: logits 2u and 2u + 1 with the tag.  Lane i takes units i, i + 64, ...: always unit i % 4,
    // of slabs i / 4, i / 4 + 16, ...; the sixteen running sums of a unit are then added across the lanes.
    u32x4* units = p.share + (size_t)b * p.C * 4;
    if (lane < 4) {
      float e0 = 0.f, e1 = 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (lane == u) { e0 = lg[2 * u]; e1 = lg[2 * u + 1]; }
      st_through(units + c * 4 + lane, u32x4{__float_as_uint(e0), __float_as_uint(e1), p.tag_lo, p.tag_hi});
    }
    wait_all_mem();
    bool all = true;
    float a0 = 0.f, a1 = 0.f;
    for (int i = lane; i < 4 * p.C; i += 64) {
      const u32x4 g = ld_through(units + i);
      all = all && g[2] == p.tag_lo && g[3] == p.tag_hi;
      a0 += __uint_as_float(g[0]);
      a1 += __uint_as_float(g[1]);
    }
    if (__builtin_amdgcn_readfirstlane(__ballot(all) != ~0ull)) return;
    for (int i = lane; i < 4 * p.C; i += 64) st_through(units + i, u32x4{0u, 0u, 0u, 0u});
    for (int off = 4; off < 64; off <<= 1) {
      a0 += __shfl_xor(a0, off, 64);
      a1 += __shfl_xor(a1, off, 64);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      lg[2 * u] = __shfl(a0, u, 64);
      lg[2 * u + 1] = __shfl(a1, u, 64);
    }
  }
  float logit[MILORA_NUM_SITES];
#pragma unroll
  for (int j = 0; j < MILORA_NUM_SITES; ++j) logit[j] = lg[j];
  if (lane == 0) {
    if (p.logits_out)
      for (int j = 0; j < MILORA_NUM_SITES; ++j) p.logits_out[b * MILORA_NUM_SITES + j] = logit[j];
    p.route_out[b] = select_route(logit, p.top_k);
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

// Finish of the self-attention pooler: one workgroup of 1024 threads per request merges the slices (each holds a
// sum weighted by exp(u - m_s): brought to the common maximum and normalised), then z = g(h), the seven logits and
// the selection.  A thread owns four neighbouring columns; the S slice sums of a column are added as eight
// interleaved running sums (slice s goes to sum s % 8) that are combined pairwise at the end, so eight loads are
// in flight and the order is fixed.
constexpr int kFinishThreads = 1024;
constexpr int kFinishWays = 8;

template <typename T>
__global__ void __launch_bounds__(kFinishThreads) selfattn_finish_kernel(int64_t M_tok, int d,
                                                                         const int32_t* __restrict__ seq_start,
                                                                         const int32_t* __restrict__ seq_len,
                                                                         const int32_t* __restrict__ tenant_id,
                                                                         int T_tenants, const T* __restrict__ Wr,
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
  const bool vec = (d % 4) == 0;  // rows of `partial` are then 16-byte aligned
  const float* pb = partial + (size_t)b * S * d;
  {
    const float* mlb = ml + (size_t)b * S * 2;
    float mx = -INFINITY, z = 0.f;
    for (int s = 0; s < S; ++s) mx = fmaxf(mx, mlb[2 * s]);
    for (int s = 0; s < S; ++s) z += mlb[2 * s + 1] * expf(mlb[2 * s] - mx);
    if (threadIdx.x < S) wts[threadIdx.x] = mlb[2 * threadIdx.x + 1] > 0.f ? expf(mlb[2 * threadIdx.x] - mx) / z : 0.f;
  }
  __syncthreads();
  for (int i0 = threadIdx.x * 4; i0 < d; i0 += kFinishThreads * 4) {
    const int nv = d - i0 < 4 ? d - i0 : 4;
    float h[4];
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
          float x[4] = {0.f, 0.f, 0.f, 0.f};
          if (vec) {
            const float4 x4 = *reinterpret_cast<const float4*>(q);
            x[0] = x4.x; x[1] = x4.y; x[2] = x4.z; x[3] = x4.w;
          } else {
            for (int v = 0; v < nv; ++v) x[v] = q[v];
          }
          const float wgt = wts[s0 + u];
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (wgt != 0.f) run[u][v] += wgt * x[v];  // a slice without tokens holds nothing to read
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v)
      h[v] = ((run[0][v] + run[1][v]) + (run[2][v] + run[3][v])) + ((run[4][v] + run[5][v]) + (run[6][v] + run[7][v]));
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
    route_out[b] = select_route(logit, top_k);
  }
}

// Token slices per request of the self-attention pooler.
int pick_splits(int B, int64_t M_tok) {
  int64_t avg = (M_tok + B - 1) / B;
  int64_t s = (4096 + B - 1) / B;  // aim at a few thousand workgroups
  if (s > (avg + 15) / 16) s = (avg + 15) / 16;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  return (int)s;
}

// Token slices per request of pool_route_kernel with C column slabs: one, unless the requests are so few that
// compute units would be left without work; none shorter than 64 rows.  (Slices of a fixed 256 rows, eight per
// 2048-token prompt, measured a third slower than two: every cut adds the hand-over through memory.)
int pick_slices(int B, int C, int64_t M_tok) {
  const int64_t avg = (M_tok + B - 1) / B;
  int64_t s = (512 + (int64_t)B * C - 1) / ((int64_t)B * C);
  if (s > (avg + 63) / 64) s = (avg + 63) / 64;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  return (int)s;
}

// Workspace of pool_route_kernel: slab sums of the slices, their flags, the slabs' logit shares.
struct PoolRouteCarve {
  int S, C;
  size_t partial, arrived, share, total;  // byte offsets, and the size
};
PoolRouteCarve carve_pool_route(int B, int d, int64_t M_tok, int slab_cols, bool last_only) {
  PoolRouteCarve c;
  c.C = (d + slab_cols - 1) / slab_cols;
  c.S = last_only ? 1 : pick_slices(B, c.C, M_tok);
  c.partial = 0;
  c.arrived = align_up((size_t)B * c.C * c.S * slab_cols * sizeof(float), 256);
  c.share = c.arrived + align_up((size_t)B * c.C * c.S * 8, 256);
  c.total = c.share + align_up((size_t)B * c.C * 4 * 16, 256);
  return c;
}

std::atomic<uint32_t> g_route_calls{0};

template <typename T, int VEC>
int launch_pool_route(PoolRouteArgs<T> a, int B, int64_t M_tok, void* workspace, size_t workspace_bytes,
                      hipStream_t st) {
  const PoolRouteCarve cv = carve_pool_route(B, a.d, M_tok, kColLanes * VEC, a.pool == MILORA_POOL_LAST);
  if (!workspace || workspace_bytes < cv.total) return MILORA_EWORKSPACE;
  if ((size_t)cv.C * cv.S > 65535u * 32u) return MILORA_ERANGE;
  a.S = cv.S;
  a.C = cv.C;
  a.tag_hi = ++g_route_calls;
  a.tag_lo = (a.tag_hi * 2654435761u ^ 0x9e3779b9u) | 1u;
  a.partial = (float*)((char*)workspace + cv.partial);
  a.arrived = (u32x2*)((char*)workspace + cv.arrived);
  a.share = (u32x4*)((char*)workspace + cv.share);
  hipLaunchKernelGGL((pool_route_kernel<T, VEC>), dim3(cv.C * cv.S, B), dim3(kPoolThreads), 0, st, a);
  return check_launch();
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
  size_t need = partial_bytes(B, S, d) + align_up((size_t)B * S * 2 * sizeof(float), 256);  // self-attention pooler
  for (int slab_cols : {32, 128, 256}) {  // the slab widths pool_route_kernel is built for
    const size_t n = carve_pool_route(B, d, M_tok, slab_cols, false).total;
    if (n > need) need = n;
  }
  return need;
}

namespace {

template <typename T>
int route_typed(const void* H, int64_t M_tok, int d, const int32_t* seq_start, const int32_t* seq_len,
                const int32_t* tenant_id, int B, int n_tenants, const void* Wr, int pool, int act, const void* w_sa,
                const RationalCoef& coef, int top_k, uint8_t* route_out, float* logits_out, void* workspace,
                size_t workspace_bytes, hipStream_t st) {
  constexpr int VEC = 16 / (int)sizeof(T);  // elements of a 16-byte load
  const bool vec = ((uintptr_t)H % 16) == 0 && d % VEC == 0;
  if (pool == MILORA_POOL_SELFATTN) {
    if (workspace_bytes < milora_route_workspace_bytes(B, d, M_tok)) return MILORA_EWORKSPACE;
    const int S = pick_splits(B, M_tok);
    float* partial = (float*)workspace;
    float* ml = (float*)((char*)workspace + partial_bytes(B, S, d));
    if (vec && ((uintptr_t)w_sa % 16) == 0)
      launch_selfattn<T, VEC>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
    else
      launch_selfattn<T, 1>(H, M_tok, d, seq_start, seq_len, tenant_id, n_tenants, w_sa, B, S, partial, ml, st);
    int rc = check_launch();
    if (rc != MILORA_OK) return rc;
    hipLaunchKernelGGL((selfattn_finish_kernel<T>), dim3(B), dim3(kFinishThreads), 0, st, M_tok, d, seq_start, seq_len,
                       tenant_id, n_tenants, (const T*)Wr, act, coef, top_k, S, partial, ml, route_out, logits_out);
    return check_launch();
  }
  PoolRouteArgs<T> a;
  a.H = (const T*)H;
  a.M_tok = M_tok;
  a.d = d;
  a.seq_start = seq_start;
  a.seq_len = seq_len;
  a.tenant_id = tenant_id;
  a.T_tenants = n_tenants;
  a.Wr = (const T*)Wr;
  a.pool = pool;
  a.act = act;
  a.top_k = top_k;
  a.route_out = route_out;
  a.logits_out = logits_out;
  a.coef = coef;
  if (vec) return launch_pool_route<T, VEC>(a, B, M_tok, workspace, workspace_bytes, st);
  return launch_pool_route<T, 1>(a, B, M_tok, workspace, workspace_bytes, st);
}

}  // namespace

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
  if (!workspace) return MILORA_EWORKSPACE;
  RationalCoef coef = {};
  if (act == MILORA_ACT_RATIONAL) {
    for (int j = 0; j < 7; ++j) coef.a[j] = act_coef[j];
    for (int j = 0; j < 5; ++j) coef.b[j] = act_coef[7 + j];
  }
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MILORA_BF16)
    return route_typed<bf16_t>(H, M_tok, d, seq_start, seq_len, tenant_id, B, n_tenants, Wr, pool, act, w_sa, coef, top_k,
                               route_out, logits_out, workspace, workspace_bytes, st);
  return route_typed<float>(H, M_tok, d, seq_start, seq_len, tenant_id, B, n_tenants, Wr, pool, act, w_sa, coef, top_k,
                            route_out, logits_out, workspace, workspace_bytes, st);
}
