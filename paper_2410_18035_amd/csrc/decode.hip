// Decode-time routed LoRA linears on packed bf16 weights (paper Eq. 1; Sec. 3.3 route reuse).
//
// At decode the batch is skinny (B <= 128 rows) and every base weight is read exactly once per
// step, so the kernels are built around the HBM stream of W: weights are pre-packed in 1 KiB
// blocks that are already in 16x16x32 matrix-core operand order (a wave's load instruction
// fetches one contiguous block), a workgroup owns one 16-column output tile over the whole
// reduction length with its waves interleaved along k, and a register ring keeps D blocks per
// wave in flight.  The batch rows ride in the other MFMA operand, either straight from the
// caller's row-major activations or from a block-packed activation buffer an earlier kernel
// of the layer wrote.  The epilogue reduces the waves' partial tiles through LDS, adds the
// LoRA expand t W^B of the routed rows in fp32, and applies the layer glue (normalisation
// scale, residual, silu*up) before the single rounding to bf16.
#include "common.h"

namespace milora {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kShrinkChunk = 1024;  // reduction rows per shrink workgroup
constexpr int kTCache = 4096;       // floats of LDS that hold the t vectors of one group of routed rows
constexpr int kMaxRows = MILORA_MAX_DECODE_BATCH;

// Offset (in bf16 elements) of activation element (row m, feature k) in a block-packed buffer of MT row tiles.
__device__ __host__ __forceinline__ size_t packed_act_offset(int m, int k, int MT) {
  return ((((size_t)(k >> 5) * MT + (m >> 4)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

struct GemmParams {
  // input operand
  const bf16_t* X;  // row-major [M][K] or block-packed
  int K, M, Breq;
  int norm;  // scale every output row by rsqrt(mean(x_row^2) + 1e-5)
  // weight streams: up to three sites share X; with `pair` the workgroup takes tile j of W[0] and of W[1]
  int n_sites, pair;
  const bf16_t* W[3];
  int N[3], site[3], tile_end[3];
  // LoRA
  AdapterView ad;
  const int32_t* tenant_id;
  const uint8_t* route;
  const int32_t* row_to_req;
  const float* tpart;  // [n_sites][M][NC][r_max] partial shrink results, or null
  int NC;
  // epilogue
  const bf16_t* bias[3];
  const bf16_t* resid_bf16;
  const float* resid_f32;
  int ld_resid;
  float* out_f32;
  int ld_f32;
  bf16_t* out_rm[3];
  int ld_rm, col_off[3];
  bf16_t* out_pk[3];
  int silu_mul;
};

__device__ __forceinline__ float sumsq8(u32x4 v) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return s;
}

template <int MT, int NACC, int NW, int D, bool XPACKED, bool NORM>
__global__ void __launch_bounds__(NW * 64) decode_gemm_kernel(const GemmParams p) {
  constexpr int kThreads = NW * 64;
  constexpr int kRedSlots = NW / 2 > 0 ? NW / 2 : 1;
  __shared__ float red[kRedSlots * NACC * MT * 256];
  __shared__ float t_s[kTCache];
  __shared__ float ssq_s[NW * MT * 16];
  __shared__ int l_m[kMaxRows], l_r[kMaxRows], l_t[kMaxRows], l_a[kMaxRows];
  __shared__ int l_cnt;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, kept in a scalar register
  int si = 0, j = blockIdx.x;
  if (!p.pair) {
    while (si + 1 < p.n_sites && j >= p.tile_end[si]) ++si;
    if (si > 0) j -= p.tile_end[si - 1];
  }
  const int KT = p.K >> 5;
  const u32x4* wp[NACC];
#pragma unroll
  for (int a = 0; a < NACC; ++a)
    wp[a] = reinterpret_cast<const u32x4*>(p.W[p.pair ? a : si]) + (size_t)j * KT * 64 + lane;
  const u32x4* xp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (XPACKED) {
      xp[mt] = reinterpret_cast<const u32x4*>(p.X) + mt * 64 + lane;
    } else {
      int row = mt * 16 + (lane & 15);
      if (row > p.M - 1) row = p.M - 1;
      xp[mt] = reinterpret_cast<const u32x4*>(p.X + (size_t)row * p.K) + (lane >> 4);
    }
  }
  constexpr int kXStride = XPACKED ? MT * 64 : 4;  // u32x4 units between consecutive 32-wide k blocks

  f32x4 acc[NACC][MT];
  float ss[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    ss[mt] = 0.f;
#pragma unroll
    for (int a = 0; a < NACC; ++a) acc[a][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // this wave's k blocks: f = w, w + NW, ...  (the workgroup reads NW consecutive KiB per step)
  const int nf = (KT - w + NW - 1) / NW;
  u32x4 wb[D][NACC], xb[D][MT];
  auto issue = [&](int s, int i) {
    const size_t f = (size_t)w + (size_t)i * NW;
#pragma unroll
    for (int a = 0; a < NACC; ++a) wb[s][a] = __builtin_nontemporal_load(wp[a] + f * 64);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xb[s][mt] = xp[mt][f * kXStride];
  };
  auto consume = [&](int s) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const bf16x8 xv = __builtin_bit_cast(bf16x8, xb[s][mt]);
#pragma unroll
      for (int a = 0; a < NACC; ++a)
        acc[a][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wb[s][a]), xv, acc[a][mt], 0, 0, 0);
      if (NORM) ss[mt] += sumsq8(xb[s][mt]);
    }
  };
  if (nf >= 2 * D) {
    // Register ring of D blocks per stream.  The fill and the steady loop issue unconditionally, so the
    // number of loads in flight is the same on every path into a consume and the compiler can wait for
    // the oldest block only.
#pragma unroll
    for (int s = 0; s < D; ++s) {
      issue(s, s);
      __builtin_amdgcn_sched_barrier(0);  // the fill must reach memory oldest block first
    }
    int i0 = 0;
    for (; i0 + 2 * D <= nf; i0 += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        consume(s);
        issue(s, i0 + D + s);
        __builtin_amdgcn_sched_barrier(0);  // keep the refill next to its consume: no batching of the loads
      }
    }
#pragma unroll
    for (int s = 0; s < D; ++s) {
      consume(s);
      if (i0 + D + s < nf) issue(s, i0 + D + s);
    }
#pragma unroll
    for (int s = 0; s < D; ++s)
      if (i0 + D + s < nf) consume(s);
  } else {
    for (int i = 0; i < nf; ++i) {  // short reductions: no ring
      issue(0, i);
      consume(0);
    }
  }

  // ---- cross-wave reduction of the partial tiles (fixed order) -------------------------------
  auto red_idx = [&](int slot, int a, int mt, int i, int ln) { return (((slot * NACC + a) * MT + mt) * 4 + i) * 64 + ln; };
#pragma unroll
  for (int s = NW / 2; s >= 1; s >>= 1) {
    if (w >= s && w < 2 * s) {
#pragma unroll
      for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) red[red_idx(w - s, a, mt, i, lane)] = acc[a][mt][i];
    }
    __syncthreads();
    if (w < s) {
#pragma unroll
      for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[a][mt][i] += red[red_idx(w, a, mt, i, lane)];
    }
    __syncthreads();
  }
  if (w == 0) {
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[red_idx(0, a, mt, i, lane)] = acc[a][mt][i];
  }
  if (NORM) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float v = ss[mt];
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      if (lane < 16) ssq_s[(w * MT + mt) * 16 + lane] = v;
    }
  }
  if (tid == 0) l_cnt = 0;
  __syncthreads();

  // ---- LoRA expand of the rows routed to this tile's site(s), added to the fp32 sums ---------
  const int n0 = j * 16;
  if (p.tpart) {
    for (int m = tid; m < p.M; m += kThreads) {
      const int req = p.row_to_req ? p.row_to_req[m] : m;
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        int tenant = 0;
        const int r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, p.site[p.pair ? a : si], &tenant);
        if (r) {
          const int idx = atomicAdd(&l_cnt, 1);
          l_m[idx] = m; l_r[idx] = r; l_t[idx] = tenant; l_a[idx] = a;
        }
      }
    }
    __syncthreads();
    const int cnt = l_cnt, rmax = p.ad.r_max;
    int G = kTCache / rmax;
    if (G > kThreads / 8) G = kThreads / 8;
    for (int g0 = 0; g0 < cnt; g0 += G) {
      const int ng = cnt - g0 < G ? cnt - g0 : G;
      for (int e = tid; e < ng * rmax; e += kThreads) {
        const int gi = e / rmax, c = e - gi * rmax, idx = g0 + gi;
        if (c < l_r[idx]) {
          const int ts = p.pair ? l_a[idx] : si;
          const float* tp = p.tpart + (((size_t)ts * p.M + l_m[idx]) * p.NC) * rmax + c;
          float s = 0.f;
          for (int kc = 0; kc < p.NC; ++kc) s += tp[(size_t)kc * rmax];
          t_s[gi * rmax + c] = s;
        }
      }
      __syncthreads();
      const int gi = tid >> 3, pp = tid & 7;
      if (gi < ng) {
        const int idx = g0 + gi, m = l_m[idx], r = l_r[idx], a = l_a[idx];
        const int sidx = p.pair ? a : si;
        const bf16_t* Bm = (const bf16_t*)p.ad.B[l_t[idx] * MILORA_NUM_SITES + p.site[sidx]] + n0 + 2 * pp;
        const size_t ldb = (size_t)p.N[sidx];
        float d0 = 0.f, d1 = 0.f;
        if (((uintptr_t)Bm & 3) == 0 && (ldb & 1) == 0) {
          for (int c = 0; c < r; ++c) {
            const uint32_t bb = *reinterpret_cast<const uint32_t*>(Bm + (size_t)c * ldb);
            const float tv = t_s[gi * rmax + c];
            d0 += tv * __uint_as_float(bb << 16);
            d1 += tv * __uint_as_float(bb & 0xffff0000u);
          }
        } else {
          for (int c = 0; c < r; ++c) {
            const float tv = t_s[gi * rmax + c];
            d0 += tv * bf16_to_f32(Bm[(size_t)c * ldb]);
            d1 += tv * bf16_to_f32(Bm[(size_t)c * ldb + 1]);
          }
        }
        const int mt = m >> 4, nl = 2 * pp;
        red[red_idx(0, a, mt, nl & 3, (m & 15) + 16 * (nl >> 2))] += d0;
        red[red_idx(0, a, mt, (nl + 1) & 3, (m & 15) + 16 * ((nl + 1) >> 2))] += d1;
      }
      __syncthreads();
    }
  }

  // ---- glue and stores: thread (row m, column pair pp) ------------------------------------------
  const int pp = tid & 7;
  for (int m = tid >> 3; m < p.M; m += kThreads / 8) {
    const int mt = m >> 4;
    float inv = 1.f;
    if (NORM) {
      float s = 0.f;
      for (int ww = 0; ww < NW; ++ww) s += ssq_s[(ww * MT + mt) * 16 + (m & 15)];
      inv = rsqrtf(s / (float)p.K + 1e-5f);
    }
    float val[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int nl = 2 * pp + e;
      const int ln = (m & 15) + 16 * (nl >> 2);
      const float v0 = red[red_idx(0, 0, mt, nl & 3, ln)] * inv;
      if (NACC == 2 && p.silu_mul) val[e] = silu(v0) * (red[red_idx(0, NACC - 1, mt, nl & 3, ln)] * inv);
      else val[e] = v0;
    }
    const int n = n0 + 2 * pp;
    if (p.bias[si]) {
      val[0] += bf16_to_f32(p.bias[si][n]);
      val[1] += bf16_to_f32(p.bias[si][n + 1]);
    }
    if (p.resid_bf16) {
      const uint32_t rr = *reinterpret_cast<const uint32_t*>(p.resid_bf16 + (size_t)m * p.ld_resid + n);
      val[0] += __uint_as_float(rr << 16);
      val[1] += __uint_as_float(rr & 0xffff0000u);
    }
    if (p.resid_f32) {
      const float2 rr = *reinterpret_cast<const float2*>(p.resid_f32 + (size_t)m * p.ld_resid + n);
      val[0] += rr.x;
      val[1] += rr.y;
    }
    if (p.out_f32) *reinterpret_cast<float2*>(p.out_f32 + (size_t)m * p.ld_f32 + n) = make_float2(val[0], val[1]);
    const uint32_t packed = pack_bf16x2(val[0], val[1]);
    if (p.out_rm[si]) *reinterpret_cast<uint32_t*>(p.out_rm[si] + (size_t)m * p.ld_rm + p.col_off[si] + n) = packed;
    if (p.out_pk[si]) *reinterpret_cast<uint32_t*>(p.out_pk[si] + packed_act_offset(m, n, MT)) = packed;
  }
}

// LoRA shrink at decode: workgroup (k chunk, row, site slot) forms the partial t = x[chunk] . A[chunk]
// of one routed row; non-routed rows exit at once.  tpart[slot][m][kc][0..r).
template <int MT, bool XPACKED>
__global__ void __launch_bounds__(256) decode_shrink_kernel(const bf16_t* __restrict__ X, int K, int M, int Breq,
                                                            AdapterView ad, int n_sites, int s0, int s1, int s2,
                                                            const int32_t* __restrict__ tenant_id,
                                                            const uint8_t* __restrict__ route,
                                                            const int32_t* __restrict__ row_to_req, int NC,
                                                            float* __restrict__ tpart) {
  __shared__ float red[256 * 8];
  const int kc = blockIdx.x, m = blockIdx.y, slot = blockIdx.z;
  const int site = slot == 0 ? s0 : (slot == 1 ? s1 : s2);
  const int req = row_to_req ? row_to_req[m] : m;
  int tenant = 0;
  const int r = routed_rank(ad, tenant_id, route, req, Breq, site, &tenant);
  if (r == 0) return;
  const bf16_t* A = (const bf16_t*)ad.A[tenant * MILORA_NUM_SITES + site];
  const int k_lo = kc * kShrinkChunk;
  const int k_hi = k_lo + kShrinkChunk < K ? k_lo + kShrinkChunk : K;
  float* out = tpart + (((size_t)slot * M + m) * NC + kc) * ad.r_max;
  auto xval = [&](int k) -> float {
    return bf16_to_f32(XPACKED ? X[packed_act_offset(m, k, MT)] : X[(size_t)m * K + k]);
  };
  const int tid = threadIdx.x;
  if ((r & 7) == 0 && ((uintptr_t)A & 15) == 0) {
    const int lpr = r >> 3, rpp = 256 / lpr;  // lanes per row of A, rows per pass
    const int cg = tid % lpr, kr = tid / lpr;
    float acc[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) acc[v] = 0.f;
    if (kr < rpp) {
      const u32x4* Ap = reinterpret_cast<const u32x4*>(A) + cg;
      int k = k_lo + kr;
      for (; k + 3 * rpp < k_hi; k += 4 * rpp) {
        u32x4 a[4];
        float x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          a[u] = __builtin_nontemporal_load(Ap + (size_t)(k + u * rpp) * lpr);
          x[u] = xval(k + u * rpp);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            acc[2 * v] += x[u] * __uint_as_float(a[u][v] << 16);
            acc[2 * v + 1] += x[u] * __uint_as_float(a[u][v] & 0xffff0000u);
          }
      }
      for (; k < k_hi; k += rpp) {
        const u32x4 a = Ap[(size_t)k * lpr];
        const float x = xval(k);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          acc[2 * v] += x * __uint_as_float(a[v] << 16);
          acc[2 * v + 1] += x * __uint_as_float(a[v] & 0xffff0000u);
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) red[tid * 8 + v] = acc[v];
    __syncthreads();
    if (tid < r) {
      const int g = tid >> 3, v = tid & 7;
      float s = 0.f;
      for (int q = 0; q < rpp; ++q) s += red[(q * lpr + g) * 8 + v];
      out[tid] = s;
    }
  } else {
    int rpad = 1;
    while (rpad < r) rpad <<= 1;
    const int c = tid % rpad, kr = tid / rpad, rpp = 256 / rpad;
    float acc = 0.f;
    if (c < r)
      for (int k = k_lo + kr; k < k_hi; k += rpp) acc += xval(k) * bf16_to_f32(A[(size_t)k * r + c]);
    red[tid] = acc;
    __syncthreads();
    if (kr == 0 && c < r) {
      float s = 0.f;
      for (int q = 0; q < rpp; ++q) s += red[q * rpad + c];
      out[c] = s;
    }
  }
}

// Row-major [d2][d1] -> packed blocks (see milora_wlayout): one thread per 16-byte group of 8 inputs.
__global__ void __launch_bounds__(256) pack_weight_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int d1,
                                                          int d2) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;  // index of the 8-element group in dst
  const size_t total = (size_t)d1 * d2 / 8;
  if (g >= total) return;
  const int KT = d1 >> 5;
  const size_t blk = g >> 6;
  const int ln = (int)(g & 63);
  const int nt = (int)(blk / KT), kt = (int)(blk % KT);
  const int jrow = nt * 16 + (ln & 15), i0 = kt * 32 + (ln >> 4) * 8;
  dst[g] = src[((size_t)jrow * d1 + i0) / 8];
}

// Row-major bf16 activations [M][K] -> block-packed buffer (used when a caller-supplied tensor feeds
// a single-tile phase, where the strided operand pattern would throttle the vector memory pipe).
template <int MT>
__global__ void __launch_bounds__(256) pack_act_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int M, int K) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total = (size_t)(K >> 5) * MT * 64;
  if (g >= total) return;
  const int ln = (int)(g & 63);
  const size_t blk = g >> 6;
  const int mt = (int)(blk % MT), kt = (int)(blk / MT);
  int row = mt * 16 + (ln & 15);
  if (row > M - 1) row = M - 1;
  dst[g] = src[((size_t)row * K + kt * 32 + (ln >> 4) * 8) / 8];
}

template <int MT, int NACC, bool XPACKED>
void launch_gemm_t(const GemmParams& p, int tiles, hipStream_t st) {
  constexpr int NW = 4;
  constexpr int D = MT <= 2 ? 8 : (MT == 4 ? 6 : 4);
  if (p.norm) hipLaunchKernelGGL((decode_gemm_kernel<MT, NACC, NW, D, XPACKED, true>), dim3(tiles), dim3(NW * 64), 0, st, p);
  else hipLaunchKernelGGL((decode_gemm_kernel<MT, NACC, NW, D, XPACKED, false>), dim3(tiles), dim3(NW * 64), 0, st, p);
}

template <int MT>
void launch_gemm_mt(const GemmParams& p, int tiles, bool xpacked, hipStream_t st) {
  if (p.pair) {
    if (xpacked) launch_gemm_t<MT, 2, true>(p, tiles, st); else launch_gemm_t<MT, 2, false>(p, tiles, st);
  } else {
    if (xpacked) launch_gemm_t<MT, 1, true>(p, tiles, st); else launch_gemm_t<MT, 1, false>(p, tiles, st);
  }
}

int launch_gemm(const GemmParams& p, int MT, bool xpacked, hipStream_t st) {
  const int tiles = p.pair ? p.N[0] / 16 : p.tile_end[p.n_sites - 1];
  switch (MT) {
    case 1: launch_gemm_mt<1>(p, tiles, xpacked, st); break;
    case 2: launch_gemm_mt<2>(p, tiles, xpacked, st); break;
    case 4: launch_gemm_mt<4>(p, tiles, xpacked, st); break;
    default: launch_gemm_mt<8>(p, tiles, xpacked, st); break;
  }
  return check_launch();
}

int launch_decode_shrink(const bf16_t* X, bool xpacked, int MT, int K, int M, int Breq, const AdapterView& ad,
                         int n_sites, const int* sites, const int32_t* tenant_id, const uint8_t* route,
                         const int32_t* row_to_req, int NC, float* tpart, hipStream_t st) {
  dim3 grid(NC, M, n_sites);
  const int s0 = sites[0], s1 = n_sites > 1 ? sites[1] : 0, s2 = n_sites > 2 ? sites[2] : 0;
#define MILORA_SHRINK(MTV, XP)                                                                                     \
  hipLaunchKernelGGL((decode_shrink_kernel<MTV, XP>), grid, dim3(256), 0, st, X, K, M, Breq, ad, n_sites, s0, s1, s2, \
                     tenant_id, route, row_to_req, NC, tpart)
  if (!xpacked) MILORA_SHRINK(1, false);
  else if (MT == 1) MILORA_SHRINK(1, true);
  else if (MT == 2) MILORA_SHRINK(2, true);
  else if (MT == 4) MILORA_SHRINK(4, true);
  else MILORA_SHRINK(8, true);
#undef MILORA_SHRINK
  return check_launch();
}

int mt_for(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : (M <= 64 ? 4 : 8)); }
int shrink_chunks(int K) { return (K + kShrinkChunk - 1) / kShrinkChunk; }

}  // namespace

// ---- workspace layout of the packed-weight decode paths -------------------------------------------
struct DecodeWs {
  float* tpart;    // [3][M][NCmax][r_max]
  float* h_f32;    // [M][d]
  bf16_t* pk_a;    // packed, K = max(d, F): a = v (or attn_out), later m = silu(g) * u
  bf16_t* pk_b;    // packed, K = d       : h
  size_t bytes;
};

static DecodeWs carve_decode_ws(void* base, int M, int d, int F, int r_max) {
  const int MT = mt_for(M);
  const int ncmax = shrink_chunks(F > d ? F : d);
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_t = take((size_t)3 * M * ncmax * r_max * sizeof(float));
  const size_t o_h = take((size_t)M * d * sizeof(float));
  const size_t o_a = take((size_t)MT * 16 * (F > d ? F : d) * sizeof(bf16_t));
  const size_t o_b = take((size_t)MT * 16 * d * sizeof(bf16_t));
  char* b = (char*)base;
  return DecodeWs{(float*)(b + o_t), (float*)(b + o_h), (bf16_t*)(b + o_a), (bf16_t*)(b + o_b), off};
}

size_t decode_packed_workspace_bytes(int M, int d, int F, int r_max) { return carve_decode_ws(nullptr, M, d, F, r_max).bytes; }

static void clear_epilogue(GemmParams& p) {
  for (int s = 0; s < 3; ++s) {
    p.W[s] = nullptr; p.N[s] = 0; p.site[s] = 0; p.tile_end[s] = 0;
    p.bias[s] = nullptr; p.out_rm[s] = nullptr; p.out_pk[s] = nullptr; p.col_off[s] = 0;
  }
  p.resid_bf16 = nullptr; p.resid_f32 = nullptr; p.ld_resid = 0;
  p.out_f32 = nullptr; p.ld_f32 = 0; p.ld_rm = 0; p.silu_mul = 0; p.pair = 0; p.norm = 0;
  p.tpart = nullptr; p.NC = 0; p.row_to_req = nullptr;
}

// One decode step of a layer on packed weights: four dependency levels, each a shrink launch for the
// rows routed to that level's sites followed by one weight-streaming launch.  With `marks`, an event is
// recorded after every launch (slot order: shrink, gemm of level 0, 1, 2, 3).
int layer_decode_packed(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                        const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                        bf16_t* y, bf16_t* qkv_out, void* workspace, hipStream_t st, LaunchMarks* marks) {
  const int MT = mt_for(B);
  auto mark = [&](int slot) {
    if (marks && slot < marks->n) (void)hipEventRecord(marks->ev[slot], st);
  };
  DecodeWs ws = carve_decode_ws(workspace, B, d, F, ad.r_max);
  const int norm = (flags & MILORA_LAYER_RMSNORM) ? 1 : 0;
  GemmParams p;
  int rc;
  auto common = [&](const bf16_t* X, int K) {
    clear_epilogue(p);
    p.X = X; p.K = K; p.M = B; p.Breq = B;
    p.ad = ad; p.tenant_id = tenant_id; p.route = route;
    p.tpart = ws.tpart; p.NC = shrink_chunks(K);
  };
  // level 0: q, k, v from x
  {
    const int sites[3] = {0, 1, 2};
    rc = launch_decode_shrink(x, false, MT, d, B, B, ad, 3, sites, tenant_id, route, nullptr, shrink_chunks(d), ws.tpart, st);
    if (rc) return rc;
    mark(0);
    common(x, d);
    p.n_sites = 3; p.norm = norm;
    for (int s = 0; s < 3; ++s) {
      p.W[s] = (const bf16_t*)wts->W[s]; p.N[s] = d; p.site[s] = s; p.tile_end[s] = (s + 1) * (d / 16);
      p.out_rm[s] = qkv_out; p.col_off[s] = s * d;
    }
    p.ld_rm = 3 * d;
    if (!attn_out) p.out_pk[2] = ws.pk_a;
    rc = launch_gemm(p, MT, false, st);
    if (rc) return rc;
    mark(1);
  }
  // level 1: h = x + L_o(a)
  {
    const bf16_t* a_in = ws.pk_a;
    if (attn_out) {
      const size_t groups = (size_t)(d >> 5) * MT * 64;
      const unsigned blocks = (unsigned)((groups + 255) / 256);
      switch (MT) {
        case 1: hipLaunchKernelGGL(pack_act_kernel<1>, dim3(blocks), dim3(256), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        case 2: hipLaunchKernelGGL(pack_act_kernel<2>, dim3(blocks), dim3(256), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        case 4: hipLaunchKernelGGL(pack_act_kernel<4>, dim3(blocks), dim3(256), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        default: hipLaunchKernelGGL(pack_act_kernel<8>, dim3(blocks), dim3(256), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
      }
      if ((rc = check_launch())) return rc;
    }
    const int sites[1] = {3};
    rc = launch_decode_shrink(a_in, true, MT, d, B, B, ad, 1, sites, tenant_id, route, nullptr, shrink_chunks(d), ws.tpart, st);
    if (rc) return rc;
    mark(2);
    common(a_in, d);
    p.n_sites = 1;
    p.W[0] = (const bf16_t*)wts->W[3]; p.N[0] = d; p.site[0] = 3; p.tile_end[0] = d / 16;
    p.resid_bf16 = x; p.ld_resid = d;
    p.out_f32 = ws.h_f32; p.ld_f32 = d;
    // other workgroups may still be reading a while this one stores, so h goes to the second buffer
    p.out_pk[0] = ws.pk_b;
    rc = launch_gemm(p, MT, true, st);
    if (rc) return rc;
    mark(3);
  }
  // level 2: m = silu(L_gate(n(h))) * L_up(n(h))
  {
    const int sites[2] = {4, 5};
    rc = launch_decode_shrink(ws.pk_b, true, MT, d, B, B, ad, 2, sites, tenant_id, route, nullptr, shrink_chunks(d), ws.tpart, st);
    if (rc) return rc;
    mark(4);
    common(ws.pk_b, d);
    p.n_sites = 2; p.pair = 1; p.silu_mul = 1; p.norm = norm;
    for (int s = 0; s < 2; ++s) { p.W[s] = (const bf16_t*)wts->W[4 + s]; p.N[s] = F; p.site[s] = 4 + s; }
    p.tile_end[0] = F / 16; p.tile_end[1] = F / 16;
    p.out_pk[0] = ws.pk_a;
    rc = launch_gemm(p, MT, true, st);
    if (rc) return rc;
    mark(5);
  }
  // level 3: y = h + L_down(m)
  {
    const int sites[1] = {6};
    rc = launch_decode_shrink(ws.pk_a, true, MT, F, B, B, ad, 1, sites, tenant_id, route, nullptr, shrink_chunks(F), ws.tpart, st);
    if (rc) return rc;
    mark(6);
    common(ws.pk_a, F);
    p.n_sites = 1;
    p.W[0] = (const bf16_t*)wts->W[6]; p.N[0] = d; p.site[0] = 6; p.tile_end[0] = d / 16;
    p.resid_f32 = ws.h_f32; p.ld_resid = d;
    p.out_rm[0] = y; p.ld_rm = d; p.col_off[0] = 0;
    rc = launch_gemm(p, MT, true, st);
    if (rc) return rc;
    mark(7);
  }
  return MILORA_OK;
}

// One routed linear of M <= 128 rows on a packed weight.
int routed_linear_packed(const bf16_t* X, int M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                         const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                         const uint8_t* route, int B, bf16_t* Y, void* workspace, hipStream_t st) {
  const int MT = mt_for(M);
  float* tpart = (float*)workspace;
  const int NC = shrink_chunks(d1);
  const int sites[1] = {site};
  int rc = launch_decode_shrink(X, false, MT, d1, M, B, ad, 1, sites, tenant_id, route, row_to_req, NC, tpart, st);
  if (rc) return rc;
  GemmParams p;
  clear_epilogue(p);
  p.X = X; p.K = d1; p.M = M; p.Breq = B;
  p.ad = ad; p.tenant_id = tenant_id; p.route = route; p.row_to_req = row_to_req;
  p.tpart = tpart; p.NC = NC;
  p.n_sites = 1;
  p.W[0] = W; p.N[0] = d2; p.site[0] = site; p.tile_end[0] = d2 / 16;
  p.bias[0] = bias;
  p.out_rm[0] = Y; p.ld_rm = d2;
  return launch_gemm(p, MT, false, st);
}

size_t routed_linear_packed_workspace_bytes(int M, int d1, int r_max) {
  return align_up((size_t)M * shrink_chunks(d1) * r_max * sizeof(float), 256);
}

int pack_weight(const void* src, void* dst, int d1, int d2, hipStream_t st) {
  const size_t groups = (size_t)d1 * d2 / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, (const u32x4*)src,
                     (u32x4*)dst, d1, d2);
  return check_launch();
}

}  // namespace milora
