// Decode-time routed LoRA linears on packed bf16 weights (paper Eq. 1; Sec. 3.3 route reuse).
//
// At decode the batch is skinny (B <= 128 rows) and every base weight is read exactly once per
// step, so everything is built around the HBM stream of W.  Weights are pre-packed in 1 KiB blocks
// that already are 16x16x32 matrix-core operands (one wave load = one contiguous block).  One launch
// covers one dependency level of the layer (q,k,v | o | gate,up | down) and holds two kinds of
// workgroups:
//   * LoRA workgroups (lowest block indices, so they are dispatched first and never wait): each
//     forms the partial shrink t = x[chunk] . A[chunk] of one routed row, publishes it and bumps
//     that row's counter;
//   * stream workgroups: each owns a group of four 16-column tiles and a slice of the reduction
//     length, its four waves interleaved along k.  The batch rows ride in the other MFMA operand
//     and are loaded once per k block for all four tiles.  A register ring keeps D blocks per
//     stream in flight.  Slices of one group are summed, in slice order, by whichever workgroup
//     of the group finishes last; that workgroup waits (bounded) for the counters of the routed
//     rows, adds the LoRA expand t W^B in fp32, applies the layer glue (normalisation scale,
//     residual, silu*up) and rounds once to bf16.
// Data handed from one workgroup to another (shrink partials, slice partials) is written and read
// with agent-scope atomic stores and loads, which go through to memory that all XCDs share instead
// of staying in one XCD's L2; the producer waits for its stores, passes a workgroup barrier and
// bumps an agent-scope counter, the consumer reads the counter before the data.  No cache-wide
// write-back or invalidate is needed.  All sums run in a fixed order: results do not depend on timing.
#include "common.h"

namespace milora {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kNT = 4;              // 16-column tiles (weight streams) per stream workgroup
constexpr int kShrinkChunk = 1024;  // reduction rows per LoRA workgroup
constexpr int kMaxRows = MILORA_MAX_DECODE_BATCH;
constexpr int kMaxGroups = 2048;    // column groups per level the counters are sized for
constexpr int kSpinLimit = 1 << 22; // polls of a counter before a workgroup gives up on a row's LoRA term

// Offset (in bf16 elements) of activation element (row m, feature k) in a block-packed buffer of MT row tiles.
__device__ __host__ __forceinline__ size_t packed_act_offset(int m, int k, int MT) {
  return ((((size_t)(k >> 5) * MT + (m >> 4)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

struct LevelParams {
  // input operand
  const bf16_t* X;  // row-major [M][K] or block-packed
  int K, M, Breq;
  // weight segments: up to three sites share X.  Column groups never straddle segments.
  // pair = 1 (gate, up): group g holds tiles 2g, 2g+1 of W[0] and of W[1].
  int n_seg, pair;
  const bf16_t* W[3];
  int N[3], site[3], grp_end[3];
  int S;            // reduction slices per group
  // LoRA
  AdapterView ad;
  const int32_t* tenant_id;
  const uint8_t* route;
  const int32_t* row_to_req;
  int n_lora_wg, NC;
  float* tpart;     // [n_seg][M][NC][r_max]
  int* lora_cnt;    // [n_seg][M], zero at launch
  float* kpart;     // [groups][S][kNT*MT*256 + MT*16]
  int* k_cnt;       // [groups], zero at launch
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
};

// Agent-scope (device-coherent) accesses for data that crosses workgroups.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All of this thread's stores have completed when this returns (then barrier, then signal).
__device__ __forceinline__ void wait_own_stores() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

__device__ __forceinline__ float sumsq8(u32x4 v) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return s;
}

// ---- LoRA workgroup: partial shrink of one routed row over one k chunk -------------------------
template <int MT, bool XPACKED>
__device__ __forceinline__ void lora_shrink_wg(const LevelParams& p, float* red /* 2048 floats of LDS */) {
  const int idx = blockIdx.x;
  const int kc = idx % p.NC;
  const int m = (idx / p.NC) % p.M;
  const int slot = idx / (p.NC * p.M);
  const int site = p.site[slot];
  const int req = p.row_to_req ? p.row_to_req[m] : m;
  int tenant = 0;
  const int r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, site, &tenant);
  if (r == 0) return;
  const bf16_t* A = (const bf16_t*)p.ad.A[tenant * MILORA_NUM_SITES + site];
  const int K = p.K;
  const int k_lo = kc * kShrinkChunk;
  const int k_hi = k_lo + kShrinkChunk < K ? k_lo + kShrinkChunk : K;
  float* out = p.tpart + (((size_t)slot * p.M + m) * p.NC + kc) * p.ad.r_max;
  const bf16_t* X = p.X;
  auto xval = [&](int k) -> float {
    return bf16_to_f32(XPACKED ? X[packed_act_offset(m, k, MT)] : X[(size_t)m * K + k]);
  };
  const int tid = threadIdx.x;
  if ((r & 7) == 0 && ((uintptr_t)A & 15) == 0) {
    const int lpr = r >> 3, rpp = kThreads / lpr;  // lanes per row of A, rows per pass
    const int cg = tid % lpr, kr = tid / lpr;
    float acc[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) acc[v] = 0.f;
    if (kr < rpp) {
      const u32x4* Ap = reinterpret_cast<const u32x4*>(A) + cg;
      int k = k_lo + kr;
      for (; k + 7 * rpp < k_hi; k += 8 * rpp) {
        u32x4 a[8];
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          a[u] = __builtin_nontemporal_load(Ap + (size_t)(k + u * rpp) * lpr);
          x[u] = xval(k + u * rpp);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
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
      st_agent(out + tid, s);
    }
  } else {
    int rpad = 1;
    while (rpad < r) rpad <<= 1;
    const int c = tid % rpad, kr = tid / rpad, rpp = kThreads / rpad;
    float acc = 0.f;
    if (c < r)
      for (int k = k_lo + kr; k < k_hi; k += rpp) acc += xval(k) * bf16_to_f32(A[(size_t)k * r + c]);
    red[tid] = acc;
    __syncthreads();
    if (kr == 0 && c < r) {
      float s = 0.f;
      for (int q = 0; q < rpp; ++q) s += red[q * rpad + c];
      st_agent(out + c, s);
    }
  }
  // publish: the partial of every thread, then the row's counter
  wait_own_stores();
  __syncthreads();
  if (tid == 0) {
    __hip_atomic_fetch_add(&p.lora_cnt[slot * p.M + m], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int MT, int D, bool XPACKED, bool NORM>
__global__ void __launch_bounds__(kThreads) decode_level_kernel(const LevelParams p) {
  constexpr int kRows = MT * 16;
  constexpr int kTile = kNT * MT * 256;            // floats of one workgroup's partial tile set
  constexpr int kRec = kTile + MT * 16;            // + the per-row sums of squares
  constexpr int kGroupRows = MT <= 4 ? 16 : 8;     // routed rows expanded per round
  __shared__ float red[kTile];
  __shared__ float t_s[kGroupRows * MILORA_MAX_RANK];
  __shared__ float dsum[kWaves * kGroupRows * 64];
  __shared__ float ssq_s[kWaves * MT * 16];
  __shared__ float inv_s[kRows];
  __shared__ int l_m[kMaxRows], l_r[kMaxRows], l_t[kMaxRows], l_a[kMaxRows];
  __shared__ int l_cnt, s_last;

  if ((int)blockIdx.x < p.n_lora_wg) {
    lora_shrink_wg<MT, XPACKED>(p, dsum);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, kept in a scalar register
  const int wg = blockIdx.x - p.n_lora_wg;
  const int grp = wg / p.S, ks = wg - grp * p.S;
  // segment and the group's tiles
  int si = 0, gl = grp;
  if (!p.pair) {
    while (si + 1 < p.n_seg && gl >= p.grp_end[si]) ++si;
    if (si > 0) gl -= p.grp_end[si - 1];
  }
  const int KT = p.K >> 5;
  const int tiles_seg = p.N[si] >> 4;
  const int t0 = p.pair ? gl * 2 : gl * kNT;                        // first tile of the group inside its site
  const int nvalid = p.pair ? (tiles_seg - t0 < 2 ? tiles_seg - t0 : 2) : (tiles_seg - t0 < kNT ? tiles_seg - t0 : kNT);
  const u32x4* wp[kNT];
#pragma unroll
  for (int a = 0; a < kNT; ++a) {
    // pair: streams 0,1 = gate tiles t0, t0+1; streams 2,3 = up tiles t0, t0+1.  A stream past the end
    // of the site re-reads the group's first tile (valid memory) and its result is dropped.
    const int sw = p.pair ? (a >> 1) : si;
    int tl = p.pair ? (a & 1) : a;
    if (tl >= nvalid) tl = 0;
    wp[a] = reinterpret_cast<const u32x4*>(p.W[sw]) + (size_t)(t0 + tl) * KT * 64 + lane;
  }
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

  f32x4 acc[kNT][MT];
  float ss[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    ss[mt] = 0.f;
#pragma unroll
    for (int a = 0; a < kNT; ++a) acc[a][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // this slice's k blocks [f_lo, f_hi); this wave takes f_lo + w, f_lo + w + 4, ...
  const int f_lo = (int)(((long)KT * ks) / p.S), f_hi = (int)(((long)KT * (ks + 1)) / p.S);
  const int nf = (f_hi - f_lo - w + kWaves - 1) / kWaves;
  u32x4 wb[D][kNT], xb[D][MT];
  auto issue = [&](int s, int i) {
    const size_t f = (size_t)f_lo + w + (size_t)i * kWaves;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xb[s][mt] = xp[mt][f * kXStride];
#pragma unroll
    for (int a = 0; a < kNT; ++a) wb[s][a] = __builtin_nontemporal_load(wp[a] + f * 64);
  };
  auto consume = [&](int s) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const bf16x8 xv = __builtin_bit_cast(bf16x8, xb[s][mt]);
#pragma unroll
      for (int a = 0; a < kNT; ++a)
        acc[a][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wb[s][a]), xv, acc[a][mt], 0, 0, 0);
      if (NORM) ss[mt] += sumsq8(xb[s][mt]);
    }
  };
  if (nf >= 2 * D) {
    // Register ring of D blocks per stream.  The fill and the steady loop issue unconditionally and in
    // program order, so the number of loads in flight is the same on every path into a consume and the
    // wait before it covers the oldest block only.
#pragma unroll
    for (int s = 0; s < D; ++s) {
      issue(s, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    int i0 = 0;
    for (; i0 + 2 * D <= nf; i0 += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        consume(s);
        issue(s, i0 + D + s);
        __builtin_amdgcn_sched_barrier(0);
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
    for (int i = 0; i < nf; ++i) {  // short slices: no ring
      issue(0, i);
      consume(0);
    }
  }

  // ---- the four waves' partial tiles summed in wave order through LDS ---------------------------
  auto red_idx = [&](int a, int mt, int i, int ln) { return ((a * MT + mt) * 4 + i) * 64 + ln; };
#pragma unroll
  for (int ww = 0; ww < kWaves; ++ww) {
    if (w == ww) {
#pragma unroll
      for (int a = 0; a < kNT; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (ww == 0) red[red_idx(a, mt, i, lane)] = acc[a][mt][i];
            else red[red_idx(a, mt, i, lane)] += acc[a][mt][i];
          }
    }
    __syncthreads();
  }
  if (NORM) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float v = ss[mt];
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      if (lane < 16) ssq_s[(w * MT + mt) * 16 + lane] = v;
    }
    __syncthreads();
    if (tid < kRows) {
      float s = 0.f;
      for (int ww = 0; ww < kWaves; ++ww) s += ssq_s[(ww * MT + (tid >> 4)) * 16 + (tid & 15)];
      inv_s[tid] = s;  // sum of squares of this slice; turned into the scale below
    }
    __syncthreads();
  }

  // ---- slices of one group: the last workgroup to arrive sums them in slice order -------------------
  if (p.S > 1) {
    float* mine = p.kpart + ((size_t)grp * p.S + ks) * kRec;
    for (int e = tid; e < kTile; e += kThreads) st_agent(mine + e, red[e]);
    if (NORM && tid < kRows) st_agent(mine + kTile + tid, inv_s[tid]);
    wait_own_stores();
    __syncthreads();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(&p.k_cnt[grp], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == p.S - 1);
    }
    __syncthreads();
    if (!s_last) return;
    const float* base = p.kpart + (size_t)grp * p.S * kRec;
    for (int e = tid; e < kTile; e += kThreads) {
      float s = ld_agent(base + e);
      for (int q = 1; q < p.S; ++q) s += ld_agent(base + (size_t)q * kRec + e);
      red[e] = s;
    }
    if (NORM && tid < kRows) {
      float s = 0.f;
      for (int q = 0; q < p.S; ++q) s += ld_agent(base + (size_t)q * kRec + kTile + tid);
      inv_s[tid] = s;
    }
    __syncthreads();
  }
  if (NORM) {
    if (tid < kRows) inv_s[tid] = rsqrtf(inv_s[tid] / (float)p.K + 1e-5f);
  }
  if (tid == 0) l_cnt = 0;
  __syncthreads();

  // ---- LoRA expand of the rows routed to this group's site(s), added to the fp32 sums ----------
  // column space of `red`: stream a, column nl  <->  red[a][mt][nl & 3][(m & 15) + 16 * (nl >> 2)]
  const int n0 = t0 * 16;  // first column of the group inside its site
  if (p.tpart) {
    for (int m = tid; m < p.M; m += kThreads) {
      const int req = p.row_to_req ? p.row_to_req[m] : m;
      const int nslot = p.pair ? 2 : 1;
      for (int a = 0; a < nslot; ++a) {
        int tenant = 0;
        const int slot = p.pair ? a : si;
        const int r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, p.site[slot], &tenant);
        if (r) {
          // wait for the row's shrink partials (published by workgroups that were dispatched before this one)
          const int* cnt = &p.lora_cnt[slot * p.M + m];
          int spins = 0;
          while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < p.NC && ++spins < kSpinLimit)
            __builtin_amdgcn_s_sleep(2);
          if (spins < kSpinLimit) {
            const int idx = atomicAdd(&l_cnt, 1);
            l_m[idx] = m; l_r[idx] = r; l_t[idx] = tenant; l_a[idx] = slot;
          }
        }
      }
    }
    __syncthreads();
    const int cnt = l_cnt, rmax = p.ad.r_max;
    const int ncol = p.pair ? 32 : 64;  // columns a routed row touches in this group
    for (int g0 = 0; g0 < cnt; g0 += kGroupRows) {
      const int ng = cnt - g0 < kGroupRows ? cnt - g0 : kGroupRows;
      for (int e = tid; e < ng * rmax; e += kThreads) {
        const int gi = e / rmax, c = e - gi * rmax, idx = g0 + gi;
        if (c < l_r[idx]) {
          const float* tp = p.tpart + (((size_t)l_a[idx] * p.M + l_m[idx]) * p.NC) * rmax + c;
          float s = 0.f;
          for (int kc = 0; kc < p.NC; ++kc) s += ld_agent(tp + (size_t)kc * rmax);
          t_s[gi * rmax + c] = s;
        }
      }
      __syncthreads();
      // wave w takes ranks c = w, w+4, ...; lane = (row of a block of four, column quad)
      const int quad = lane & 15, rsub = lane >> 4;
      for (int gb = 0; gb < ng; gb += 4) {
        const int gi = gb + rsub;
        float d[4] = {0.f, 0.f, 0.f, 0.f};
        if (gi < ng && quad * 4 < ncol) {
          const int idx = g0 + gi, r = l_r[idx], slot = l_a[idx];
          const size_t ldb = (size_t)p.N[slot];
          const int n = n0 + quad * 4;
          if (n < (int)ldb) {
            const bf16_t* Bm = (const bf16_t*)p.ad.B[l_t[idx] * MILORA_NUM_SITES + p.site[slot]] + n;
            const float* tv = t_s + gi * rmax;
            if (((uintptr_t)Bm & 7) == 0) {
              int c = w;
              for (; c + 7 * kWaves < r; c += 8 * kWaves) {
                u32x2 bb[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) bb[u] = *reinterpret_cast<const u32x2*>(Bm + (size_t)(c + u * kWaves) * ldb);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                  const float t = tv[c + u * kWaves];
                  d[0] += t * __uint_as_float(bb[u][0] << 16);
                  d[1] += t * __uint_as_float(bb[u][0] & 0xffff0000u);
                  d[2] += t * __uint_as_float(bb[u][1] << 16);
                  d[3] += t * __uint_as_float(bb[u][1] & 0xffff0000u);
                }
              }
              for (; c < r; c += kWaves) {
                const u32x2 bb = *reinterpret_cast<const u32x2*>(Bm + (size_t)c * ldb);
                const float t = tv[c];
                d[0] += t * __uint_as_float(bb[0] << 16);
                d[1] += t * __uint_as_float(bb[0] & 0xffff0000u);
                d[2] += t * __uint_as_float(bb[1] << 16);
                d[3] += t * __uint_as_float(bb[1] & 0xffff0000u);
              }
            } else {
              for (int c = w; c < r; c += kWaves) {
                const float t = tv[c];
#pragma unroll
                for (int q = 0; q < 4; ++q) d[q] += t * bf16_to_f32(Bm[(size_t)c * ldb + q]);
              }
            }
          }
        }
        if (gi < ng) {
#pragma unroll
          for (int q = 0; q < 4; ++q) dsum[(w * kGroupRows + gi) * 64 + quad * 4 + q] = d[q];
        }
      }
      __syncthreads();
      // the four rank classes summed in wave order and added to the base result
      for (int e = tid; e < ng * ncol; e += kThreads) {
        const int gi = e / ncol, col = e - gi * ncol, idx = g0 + gi;
        float s = 0.f;
        for (int ww = 0; ww < kWaves; ++ww) s += dsum[(ww * kGroupRows + gi) * 64 + col];
        const int m = l_m[idx];
        const int a = (p.pair ? 2 * l_a[idx] : 0) + (col >> 4), nl = col & 15;
        red[red_idx(a, m >> 4, nl & 3, (m & 15) + 16 * (nl >> 2))] += s;
      }
      __syncthreads();
    }
  }

  // ---- glue and stores: thread (row m, column pair) -------------------------------------------------
  const int nout = p.pair ? 32 : 64;  // output columns of the group
  const int ppr = nout >> 1;          // column pairs per row
  const int n_lim = p.N[si];
  for (int e = tid; e < p.M * ppr; e += kThreads) {
    const int m = e / ppr, pp = e - m * ppr;
    const int col = 2 * pp;
    const int n = n0 + col;
    if (n >= n_lim) continue;
    const int mt = m >> 4;
    const float inv = NORM ? inv_s[m] : 1.f;
    float val[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int a = (col + q) >> 4, nl = (col + q) & 15;
      const int ln = (m & 15) + 16 * (nl >> 2);
      const float v0 = red[red_idx(a, mt, nl & 3, ln)] * inv;
      if (p.pair) val[q] = silu(v0) * (red[red_idx(a + 2, mt, nl & 3, ln)] * inv);
      else val[q] = v0;
    }
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

__global__ void __launch_bounds__(kThreads) clear_ints_kernel(int* p, int n) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Row-major [d2][d1] -> packed blocks (see milora_wlayout): one thread per 16-byte group of 8 inputs.
__global__ void __launch_bounds__(kThreads) pack_weight_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                               int d1, int d2) {
  const size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;  // index of the 8-element group in dst
  const size_t total = (size_t)d1 * d2 / 8;
  if (g >= total) return;
  const int KT = d1 >> 5;
  const size_t blk = g >> 6;
  const int ln = (int)(g & 63);
  const int nt = (int)(blk / KT), kt = (int)(blk % KT);
  const int jrow = nt * 16 + (ln & 15), i0 = kt * 32 + (ln >> 4) * 8;
  dst[g] = src[((size_t)jrow * d1 + i0) / 8];
}

// Row-major bf16 activations [M][K] -> block-packed buffer.
template <int MT>
__global__ void __launch_bounds__(kThreads) pack_act_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                            int M, int K) {
  const size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t total = (size_t)(K >> 5) * MT * 64;
  if (g >= total) return;
  const int ln = (int)(g & 63);
  const size_t blk = g >> 6;
  const int mt = (int)(blk % MT), kt = (int)(blk / MT);
  int row = mt * 16 + (ln & 15);
  if (row > M - 1) row = M - 1;
  dst[g] = src[((size_t)row * K + kt * 32 + (ln >> 4) * 8) / 8];
}

int mt_for(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : (M <= 64 ? 4 : 8)); }
int shrink_chunks(int K) { return (K + kShrinkChunk - 1) / kShrinkChunk; }
size_t rec_floats(int MT) { return (size_t)kNT * MT * 256 + MT * 16; }

int level_groups(const LevelParams& p) {
  if (p.pair) return ((p.N[0] >> 4) + 1) / 2;
  return p.grp_end[p.n_seg - 1];
}

// Reduction slices per column group: enough workgroups to keep every CU streaming, slices long enough
// for the register ring.
int pick_slices(int groups, int K) {
  const int KT = K >> 5;
  int S = (320 + groups - 1) / groups;
  const int cap = KT / 32 > 1 ? KT / 32 : 1;
  if (S > cap) S = cap;
  if (S > 16) S = 16;
  return S < 1 ? 1 : S;
}

template <int MT, bool XPACKED>
void launch_level_t(const LevelParams& p, int grid, bool norm, hipStream_t st) {
  constexpr int D = MT <= 2 ? 4 : (MT == 4 ? 3 : 2);
  if (norm) hipLaunchKernelGGL((decode_level_kernel<MT, D, XPACKED, true>), dim3(grid), dim3(kThreads), 0, st, p);
  else hipLaunchKernelGGL((decode_level_kernel<MT, D, XPACKED, false>), dim3(grid), dim3(kThreads), 0, st, p);
}

int launch_level(LevelParams& p, int MT, bool xpacked, bool norm, hipStream_t st) {
  const int groups = level_groups(p);
  if (groups > kMaxGroups) return MILORA_ERANGE;
  p.NC = shrink_chunks(p.K);
  p.n_lora_wg = p.tpart ? p.n_seg * p.M * p.NC : 0;
  const int grid = p.n_lora_wg + groups * p.S;
#define MILORA_LEVEL(MTV)                                                   \
  if (xpacked) launch_level_t<MTV, true>(p, grid, norm, st);                \
  else launch_level_t<MTV, false>(p, grid, norm, st)
  switch (MT) {
    case 1: MILORA_LEVEL(1); break;
    case 2: MILORA_LEVEL(2); break;
    case 4: MILORA_LEVEL(4); break;
    default: MILORA_LEVEL(8); break;
  }
#undef MILORA_LEVEL
  return check_launch();
}

void reset_params(LevelParams& p) {
  for (int s = 0; s < 3; ++s) {
    p.W[s] = nullptr; p.N[s] = 0; p.site[s] = 0; p.grp_end[s] = 0;
    p.bias[s] = nullptr; p.out_rm[s] = nullptr; p.out_pk[s] = nullptr; p.col_off[s] = 0;
  }
  p.resid_bf16 = nullptr; p.resid_f32 = nullptr; p.ld_resid = 0;
  p.out_f32 = nullptr; p.ld_f32 = 0; p.ld_rm = 0; p.pair = 0; p.n_seg = 0; p.S = 1;
  p.tpart = nullptr; p.NC = 0; p.n_lora_wg = 0; p.row_to_req = nullptr;
  p.lora_cnt = nullptr; p.k_cnt = nullptr; p.kpart = nullptr;
}

int groups_of(int N) { return ((N >> 4) + kNT - 1) / kNT; }

// ---- workspace layout of the packed-weight decode paths -------------------------------------------
constexpr int kLevels = 4;
constexpr int kCntPerLevel = 3 * kMaxRows + kMaxGroups;

struct DecodeWs {
  int* counters;   // [kLevels][3*128 LoRA row counters | kMaxGroups group counters]
  float* tpart;    // [3][M][NCmax][r_max]
  float* kpart;    // slice partials of one level
  float* h_f32;    // [M][d]
  bf16_t* pk_a;    // packed, K = max(d, F): a = v (or attn_out), later m = silu(g) * u
  bf16_t* pk_b;    // packed, K = d       : h
  size_t bytes;
};

size_t kpart_floats(int MT, int groups, int K) { return (size_t)groups * pick_slices(groups, K) * rec_floats(MT); }

DecodeWs carve_decode_ws(void* base, int M, int d, int F, int r_max) {
  const int MT = mt_for(M);
  const int big = F > d ? F : d;
  const int ncmax = shrink_chunks(big);
  size_t kp = kpart_floats(MT, 3 * groups_of(d), d);
  size_t v = kpart_floats(MT, groups_of(d), d); if (v > kp) kp = v;
  v = kpart_floats(MT, ((F >> 4) + 1) / 2, d); if (v > kp) kp = v;
  v = kpart_floats(MT, groups_of(d), F); if (v > kp) kp = v;
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_c = take((size_t)kLevels * kCntPerLevel * sizeof(int));
  const size_t o_t = take((size_t)3 * M * ncmax * r_max * sizeof(float));
  const size_t o_k = take(kp * sizeof(float));
  const size_t o_h = take((size_t)M * d * sizeof(float));
  const size_t o_a = take((size_t)MT * 16 * big * sizeof(bf16_t));
  const size_t o_b = take((size_t)MT * 16 * d * sizeof(bf16_t));
  char* b = (char*)base;
  return DecodeWs{(int*)(b + o_c), (float*)(b + o_t), (float*)(b + o_k), (float*)(b + o_h), (bf16_t*)(b + o_a),
                  (bf16_t*)(b + o_b), off};
}

int clear_counters(int* p, int n, hipStream_t st) {
  hipLaunchKernelGGL(clear_ints_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0, st, p, n);
  return check_launch();
}

}  // namespace

size_t decode_packed_workspace_bytes(int M, int d, int F, int r_max) { return carve_decode_ws(nullptr, M, d, F, r_max).bytes; }

// One decode step of a layer on packed weights: a counter-clearing launch, then one launch per
// dependency level.  With `marks`, an event is recorded after every launch (slot 0: clear, 1..4: levels).
int layer_decode_packed(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                        const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                        bf16_t* y, bf16_t* qkv_out, void* workspace, hipStream_t st, LaunchMarks* marks) {
  const int MT = mt_for(B);
  auto mark = [&](int slot) {
    if (marks && slot < marks->n) (void)hipEventRecord(marks->ev[slot], st);
  };
  DecodeWs ws = carve_decode_ws(workspace, B, d, F, ad.r_max);
  const bool norm = (flags & MILORA_LAYER_RMSNORM) != 0;
  int rc = clear_counters(ws.counters, kLevels * kCntPerLevel, st);
  if (rc) return rc;
  mark(0);
  LevelParams p;
  auto common = [&](int level, const bf16_t* X, int K) {
    reset_params(p);
    p.X = X; p.K = K; p.M = B; p.Breq = B;
    p.ad = ad; p.tenant_id = tenant_id; p.route = route;
    p.tpart = ws.tpart; p.kpart = ws.kpart;
    p.lora_cnt = ws.counters + level * kCntPerLevel;
    p.k_cnt = p.lora_cnt + 3 * kMaxRows;
  };
  // level 0: q, k, v from x
  {
    common(0, x, d);
    p.n_seg = 3;
    for (int s = 0; s < 3; ++s) {
      p.W[s] = (const bf16_t*)wts->W[s]; p.N[s] = d; p.site[s] = s; p.grp_end[s] = (s + 1) * groups_of(d);
      p.out_rm[s] = qkv_out; p.col_off[s] = s * d;
    }
    p.ld_rm = 3 * d;
    if (!attn_out) p.out_pk[2] = ws.pk_a;
    p.S = pick_slices(level_groups(p), d);
    if ((rc = launch_level(p, MT, false, norm, st))) return rc;
    mark(1);
  }
  // level 1: h = x + L_o(a)
  {
    if (attn_out) {
      const size_t groups = (size_t)(d >> 5) * MT * 64;
      const unsigned blocks = (unsigned)((groups + kThreads - 1) / kThreads);
      switch (MT) {
        case 1: hipLaunchKernelGGL(pack_act_kernel<1>, dim3(blocks), dim3(kThreads), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        case 2: hipLaunchKernelGGL(pack_act_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        case 4: hipLaunchKernelGGL(pack_act_kernel<4>, dim3(blocks), dim3(kThreads), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
        default: hipLaunchKernelGGL(pack_act_kernel<8>, dim3(blocks), dim3(kThreads), 0, st, (const u32x4*)attn_out, (u32x4*)ws.pk_a, B, d); break;
      }
      if ((rc = check_launch())) return rc;
    }
    common(1, ws.pk_a, d);
    p.n_seg = 1;
    p.W[0] = (const bf16_t*)wts->W[3]; p.N[0] = d; p.site[0] = 3; p.grp_end[0] = groups_of(d);
    p.resid_bf16 = x; p.ld_resid = d;
    p.out_f32 = ws.h_f32; p.ld_f32 = d;
    p.out_pk[0] = ws.pk_b;  // other workgroups may still be reading a, so h goes to the second buffer
    p.S = pick_slices(level_groups(p), d);
    if ((rc = launch_level(p, MT, true, false, st))) return rc;
    mark(2);
  }
  // level 2: m = silu(L_gate(n(h))) * L_up(n(h))
  {
    common(2, ws.pk_b, d);
    p.n_seg = 2; p.pair = 1;
    for (int s = 0; s < 2; ++s) { p.W[s] = (const bf16_t*)wts->W[4 + s]; p.N[s] = F; p.site[s] = 4 + s; }
    p.out_pk[0] = ws.pk_a;
    p.S = pick_slices(level_groups(p), d);
    if ((rc = launch_level(p, MT, true, norm, st))) return rc;
    mark(3);
  }
  // level 3: y = h + L_down(m)
  {
    common(3, ws.pk_a, F);
    p.n_seg = 1;
    p.W[0] = (const bf16_t*)wts->W[6]; p.N[0] = d; p.site[0] = 6; p.grp_end[0] = groups_of(d);
    p.resid_f32 = ws.h_f32; p.ld_resid = d;
    p.out_rm[0] = y; p.ld_rm = d; p.col_off[0] = 0;
    p.S = pick_slices(level_groups(p), F);
    if ((rc = launch_level(p, MT, true, false, st))) return rc;
    mark(4);
  }
  return MILORA_OK;
}

// ---- one routed linear of M <= 128 rows on a packed weight ------------------------------------------
struct LinearWs {
  int* counters;
  float* tpart;
  float* kpart;
  size_t bytes;
};

static LinearWs carve_linear_ws(void* base, int M, int d1, int d2, int r_max) {
  const int MT = mt_for(M);
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_c = take((size_t)kCntPerLevel * sizeof(int));
  const size_t o_t = take((size_t)M * shrink_chunks(d1) * r_max * sizeof(float));
  const size_t o_k = take(kpart_floats(MT, groups_of(d2), d1) * sizeof(float));
  char* b = (char*)base;
  return LinearWs{(int*)(b + o_c), (float*)(b + o_t), (float*)(b + o_k), off};
}

size_t routed_linear_packed_workspace_bytes(int M, int d1, int d2, int r_max) {
  return carve_linear_ws(nullptr, M, d1, d2, r_max).bytes;
}

int routed_linear_packed(const bf16_t* X, int M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                         const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                         const uint8_t* route, int B, bf16_t* Y, void* workspace, hipStream_t st) {
  const int MT = mt_for(M);
  if (groups_of(d2) > kMaxGroups) return MILORA_ERANGE;
  LinearWs ws = carve_linear_ws(workspace, M, d1, d2, ad.r_max);
  int rc = clear_counters(ws.counters, kCntPerLevel, st);
  if (rc) return rc;
  LevelParams p;
  reset_params(p);
  p.X = X; p.K = d1; p.M = M; p.Breq = B;
  p.ad = ad; p.tenant_id = tenant_id; p.route = route; p.row_to_req = row_to_req;
  p.tpart = ws.tpart; p.kpart = ws.kpart;
  p.lora_cnt = ws.counters; p.k_cnt = ws.counters + 3 * kMaxRows;
  p.n_seg = 1;
  p.W[0] = W; p.N[0] = d2; p.site[0] = site; p.grp_end[0] = groups_of(d2);
  p.bias[0] = bias;
  p.out_rm[0] = Y; p.ld_rm = d2;
  p.S = pick_slices(level_groups(p), d1);
  return launch_level(p, MT, false, false, st);
}

int pack_weight(const void* src, void* dst, int d1, int d2, hipStream_t st) {
  const size_t groups = (size_t)d1 * d2 / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     (const u32x4*)src, (u32x4*)dst, d1, d2);
  return check_launch();
}

}  // namespace milora
