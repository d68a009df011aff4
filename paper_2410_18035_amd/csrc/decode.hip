// Decode-time routed LoRA linears on packed bf16 weights (paper Eq. 1; Sec. 3.3 route reuse).
//
// At decode the batch is skinny (B <= 128 rows) and every base weight is read exactly once per
// step, so everything is built around keeping the HBM stream of W running on all 256 CUs.  Weights
// are pre-packed in 1 KiB blocks that already are 16x16x32 matrix-core operands (one wave load =
// one contiguous block).  A whole decode step of a layer is one persistent launch of G = 256 k
// workgroups that walks the four dependency levels (q,k,v | o | gate,up | down) with a grid barrier
// between levels.  Inside a level every workgroup
//   1. takes its share of the LoRA shrink items (routed row x 512-row chunk of A): partial
//      t = x[chunk] . A[chunk]; the workgroup that delivers a row's last partial sums them in
//      chunk order and publishes the row's t;
//   2. takes an equal share of the level's weight blocks: the level is the list of (column group of
//      four 16-column tiles, k block) units and workgroup i owns units [iU/G, (i+1)U/G), so a share
//      is one or two runs inside a column group ("segments").  The four waves interleave along k;
//      the batch rows ride in the other MFMA operand and are loaded once per k block for all four
//      tiles; a register ring keeps D blocks per stream in flight;
//   3. for each segment reduces the waves' partial tiles through LDS; a group whose k range is
//      split over several workgroups is summed, in workgroup order, by whichever of them finishes
//      last; that workgroup adds the LoRA expand t W^B of the routed rows in fp32, applies the layer
//      glue (normalisation scale, residual, silu*up) and rounds once to bf16.
// Data handed from one workgroup to another (partials, t, the activations of the next level) is
// written with agent-scope stores, which go through to memory that all XCDs share instead of
// staying in one XCD's L2; partials and t are also read with agent-scope loads.  A producer waits
// for its own stores, passes a workgroup barrier and bumps an agent-scope counter; a consumer reads
// the counter before the data.  Activation buffers are distinct per level, so no XCD can hold a
// stale line of them.  Every wait is bounded, and all sums run in a fixed order: results do not
// depend on timing.
#include "common.h"

namespace milora {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kNT = 4;              // 16-column tiles (weight streams) per column group
constexpr int kShrinkChunk = 512;   // reduction rows per LoRA shrink item
constexpr int kMaxRows = MILORA_MAX_DECODE_BATCH;
constexpr int kMaxGroups = 2048;    // column groups per level the counters are sized for
constexpr int kMaxLevels = 4;
constexpr int kSpinLimit = 1 << 20; // polls of a counter before a workgroup stops waiting
constexpr int kCntPerLevel = 3 * kMaxRows + kMaxGroups;
constexpr int kSync = kMaxLevels * kCntPerLevel + 64;  // ints of the synchronisation block (+ barrier word, status)

// Offset (in bf16 elements) of activation element (row m, feature k) in a block-packed buffer of MT row tiles.
__device__ __host__ __forceinline__ size_t packed_act_offset(int m, int k, int MT) {
  return ((((size_t)(k >> 5) * MT + (m >> 4)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

struct LevelDesc {
  const bf16_t* X;  // block-packed input of the level
  int K;
  // weight segments: up to three sites share X.  Column groups never straddle segments.
  // pair = 1 (gate, up): group g holds tiles 2g, 2g+1 of W[0] and of W[1] and emits silu(gate)*up.
  int n_seg, pair, norm, groups;
  const bf16_t* W[3];
  int N[3], site[3], grp_end[3];
  int* lora_cnt;  // [n_seg][M], zero at launch
  int* k_cnt;     // [groups], zero at launch
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

struct DecodeParams {
  int n_levels, M, Breq;
  AdapterView ad;
  const int32_t* tenant_id;
  const uint8_t* route;
  const int32_t* row_to_req;
  int lora;        // 0: no LoRA term at all
  float* tpart;    // [3][M][NCmax][r_max] shrink partials
  float* tfin;     // [3][M][r_max] summed t
  float* kpart;    // [G][2][record] segment partials
  int* bar;        // grid barrier word, zero at launch
  int* status;     // set to 1 when a bounded wait ran out
  LevelDesc lv[kMaxLevels];
};

// Agent-scope (device-coherent) accesses for data that crosses workgroups.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All of this thread's stores have completed when this returns (then barrier, then signal).
__device__ __forceinline__ void wait_own_stores() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): every store of this wave has been acknowledged
}

// Poll an agent-scope counter until it reaches `target`; false when the bound ran out.
__device__ __forceinline__ bool wait_counter(const int* cnt, int target) {
  int spins = 0;
  while (ld_agent(cnt) < target) {
    if (++spins >= kSpinLimit) return false;
    __builtin_amdgcn_s_sleep(1);
  }
  return true;
}

__device__ __forceinline__ float sumsq8(u32x4 v) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return s;
}

__host__ __device__ __forceinline__ int shrink_chunks(int K) { return (K + kShrinkChunk - 1) / kShrinkChunk; }

// ---- one LoRA shrink item: partial t of one routed row over one k chunk --------------------------
// scratch: 4096 floats of LDS.  Uniform over the workgroup.
template <int MT>
__device__ __forceinline__ void lora_shrink_item(const DecodeParams& p, const LevelDesc& lv, int item, int NC,
                                                 float* scratch, int* s_flag) {
  const int kc = item % NC;
  const int m = (item / NC) % p.M;
  const int slot = item / (NC * p.M);
  const int site = lv.site[slot];
  const int req = p.row_to_req ? p.row_to_req[m] : m;
  int tenant = 0;
  const int r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, site, &tenant);
  if (r == 0) return;
  const bf16_t* A = (const bf16_t*)p.ad.A[tenant * MILORA_NUM_SITES + site];
  const int K = lv.K, rmax = p.ad.r_max;
  const int k_lo = kc * kShrinkChunk;
  const int k_hi = k_lo + kShrinkChunk < K ? k_lo + kShrinkChunk : K;
  float* row_part = p.tpart + (((size_t)slot * p.M + m) * NC) * rmax;
  float* out = row_part + (size_t)kc * rmax;
  const bf16_t* X = lv.X;
  auto xval = [&](int k) -> float { return bf16_to_f32(X[packed_act_offset(m, k, MT)]); };
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
    for (int v = 0; v < 8; ++v) scratch[tid * 8 + v] = acc[v];
    __syncthreads();
    if (tid < r) {
      const int g = tid >> 3, v = tid & 7;
      float s = 0.f;
      for (int q = 0; q < rpp; ++q) s += scratch[(q * lpr + g) * 8 + v];
      st_agent(out + tid, s);
    }
  } else {
    int rpad = 1;
    while (rpad < r) rpad <<= 1;
    const int c = tid % rpad, kr = tid / rpad, rpp = kThreads / rpad;
    float acc = 0.f;
    if (c < r)
      for (int k = k_lo + kr; k < k_hi; k += rpp) acc += xval(k) * bf16_to_f32(A[(size_t)k * r + c]);
    scratch[tid] = acc;
    __syncthreads();
    if (kr == 0 && c < r) {
      float s = 0.f;
      for (int q = 0; q < rpp; ++q) s += scratch[q * rpad + c];
      st_agent(out + c, s);
    }
  }
  // publish the partial; whoever delivers the row's last partial sums them in chunk order
  wait_own_stores();
  __syncthreads();
  int* cnt = &lv.lora_cnt[slot * p.M + m];
  if (tid == 0) *s_flag = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (*s_flag != NC - 1) return;
  float* fin = p.tfin + ((size_t)slot * p.M + m) * rmax;
  const int blk = 4096 / r;  // chunks per round that fit the scratch
  float tot = 0.f;
  for (int k0 = 0; k0 < NC; k0 += blk) {
    const int nk = NC - k0 < blk ? NC - k0 : blk;
    __syncthreads();
    for (int e = tid; e < nk * r; e += kThreads) {
      const int q = e / r, c = e - q * r;
      scratch[e] = ld_agent(row_part + (size_t)(k0 + q) * rmax + c);
    }
    __syncthreads();
    if (tid < r)
      for (int q = 0; q < nk; ++q) tot += scratch[q * r + tid];
  }
  if (tid < r) st_agent(fin + tid, tot);
  wait_own_stores();
  __syncthreads();
  if (tid == 0) __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // NC + 1: t is ready
}

// Workgroup that owns unit u when G workgroups split U units as [iU/G, (i+1)U/G).
__device__ __forceinline__ int wg_of_unit(long u, long U, int G) { return (int)(((u + 1) * G + U - 1) / U) - 1; }

template <int MT, int D>
__global__ void __launch_bounds__(kThreads) decode_persist_kernel(const DecodeParams p) {
  constexpr int kRows = MT * 16;
  constexpr int kTile = kNT * MT * 256;            // floats of one segment's partial tile set
  constexpr int kRec = kTile + MT * 16;            // + the per-row sums of squares
  constexpr int kEPT = kTile / kThreads;           // floats per thread of a partial record
  constexpr int kGroupRows = MT <= 4 ? 16 : 8;     // routed rows expanded per round
  __shared__ float red[kTile];
  __shared__ float t_s[kGroupRows * MILORA_MAX_RANK];
  __shared__ float dsum[4096];
  __shared__ float ssq_s[kWaves * MT * 16];
  __shared__ float inv_s[kRows];
  __shared__ int l_m[kMaxRows], l_r[kMaxRows], l_t[kMaxRows], l_a[kMaxRows];
  __shared__ int l_cnt, s_flag;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, kept in a scalar register
  const int wg = blockIdx.x, G = gridDim.x;
  auto red_idx = [&](int a, int mt, int i, int ln) { return ((a * MT + mt) * 4 + i) * 64 + ln; };

  for (int L = 0; L < p.n_levels; ++L) {
    const LevelDesc& lv = p.lv[L];
    const int KT = lv.K >> 5;
    const int NC = shrink_chunks(lv.K);

    // ---- 1. this workgroup's LoRA shrink items -----------------------------------------------------
    if (p.lora) {
      const int items = lv.n_seg * p.M * NC;
      for (int item = wg; item < items; item += G) {
        lora_shrink_item<MT>(p, lv, item, NC, dsum, &s_flag);
        __syncthreads();
      }
    }

    // ---- 2. this workgroup's share of the weight blocks, one segment at a time ---------------------
    const long U = (long)lv.groups * KT;
    const int Gl = U < (long)G ? (int)U : G;  // workgroups that stream in this level: none of them empty-handed
    long u0 = wg < Gl ? (U * wg) / Gl : 0;
    const long u1 = wg < Gl ? (U * (wg + 1)) / Gl : 0;
    while (u0 < u1) {
      const int grp = (int)(u0 / KT);
      const int f_lo = (int)(u0 - (long)grp * KT);
      const int f_hi = (u1 - u0) < (long)(KT - f_lo) ? f_lo + (int)(u1 - u0) : KT;
      u0 += f_hi - f_lo;
      // site and tiles of the group
      int si = 0, gl = grp;
      if (!lv.pair) {
        while (si + 1 < lv.n_seg && gl >= lv.grp_end[si]) ++si;
        if (si > 0) gl -= lv.grp_end[si - 1];
      }
      const int tiles_seg = lv.N[si] >> 4;
      const int t0 = lv.pair ? gl * 2 : gl * kNT;  // first tile of the group inside its site
      const int tper = lv.pair ? 2 : kNT;
      const int nvalid = tiles_seg - t0 < tper ? tiles_seg - t0 : tper;
      const u32x4* wp[kNT];
#pragma unroll
      for (int a = 0; a < kNT; ++a) {
        // pair: streams 0,1 = gate tiles t0, t0+1; streams 2,3 = up tiles t0, t0+1.  A stream past the end
        // of the site re-reads the group's first tile (valid memory) and its result is dropped.
        const int sw = lv.pair ? (a >> 1) : si;
        int tl = lv.pair ? (a & 1) : a;
        if (tl >= nvalid) tl = 0;
        wp[a] = reinterpret_cast<const u32x4*>(lv.W[sw]) + (size_t)(t0 + tl) * KT * 64 + lane;
      }
      const u32x4* xp = reinterpret_cast<const u32x4*>(lv.X) + lane;

      f32x4 acc[kNT][MT];
      float ss[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        ss[mt] = 0.f;
#pragma unroll
        for (int a = 0; a < kNT; ++a) acc[a][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      // k blocks [f_lo, f_hi) of the group; this wave takes f_lo + w, f_lo + w + 4, ...
      const int nf = (f_hi - f_lo - w + kWaves - 1) / kWaves;
      u32x4 wb[D][kNT], xb[D][MT];
      auto issue = [&](int s, int i) {
        const size_t f = (size_t)f_lo + w + (size_t)i * kWaves;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xb[s][mt] = xp[(f * MT + mt) * 64];
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
          ss[mt] += sumsq8(xb[s][mt]);
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
        for (int i0 = 0; i0 < nf; i0 += D) {  // short runs: everything of a round in flight at once
#pragma unroll
          for (int s = 0; s < D; ++s)
            if (i0 + s < nf) issue(s, i0 + s);
#pragma unroll
          for (int s = 0; s < D; ++s)
            if (i0 + s < nf) consume(s);
        }
      }

      // ---- the four waves' partial tiles summed in wave order through LDS -------------------------
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
        inv_s[tid] = s;  // sum of squares over this segment; turned into the scale below
      }
      __syncthreads();

      // ---- a group split over several workgroups: the last one to arrive sums in workgroup order ----
      const long g_first_u = (long)grp * KT;
      const int wg_first = wg_of_unit(g_first_u, U, Gl), wg_last = wg_of_unit(g_first_u + KT - 1, U, Gl);
      const int nparts = wg_last - wg_first + 1;
      bool finisher = true;
      if (nparts > 1) {
        float* mine = p.kpart + ((size_t)wg * 2 + (f_lo > 0 ? 0 : 1)) * kRec;
#pragma unroll
        for (int e = 0; e < kEPT; ++e) st_agent(mine + tid + e * kThreads, red[tid + e * kThreads]);
        if (tid < kRows) st_agent(mine + kTile + tid, inv_s[tid]);
        wait_own_stores();
        __syncthreads();
        if (tid == 0) s_flag = __hip_atomic_fetch_add(&lv.k_cnt[grp], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        finisher = (s_flag == nparts - 1);
        if (finisher) {
          float s[kEPT];
#pragma unroll
          for (int e = 0; e < kEPT; ++e) s[e] = 0.f;
          float sq = 0.f;
          for (int i = wg_first; i <= wg_last; ++i) {
            const long st_i = (U * i) / Gl;
            const float* rec = p.kpart + ((size_t)i * 2 + (st_i > g_first_u ? 0 : 1)) * kRec;
            float v[kEPT];
#pragma unroll
            for (int e = 0; e < kEPT; ++e) v[e] = ld_agent(rec + tid + e * kThreads);
            const float q = tid < kRows ? ld_agent(rec + kTile + tid) : 0.f;
#pragma unroll
            for (int e = 0; e < kEPT; ++e) s[e] += v[e];
            sq += q;
          }
#pragma unroll
          for (int e = 0; e < kEPT; ++e) red[tid + e * kThreads] = s[e];
          if (tid < kRows) inv_s[tid] = sq;
        }
        __syncthreads();
      }
      if (finisher) {
        if (tid < kRows) inv_s[tid] = lv.norm ? rsqrtf(inv_s[tid] / (float)lv.K + 1e-5f) : 1.f;
        if (tid == 0) l_cnt = 0;
        __syncthreads();

        // ---- LoRA expand of the rows routed to this group's site(s), added to the fp32 sums --------
        // column space of `red`: stream a, column nl  <->  red[a][mt][nl & 3][(m & 15) + 16 * (nl >> 2)]
        const int n0 = t0 * 16;  // first column of the group inside its site
        if (p.lora) {
          for (int m = tid; m < p.M; m += kThreads) {
            const int req = p.row_to_req ? p.row_to_req[m] : m;
            const int nslot = lv.pair ? 2 : 1;
            for (int a = 0; a < nslot; ++a) {
              int tenant = 0;
              const int slot = lv.pair ? a : si;
              const int r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, lv.site[slot], &tenant);
              if (r) {
                // the row's t is published by workgroups that finished their shrink items before streaming
                if (wait_counter(&lv.lora_cnt[slot * p.M + m], NC + 1)) {
                  const int idx = atomicAdd(&l_cnt, 1);
                  l_m[idx] = m; l_r[idx] = r; l_t[idx] = tenant; l_a[idx] = slot;
                } else {
                  *p.status = 1;
                }
              }
            }
          }
          __syncthreads();
          const int cnt = l_cnt, rmax = p.ad.r_max;
          const int ncol = lv.pair ? 32 : 64;  // columns a routed row touches in this group
          for (int g0 = 0; g0 < cnt; g0 += kGroupRows) {
            const int ng = cnt - g0 < kGroupRows ? cnt - g0 : kGroupRows;
            for (int e = tid; e < ng * rmax; e += kThreads) {
              const int gi = e / rmax, c = e - gi * rmax, idx = g0 + gi;
              if (c < l_r[idx]) t_s[gi * rmax + c] = ld_agent(p.tfin + ((size_t)l_a[idx] * p.M + l_m[idx]) * rmax + c);
            }
            __syncthreads();
            // wave w takes ranks c = w, w+4, ...; lane = (row of a block of four, column quad)
            const int quad = lane & 15, rsub = lane >> 4;
            for (int gb = 0; gb < ng; gb += 4) {
              const int gi = gb + rsub;
              float d[4] = {0.f, 0.f, 0.f, 0.f};
              if (gi < ng && quad * 4 < ncol) {
                const int idx = g0 + gi, r = l_r[idx], slot = l_a[idx];
                const size_t ldb = (size_t)lv.N[slot];
                const int n = n0 + quad * 4;
                if (n < (int)ldb) {
                  const bf16_t* Bm = (const bf16_t*)p.ad.B[l_t[idx] * MILORA_NUM_SITES + lv.site[slot]] + n;
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
              const int a = (lv.pair ? 2 * l_a[idx] : 0) + (col >> 4), nl = col & 15;
              red[red_idx(a, m >> 4, nl & 3, (m & 15) + 16 * (nl >> 2))] += s;
            }
            __syncthreads();
          }
        }

        // ---- glue and stores: thread (row m, column pair) ---------------------------------------------
        const int nout = lv.pair ? 32 : 64;  // output columns of the group
        const int ppr = nout >> 1;           // column pairs per row
        const int n_lim = lv.N[si];
        for (int e = tid; e < p.M * ppr; e += kThreads) {
          const int m = e / ppr, pp = e - m * ppr;
          const int col = 2 * pp;
          const int n = n0 + col;
          if (n >= n_lim) continue;
          const int mt = m >> 4;
          const float inv = inv_s[m];
          float val[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int a = (col + q) >> 4, nl = (col + q) & 15;
            const int ln = (m & 15) + 16 * (nl >> 2);
            const float v0 = red[red_idx(a, mt, nl & 3, ln)] * inv;
            if (lv.pair) val[q] = silu(v0) * (red[red_idx(a + 2, mt, nl & 3, ln)] * inv);
            else val[q] = v0;
          }
          if (lv.bias[si]) {
            val[0] += bf16_to_f32(lv.bias[si][n]);
            val[1] += bf16_to_f32(lv.bias[si][n + 1]);
          }
          if (lv.resid_bf16) {
            const uint32_t rr = *reinterpret_cast<const uint32_t*>(lv.resid_bf16 + (size_t)m * lv.ld_resid + n);
            val[0] += __uint_as_float(rr << 16);
            val[1] += __uint_as_float(rr & 0xffff0000u);
          }
          if (lv.resid_f32) {
            const float* rr = lv.resid_f32 + (size_t)m * lv.ld_resid + n;
            val[0] += rr[0];
            val[1] += rr[1];
          }
          if (lv.out_f32) {
            st_agent(lv.out_f32 + (size_t)m * lv.ld_f32 + n, val[0]);
            st_agent(lv.out_f32 + (size_t)m * lv.ld_f32 + n + 1, val[1]);
          }
          const uint32_t packed = pack_bf16x2(val[0], val[1]);
          if (lv.out_rm[si]) *reinterpret_cast<uint32_t*>(lv.out_rm[si] + (size_t)m * lv.ld_rm + lv.col_off[si] + n) = packed;
          if (lv.out_pk[si]) st_agent(reinterpret_cast<uint32_t*>(lv.out_pk[si] + packed_act_offset(m, n, MT)), packed);
        }
      }
      __syncthreads();  // `red` and the lists are free for the next segment
    }

    // ---- 3. grid barrier: the next level reads what every workgroup of this one wrote ---------------
    if (L + 1 < p.n_levels) {
      wait_own_stores();
      __syncthreads();
      if (tid == 0) {
        __hip_atomic_fetch_add(p.bar, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!wait_counter(p.bar, G * (L + 1))) *p.status = 1;
      }
      __syncthreads();
    }
  }
}

// Zero the synchronisation block and re-order up to two row-major activation tensors into block-packed form.
template <int MT>
__global__ void __launch_bounds__(kThreads) prep_kernel(int* sync, int n_sync, const u32x4* __restrict__ src0,
                                                        u32x4* __restrict__ dst0, int K0,
                                                        const u32x4* __restrict__ src1, u32x4* __restrict__ dst1,
                                                        int K1, int M) {
  const size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (g < (size_t)n_sync) sync[g] = 0;
  const size_t n0 = src0 ? (size_t)(K0 >> 5) * MT * 64 : 0;
  const size_t n1 = src1 ? (size_t)(K1 >> 5) * MT * 64 : 0;
  const u32x4* src; u32x4* dst; int K; size_t q;
  if (g < n0) { src = src0; dst = dst0; K = K0; q = g; }
  else if (g < n0 + n1) { src = src1; dst = dst1; K = K1; q = g - n0; }
  else return;
  const int ln = (int)(q & 63);
  const size_t blk = q >> 6;
  const int mt = (int)(blk % MT), kt = (int)(blk / MT);
  int row = mt * 16 + (ln & 15);
  if (row > M - 1) row = M - 1;
  dst[q] = src[((size_t)row * K + kt * 32 + (ln >> 4) * 8) / 8];
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

int mt_for(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : (M <= 64 ? 4 : 8)); }
size_t rec_floats(int MT) { return (size_t)kNT * MT * 256 + MT * 16; }
int groups_of(int N) { return ((N >> 4) + kNT - 1) / kNT; }

template <int MT> constexpr int ring_depth() { return MT <= 2 ? 4 : (MT == 4 ? 3 : 2); }

// Workgroups of the persistent launch: one or two per CU, all resident at once (the grid barrier and the
// bounded waits rely on that), never more than the work can feed.
template <int MT>
int persistent_grid() {
  static int cached = 0;
  if (cached) return cached;
  int dev = 0, cus = 0, occ = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, decode_persist_kernel<MT, ring_depth<MT>()>, kThreads, 0) !=
      hipSuccess)
    return 0;
  if (occ < 1) return 0;
  cached = cus * (occ >= 2 ? 2 : 1);
  return cached;
}

int grid_for(int MT) {
  switch (MT) {
    case 1: return persistent_grid<1>();
    case 2: return persistent_grid<2>();
    case 4: return persistent_grid<4>();
    default: return persistent_grid<8>();
  }
}

int launch_persist(const DecodeParams& p, int MT, int G, hipStream_t st) {
  switch (MT) {
    case 1: hipLaunchKernelGGL((decode_persist_kernel<1, ring_depth<1>()>), dim3(G), dim3(kThreads), 0, st, p); break;
    case 2: hipLaunchKernelGGL((decode_persist_kernel<2, ring_depth<2>()>), dim3(G), dim3(kThreads), 0, st, p); break;
    case 4: hipLaunchKernelGGL((decode_persist_kernel<4, ring_depth<4>()>), dim3(G), dim3(kThreads), 0, st, p); break;
    default: hipLaunchKernelGGL((decode_persist_kernel<8, ring_depth<8>()>), dim3(G), dim3(kThreads), 0, st, p); break;
  }
  return check_launch();
}

int launch_prep(int MT, int* sync, const bf16_t* src0, bf16_t* dst0, int K0, const bf16_t* src1, bf16_t* dst1, int K1,
                int M, hipStream_t st) {
  size_t n = kSync;
  const size_t np = (src0 ? (size_t)(K0 >> 5) * MT * 64 : 0) + (src1 ? (size_t)(K1 >> 5) * MT * 64 : 0);
  if (np > n) n = np;
  const unsigned blocks = (unsigned)((n + kThreads - 1) / kThreads);
#define MILORA_PREP(MTV)                                                                                       \
  hipLaunchKernelGGL(prep_kernel<MTV>, dim3(blocks), dim3(kThreads), 0, st, sync, kSync, (const u32x4*)src0, \
                     (u32x4*)dst0, K0, (const u32x4*)src1, (u32x4*)dst1, K1, M)
  switch (MT) {
    case 1: MILORA_PREP(1); break;
    case 2: MILORA_PREP(2); break;
    case 4: MILORA_PREP(4); break;
    default: MILORA_PREP(8); break;
  }
#undef MILORA_PREP
  return check_launch();
}

void reset_level(LevelDesc& l) {
  l.X = nullptr; l.K = 0; l.n_seg = 0; l.pair = 0; l.norm = 0; l.groups = 0;
  for (int s = 0; s < 3; ++s) {
    l.W[s] = nullptr; l.N[s] = 0; l.site[s] = 0; l.grp_end[s] = 0;
    l.bias[s] = nullptr; l.out_rm[s] = nullptr; l.out_pk[s] = nullptr; l.col_off[s] = 0;
  }
  l.lora_cnt = nullptr; l.k_cnt = nullptr;
  l.resid_bf16 = nullptr; l.resid_f32 = nullptr; l.ld_resid = 0;
  l.out_f32 = nullptr; l.ld_f32 = 0; l.ld_rm = 0;
}

// ---- workspace layout of the packed-weight decode paths -------------------------------------------
struct DecodeWs {
  int* sync;       // level counters, barrier word, status
  float* tpart;    // [3][M][NCmax][r_max]
  float* tfin;     // [3][M][r_max]
  float* kpart;    // [Gmax][2][record]
  float* h_f32;    // [M][d]
  bf16_t* pk_x;    // packed x                      (K = d)
  bf16_t* pk_v;    // packed a = v or attn_out      (K = d)
  bf16_t* pk_h;    // packed h                      (K = d)
  bf16_t* pk_m;    // packed m = silu(g) * u        (K = F)
  size_t bytes;
};

constexpr int kGridMax = 512;

DecodeWs carve_decode_ws(void* base, int M, int d, int F, int r_max) {
  const int MT = mt_for(M);
  const int big = F > d ? F : d;
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_s = take((size_t)kSync * sizeof(int));
  const size_t o_t = take((size_t)3 * M * shrink_chunks(big) * r_max * sizeof(float));
  const size_t o_f = take((size_t)3 * M * r_max * sizeof(float));
  const size_t o_k = take((size_t)kGridMax * 2 * rec_floats(MT) * sizeof(float));
  const size_t o_h = take((size_t)M * d * sizeof(float));
  const size_t o_x = take((size_t)MT * 16 * big * sizeof(bf16_t));
  const size_t o_v = take((size_t)MT * 16 * d * sizeof(bf16_t));
  const size_t o_hp = take((size_t)MT * 16 * d * sizeof(bf16_t));
  const size_t o_m = take((size_t)MT * 16 * F * sizeof(bf16_t));
  char* b = (char*)base;
  return DecodeWs{(int*)(b + o_s), (float*)(b + o_t), (float*)(b + o_f), (float*)(b + o_k), (float*)(b + o_h),
                  (bf16_t*)(b + o_x), (bf16_t*)(b + o_v), (bf16_t*)(b + o_hp), (bf16_t*)(b + o_m), off};
}

void fill_common(DecodeParams& p, const DecodeWs& ws, int M, int Breq, const AdapterView& ad, const int32_t* tenant_id,
                 const uint8_t* route, const int32_t* row_to_req) {
  p.M = M; p.Breq = Breq; p.ad = ad; p.tenant_id = tenant_id; p.route = route; p.row_to_req = row_to_req;
  p.lora = 1;
  p.tpart = ws.tpart; p.tfin = ws.tfin; p.kpart = ws.kpart;
  p.bar = ws.sync + kMaxLevels * kCntPerLevel;
  p.status = p.bar + 1;
  for (int L = 0; L < kMaxLevels; ++L) {
    reset_level(p.lv[L]);
    p.lv[L].lora_cnt = ws.sync + L * kCntPerLevel;
    p.lv[L].k_cnt = p.lv[L].lora_cnt + 3 * kMaxRows;
  }
}

}  // namespace

size_t decode_packed_workspace_bytes(int M, int d, int F, int r_max) { return carve_decode_ws(nullptr, M, d, F, r_max).bytes; }

// One decode step of a layer on packed weights: a preparation launch (zero the counters, pack x and
// attn_out) and one persistent launch over the four dependency levels.  With `marks`, an event is
// recorded after each of the two launches (slots 0 and 1).
int layer_decode_packed(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                        const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                        bf16_t* y, bf16_t* qkv_out, void* workspace, hipStream_t st, LaunchMarks* marks) {
  const int MT = mt_for(B);
  auto mark = [&](int slot) {
    if (marks && slot < marks->n) (void)hipEventRecord(marks->ev[slot], st);
  };
  if (3 * groups_of(d) > kMaxGroups || ((F >> 4) + 1) / 2 > kMaxGroups) return MILORA_ERANGE;
  int G = grid_for(MT);
  if (G <= 0) return hip_fail(hipGetLastError());
  if (G > kGridMax) G = kGridMax;
  DecodeWs ws = carve_decode_ws(workspace, B, d, F, ad.r_max);
  const int norm = (flags & MILORA_LAYER_RMSNORM) ? 1 : 0;
  int rc = launch_prep(MT, ws.sync, x, ws.pk_x, d, attn_out, ws.pk_v, d, B, st);
  if (rc) return rc;
  mark(0);
  DecodeParams p;
  fill_common(p, ws, B, B, ad, tenant_id, route, nullptr);
  p.n_levels = 4;
  {  // level 0: q, k, v from x
    LevelDesc& l = p.lv[0];
    l.X = ws.pk_x; l.K = d; l.n_seg = 3; l.norm = norm;
    for (int s = 0; s < 3; ++s) {
      l.W[s] = (const bf16_t*)wts->W[s]; l.N[s] = d; l.site[s] = s; l.grp_end[s] = (s + 1) * groups_of(d);
      l.out_rm[s] = qkv_out; l.col_off[s] = s * d;
    }
    l.groups = 3 * groups_of(d);
    l.ld_rm = 3 * d;
    if (!attn_out) l.out_pk[2] = ws.pk_v;
  }
  {  // level 1: h = x + L_o(a)
    LevelDesc& l = p.lv[1];
    l.X = ws.pk_v; l.K = d; l.n_seg = 1;
    l.W[0] = (const bf16_t*)wts->W[3]; l.N[0] = d; l.site[0] = 3; l.grp_end[0] = groups_of(d);
    l.groups = groups_of(d);
    l.resid_bf16 = x; l.ld_resid = d;
    l.out_f32 = ws.h_f32; l.ld_f32 = d;
    l.out_pk[0] = ws.pk_h;
  }
  {  // level 2: m = silu(L_gate(n(h))) * L_up(n(h))
    LevelDesc& l = p.lv[2];
    l.X = ws.pk_h; l.K = d; l.n_seg = 2; l.pair = 1; l.norm = norm;
    for (int s = 0; s < 2; ++s) { l.W[s] = (const bf16_t*)wts->W[4 + s]; l.N[s] = F; l.site[s] = 4 + s; }
    l.groups = ((F >> 4) + 1) / 2;
    l.out_pk[0] = ws.pk_m;
  }
  {  // level 3: y = h + L_down(m)
    LevelDesc& l = p.lv[3];
    l.X = ws.pk_m; l.K = F; l.n_seg = 1;
    l.W[0] = (const bf16_t*)wts->W[6]; l.N[0] = d; l.site[0] = 6; l.grp_end[0] = groups_of(d);
    l.groups = groups_of(d);
    l.resid_f32 = ws.h_f32; l.ld_resid = d;
    l.out_rm[0] = y; l.ld_rm = d;
  }
  rc = launch_persist(p, MT, G, st);
  if (rc) return rc;
  mark(1);
  return MILORA_OK;
}

// ---- one routed linear of M <= 128 rows on a packed weight ------------------------------------------
struct LinearWs {
  int* sync;
  float* tpart;
  float* tfin;
  float* kpart;
  bf16_t* pk_x;
  size_t bytes;
};

static LinearWs carve_linear_ws(void* base, int M, int d1, int r_max) {
  const int MT = mt_for(M);
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_s = take((size_t)kSync * sizeof(int));
  const size_t o_t = take((size_t)M * shrink_chunks(d1) * r_max * sizeof(float));
  const size_t o_f = take((size_t)M * r_max * sizeof(float));
  const size_t o_k = take((size_t)kGridMax * 2 * rec_floats(MT) * sizeof(float));
  const size_t o_x = take((size_t)MT * 16 * d1 * sizeof(bf16_t));
  char* b = (char*)base;
  return LinearWs{(int*)(b + o_s), (float*)(b + o_t), (float*)(b + o_f), (float*)(b + o_k), (bf16_t*)(b + o_x), off};
}

size_t routed_linear_packed_workspace_bytes(int M, int d1, int d2, int r_max) {
  (void)d2;
  return carve_linear_ws(nullptr, M, d1, r_max).bytes;
}

int routed_linear_packed(const bf16_t* X, int M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                         const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                         const uint8_t* route, int B, bf16_t* Y, void* workspace, hipStream_t st) {
  const int MT = mt_for(M);
  if (groups_of(d2) > kMaxGroups) return MILORA_ERANGE;
  int G = grid_for(MT);
  if (G <= 0) return hip_fail(hipGetLastError());
  if (G > kGridMax) G = kGridMax;
  LinearWs ws = carve_linear_ws(workspace, M, d1, ad.r_max);
  int rc = launch_prep(MT, ws.sync, X, ws.pk_x, d1, nullptr, nullptr, 0, M, st);
  if (rc) return rc;
  DecodeWs dw{};
  dw.sync = ws.sync; dw.tpart = ws.tpart; dw.tfin = ws.tfin; dw.kpart = ws.kpart;
  DecodeParams p;
  fill_common(p, dw, M, B, ad, tenant_id, route, row_to_req);
  p.n_levels = 1;
  LevelDesc& l = p.lv[0];
  l.X = ws.pk_x; l.K = d1; l.n_seg = 1;
  l.W[0] = W; l.N[0] = d2; l.site[0] = site; l.grp_end[0] = groups_of(d2);
  l.groups = groups_of(d2);
  l.bias[0] = bias;
  l.out_rm[0] = Y; l.ld_rm = d2;
  return launch_persist(p, MT, G, st);
}

int pack_weight(const void* src, void* dst, int d1, int d2, hipStream_t st) {
  const size_t groups = (size_t)d1 * d2 / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     (const u32x4*)src, (u32x4*)dst, d1, d2);
  return check_launch();
}

}  // namespace milora
