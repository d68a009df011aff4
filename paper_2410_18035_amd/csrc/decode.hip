// Decode-time routed LoRA linears on packed bf16 weights (paper Eq. 1; Sec. 3.3 route reuse).
//
// At decode the batch is skinny (B <= 128 rows) and every base weight is read exactly once per
// step, so everything is built around never letting the HBM stream of W stop.  Weights are
// pre-packed in 1 KiB blocks that already are 16x16x32 matrix-core operands (one wave load = one
// contiguous block).  A whole decode step of a layer is ONE launch of one workgroup per compute
// unit that walks the stages q,k,v | o | gate,up | down.  A workgroup has three kinds of waves:
//   * stream waves: each owns every kSW-th 32-input block of the workgroup's 16-column tiles and
//     keeps a ring of kD weight blocks in registers.  The ring is refilled in stage order without
//     regard to stage boundaries: weights do not depend on activations, so while a stage ends
//     (reduction, LoRA expand, stores, grid barrier, first inputs of the next stage) the loads of the
//     next stage's weights are already in flight and HBM stays busy.
//   * one loader wave: moves the stage input (row-major bf16 rows) through L2 into LDS in
//     matrix-core operand order, chunk by chunk, ahead of the stream waves.  It has its own
//     memory counter, so waiting for these late-issued loads does not drain the weight ring.
//   * one LoRA wave: forms partial shrinks t = x[chunk] . A[chunk] of routed rows, the wave that
//     delivers a row's last partial sums them in chunk order and publishes t.
// Stage end: the stream waves' partial tiles are summed in wave order through LDS, the LoRA expand
// t W^B of the routed rows is added in fp32, the layer glue (normalisation scale, residual,
// silu*up) applied, one rounding to bf16.  Stages that depend on each other are separated by a
// grid barrier of per-workgroup flags (monotone values, nothing to reset between launches).
// All sums run in a fixed order: results do not depend on timing.
#include <atomic>
#include <mutex>
#include <type_traits>

#include "common.h"

namespace milora {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 gu32x4;  // in global memory: loads count on the vector-memory counter only
typedef __attribute__((address_space(1))) u32x2 gu32x2;
typedef __attribute__((address_space(1))) bf16_t gbf16;  // adapter matrices are reached through pointer tables read at run time

namespace {

constexpr int kSW = 6;                  // stream waves per workgroup
constexpr int kLoaders = 1;             // waves that copy the stage input (the LoRA wave is the second one)
constexpr int kLoader = kSW;            // wave index of the (first) input loader
constexpr int kLora = kSW + 1;          // wave index of the LoRA wave
constexpr int kWaves = kSW + 2;
constexpr int kThreads = kWaves * 64;
constexpr int kMaxStages = 12;
constexpr int kMaxRows = MILORA_MAX_DECODE_BATCH;
constexpr int kMaxGrid = 1024;          // workgroups the barrier flags are sized for
constexpr int kMaxSplitGrid = 512;      // workgroups of a ksplit stage at most (their partial-tile table is sized for it)
constexpr int kShrinkChunk = 512;       // reduction rows per LoRA shrink item
constexpr int kSteady = 8;              // weight loads per stream wave in flight between stage ends
constexpr int kSpinLimit = 1 << 22;     // polls before a bounded wait gives up (unless the caller set another limit)
constexpr int kCtrlBytes = 12288;       // control block at the start of LDS
constexpr int kLdsBytes = 160 * 1024;       // all of a compute unit's LDS: one workgroup per unit
constexpr int kTraceSlots = 16;             // time stamps per (workgroup, stage, wave) of a tracing launch

// Per row-tile-count tuning: ring depth, tiles per workgroup and stage, stream waves that share a partial-tile
// area at a stage end, bytes of LDS for LoRA expands formed ahead of the stage end.
// (Ring depth: what a wave has asked for when a stage ends is in the way of the stage end's own round trips - stores,
// flags, the next stage's first input.  Twelve blocks per wave, 18 MB over the chip, against twenty-four: -3.7 us per
// layer step of the 7B shape; six: +5 us, the stream starves between stage ends.)
template <int MT> struct Cfg;
template <> struct Cfg<1> { static constexpr int D = 12, NS = 6, CHAIN = 1, DELTA = 8192; };
template <> struct Cfg<2> { static constexpr int D = 12, NS = 6, CHAIN = 1, DELTA = 8192; };
template <> struct Cfg<4> { static constexpr int D = 12, NS = 6, CHAIN = 3, DELTA = 8192; };
template <> struct Cfg<8> { static constexpr int D = 12, NS = 2, CHAIN = 3, DELTA = 2048; };

// Polls after which a bounded wait inside a launch gives up; the launches that follow a change use the new value.
std::atomic<int> g_wait_limit{kSpinLimit};

struct Stage {
  const bf16_t* X;  // input rows: row-major bf16 [M][ldx], or operand blocks (x_packed, see packed_x_offset)
  int ldx, K, x_packed;
  int n_seg, pair, norm;
  int sync_before;  // the input is produced by earlier stages of this launch: wait for the grid barrier
  int lora_shrink;  // this stage starts the shrinks of its sites (first stage of a level)
  int tpos0;        // shrink slot position of the level's first site (see shrink_slot)
  const bf16_t* W[3];
  int N[3], site[3];
  int unit0, units;  // this stage covers units [unit0, unit0 + units) of the level (tiles, or gate/up tile pairs),
  int cap;           // workgroup g taking units [g * cap, (g + 1) * cap) of them
  int ksplit;        // 2: workgroups 2 j and 2 j + 1 stream tiles 2 j and 2 j + 1 over one half of the reduction each
                     // (half the input rows per workgroup), swap the partial tile of the other's output tile through
                     // memory, and workgroup 2 j + h finishes tile 2 j + h.  One-site stages without normalisation.
  const bf16_t* bias[3];
  const bf16_t* resid_bf16;
  const float* resid_f32;
  int ld_resid;
  float* out_f32;
  int ld_f32;
  bf16_t* out[3];  // row-major outputs per site
  int ld_out[3];
  bf16_t* out_pk;  // output as operand blocks for a later stage of this launch (one-site and gate/up stages)
};

struct Params {
  int n_stages, M, Breq;
  AdapterView ad;
  const int32_t* tenant_id;
  const uint8_t* route;
  const int32_t* row_to_req;
  int lora;
  // LoRA shrinks, one slot per (row, site position inside its level): see shrink_slot
  float* tpart;   // [slots][nc_max][r_max] shrink partials t = x[chunk] . A[chunk]
  float* tfin;    // [slots][r_max] t = x . A: the partials summed in chunk order by the wave that wrote the last one
  int* tcount;    // [slots] partials written so far in this launch; zero between launches
  int* tready;    // [slots] launch epoch * 16 + (stage that ran the shrink) + 1 of the t in tfin
  int nc_max;
  float* wpart;   // wide kernel: [segments][tiles of a group][row tiles] partial tiles, 1 KiB each
  float* wss;     // wide kernel: [segments][rows] sums of squares of the input rows over the segment
  int* segflag;   // wide kernel: [segments] launch epoch * 16 + level of the segment stored there
  int wsegs;      // wide kernel: segments per table half (even levels use the first half of the three tables, odd the second)
  int* tpflag;    // wide kernel: [slots][kTpStride] launch epoch * 16 + level + 1 of the shrink partial of each k chunk
  float* delta;   // wide kernel: LoRA terms t W^B as fp32 tiles [site tile][row tile][256], laid out like the partial tiles;
                  // tiles of even levels first, those of odd levels from tile delta_odd on
  int* dready;    // wide kernel: [level parity][site position][slab of 256 columns][row] tag of the LoRA term stored there
  int delta_odd, slabs_max;
  int* flags;     // [kMaxGrid] grid barrier flags, monotone
  float* xpart;   // [kMaxSplitGrid][row tiles][256] partial tile a workgroup of a ksplit stage hands to its partner
  int* xflag;     // [kMaxGrid] launch epoch * 16 + stage + 1 of the partial tile stored there
  int* status;    // set to 1 when a bounded wait ran out
  int spin_limit; // polls before a bounded wait gives up
  long long* trace;  // tracing launches only: [workgroup][stage][wave][8] time stamps (100 MHz clock), see TS
  Stage st[kMaxStages];
};

struct Ctrl {
  unsigned long long tb_ptr[kMaxStages][8];
  int tb_seg[kMaxStages][8];
  int tb_tile[kMaxStages][8];
  int ns[kMaxStages];
  int x_ready[2];  // per loader wave: chunks it has landed, counted over all stages
  int x_done[8];
  int slot_turn[8];  // per partial-tile area: stream waves that have put their tiles in, counted over all stages
  int part_cnt;      // the same over all areas
  int sum_cnt;       // stream waves that have summed their share of the areas into `red`, over all stages
  int red_free;      // stages whose sums the tail waves are done with
  int tail_go;       // stages whose sums carry the LoRA terms (the loader wave may apply the glue)
  int tail_done;     // stages whose outputs the loader wave has stored
  int swap_done;     // stages whose halves of the sums the loader wave has exchanged with the partner workgroup
  int epoch;
  int l_cnt;
  int seg_arr[8];  // wide kernel: stream waves that have stored their part of a segment (segment number % 8)
  int lvl_arr[kMaxStages];  // wide kernel: waves that have finished the level (a wave with nothing to do in a level runs ahead)
  int shr_next[kMaxStages];  // wide kernel: shrink items of a level handed out so far (the LoRA and loader waves draw from it)
  int shr_ready;   // wide kernel: levels whose shrink list stands in s_rows
  int exp_next[kMaxStages];  // wide kernel: expand items of a level handed out so far
  int s_flag;
  int bar_seen;    // wide kernel: last level whose grid barrier the loader wave has seen open
  float ss_part[kSW][kMaxRows];
  float inv_rows[kMaxRows];
  int l_ms[3 * kMaxRows];  // LoRA terms that land in this workgroup's tiles: row | site position << 8
  // what the route table says about each row, looked up once per launch: the sites with a LoRA term (bit m =
  // site m, 0: none), tenant, rank
  int r_mask[kMaxRows], r_ten[kMaxRows], r_rank[kMaxRows];
  int s_rows[3 * kMaxRows];  // shrinks of the current level: row | site position << 8
  int s_cnt;
};
static_assert(sizeof(Ctrl) <= kCtrlBytes, "control block");

// Shrink slot of (row, site position inside the level).  A row has kSlotsPerRow slots: q,k,v and gate,up use positions
// 0..2, o and down position 3 - levels that reuse a position are always separated by a grid barrier, while o can
// follow q,k,v without one (attention output supplied by the caller), and with several sites per request a row
// can have a LoRA term in both.
constexpr int kSlotsPerRow = 4;
constexpr int kTpStride = 64;  // flag words per shrink slot: one per k chunk (reductions of up to 64 * kShrinkChunk)
__device__ __host__ __forceinline__ int shrink_slot(const Stage& sg, int m, int pos) { return m * kSlotsPerRow + sg.tpos0 + pos; }

// ---- memory-model helpers ---------------------------------------------------------------------------
__device__ __forceinline__ int ld_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte stores of data another workgroup reads inside this launch: written through to the memory all XCDs
// share (a plain store may stay in the writer's L2 until the launch ends).  The two idle cycles behind the store
// belong to it: a store of more than eight bytes still reads its data registers for two cycles after it issues,
// the compiler keeps vector writes away from them only for stores it can see, and it reuses these registers at
// once (seen: the next store's address computed into them, and address bits arriving as partial sums).
__device__ __forceinline__ void st_through(u32x4* p, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_through(f32x4* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// One 16-byte load that bypasses the caches (data stored through by another workgroup in this launch), complete
// when the function returns.
__device__ __forceinline__ f32x4 ld_through1(const f32x4* p) {
  f32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  return v;
}
// LDS flags between the waves of a workgroup.  LDS operations of a wave execute in order, so a flag
// written after data is seen after the data; the compiler is kept from moving accesses across.
__device__ __forceinline__ int ld_lds(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void st_lds(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }
__device__ __forceinline__ void wait_lds() {
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only: vmcnt and expcnt fields left at their maxima
}
// vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt and lgkmcnt left at their maxima).
template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
// LDS flag accesses the compiler does not see as LDS accesses: the loader's asynchronous global->LDS copies
// would otherwise be waited for before every poll.
__device__ __forceinline__ uint32_t lds_off(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ int lds_peek(uint32_t off) {
  int v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(off) : "memory");
  return v;
}
__device__ __forceinline__ void lds_poke(uint32_t off, int v) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(off), "v"(v) : "memory");
}
// Every memory operation of this wave has completed (stores acknowledged by L2).
__device__ __forceinline__ void wait_all_mem() { __builtin_amdgcn_s_waitcnt(0); }

// Activations handed from one stage to the next are stored as the 1 KiB operand blocks the matrix cores take:
// block (k / 32, m / 16), inside it lane (m % 16) + 16 * ((k % 32) / 8) holds 8 consecutive k.  Offset in elements.
__device__ __host__ __forceinline__ size_t packed_x_offset(int m, int k, int MT) {
  return ((((size_t)(k >> 5) * MT + (m >> 4)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
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

// Time stamp `slot` of this wave in stage L; compiled in only for the tracing instantiation of a kernel.
#define TS(slot)                                                                                              \
  do {                                                                                                        \
    if (TRACE && lane == 0) p.trace[(((size_t)wg * kMaxStages + L) * kWaves + w) * kTraceSlots + (slot)] = wall_clock64(); \
  } while (0)


// A bounded wait ran out (another launch holds compute units this one needs, or a fault elsewhere): record it and
// end this wave.  What it waited for never came, so nothing it would do next has its inputs; the waves and
// workgroups that wait for this one run out the same way, and the launch ends with every wave gone.
__device__ __forceinline__ void give_up(int* status) {
  st_agent(status, 1);
  wait_all_mem();
  __builtin_amdgcn_endpgm();
}

// Wait until every workgroup has published `target`.  One wave.
__device__ __forceinline__ bool grid_wait(const int* flags, int G, int target, int lane, int limit) {
  int spins = 0;
  for (;;) {
    bool ok = true;
    for (int i = lane; i < G; i += 64) ok = ok && (ld_agent(flags + i) - target >= 0);
    if (__all(ok)) break;
    if (++spins >= limit) return false;
    __builtin_amdgcn_s_sleep(2);
  }
  // No cache invalidation here: what later stages read (the packed activations, the fp32 residual) is written
  // once per launch, with write-through stores, before anybody reads it in that launch, and a launch starts
  // with clean caches - so neither L2 nor L1 can hold an older copy.  (An acquire fence at this point throws away
  // the XCD's L2 lines of the stage input that the workgroups ahead of this one have just fetched.)
  compiler_fence();
  return true;
}

// ---- one LoRA shrink item by one wave: partial t of row m over one k chunk ---------------------------
template <int MT, bool PER_CHUNK = false, int BATCH = 32>
__device__ __forceinline__ void lora_shrink_item(const Params& p, const Stage& sg, int m, int pos, int tenant, int r,
                                                 int kc, int NC, int tag, int lane, long long* ts = nullptr) {
  const int site = sg.site[pos], slot = shrink_slot(sg, m, pos);
  const gbf16* A = (const gbf16*)p.ad.A[tenant * MILORA_NUM_SITES + site];
  const int K = sg.K, rmax = p.ad.r_max;
  const int k_lo = kc * kShrinkChunk;
  const int k_hi = k_lo + kShrinkChunk < K ? k_lo + kShrinkChunk : K;
  const bf16_t* const Xp = sg.X;
  const bool xpk = sg.x_packed != 0;
  const size_t xld = sg.ldx;
  auto xval = [&](int k) __attribute__((always_inline)) -> float {
    return bf16_to_f32(Xp[xpk ? packed_x_offset(m, k, MT) : (size_t)m * xld + k]);
  };
  float* row_part = p.tpart + ((size_t)slot * p.nc_max) * rmax;
  float* out = row_part + (size_t)kc * rmax;
  const int lpr = r >> 3;  // lanes per row of A when r is a multiple of 8
  if ((r & 7) == 0 && (lpr & (lpr - 1)) == 0 && lpr <= 32 && ((uintptr_t)A & 15) == 0) {
    const int kpl = 64 / lpr;  // rows of A per wave load
    const int cg = lane & (lpr - 1), kr = lane / lpr;
    float acc[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) acc[v] = 0.f;
    const gu32x4* Ap = reinterpret_cast<const gu32x4*>(A) + cg;
    int k = k_lo + kr;
    for (; k + (BATCH - 1) * kpl < k_hi; k += BATCH * kpl) {  // rank 32, BATCH 32: the whole chunk in one round trip
      u32x4 a[BATCH];
      float x[BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        a[u] = __builtin_nontemporal_load(Ap + (size_t)(k + u * kpl) * lpr);
        x[u] = xval(k + u * kpl);
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          acc[2 * v] += x[u] * __uint_as_float(a[u][v] << 16);
          acc[2 * v + 1] += x[u] * __uint_as_float(a[u][v] & 0xffff0000u);
        }
    }
    for (; k < k_hi; k += kpl) {
      const u32x4 a = Ap[(size_t)k * lpr];
      const float x = xval(k);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        acc[2 * v] += x * __uint_as_float(a[v] << 16);
        acc[2 * v + 1] += x * __uint_as_float(a[v] & 0xffff0000u);
      }
    }
    // lanes with equal cg hold partial sums over different rows: fixed butterfly over the row bits
    for (int off = lpr; off < 64; off <<= 1)
#pragma unroll
      for (int v = 0; v < 8; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
    if (lane < lpr)
#pragma unroll
      for (int v = 0; v < 8; ++v) st_agent(out + lane * 8 + v, acc[v]);
  } else {
    for (int c = lane; c < r; c += 64) {
      float acc = 0.f;
      for (int k = k_lo; k < k_hi; ++k) acc += xval(k) * bf16_to_f32(A[(size_t)k * r + c]);
      st_agent(out + c, acc);
    }
  }
  if (ts && lane == 0) ts[0] = wall_clock64();  // loads and sums done, partial stores issued
  wait_all_mem();
  if (ts && lane == 0) ts[1] = wall_clock64();  // partial stores acknowledged
  if (PER_CHUNK) {  // readers wait for the chunks' flags and add the partials themselves, in chunk order
    st_agent(p.tpflag + slot * kTpStride + kc, tag);  // (every lane stores the same word: no one-lane region at the item's end)
    return;
  }
  // The wave that completes the row's last partial adds all of them in chunk order (whoever it is: the order
  // of the sum is fixed) and publishes t; every workgroup with a tile of the site reads it from there.
  int done = 0;
  if (lane == 0) done = __hip_atomic_fetch_add(&p.tcount[slot], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
  done = __builtin_amdgcn_readfirstlane(done);
  if (ts && lane == 0) ts[2] = wall_clock64();  // arrival counted
  if (done == NC) {
    for (int c = lane; c < r; c += 64) {
      const float* tp = row_part + c;
      float t = 0.f;
      for (int k0 = 0; k0 < NC; k0 += 8) {  // eight loads in flight, added in chunk order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = ld_agent(tp + (size_t)(k0 + u < NC ? k0 + u : NC - 1) * rmax);
#pragma unroll
        for (int u = 0; u < 8; ++u) t += k0 + u < NC ? v[u] : 0.f;
      }
      st_agent(p.tfin + (size_t)slot * rmax + c, t);
    }
    wait_all_mem();
    if (lane == 0) {
      st_agent(&p.tcount[slot], 0);
      st_agent(&p.tready[slot], tag);
    }
    if (ts && lane == 0) ts[3] = wall_clock64();  // the row's shrink summed and published
  }
}

template <int MT, bool TRACE>
__global__ void __launch_bounds__(kThreads) decode_stream_kernel(const Params p) {
  constexpr int D = Cfg<MT>::D, NSMAX = Cfg<MT>::NS, CHAIN = Cfg<MT>::CHAIN;
  constexpr int kSlots = kSW / CHAIN;                     // partial-tile areas of the stream waves at a stage end
  constexpr int kChunkBlocks = kSW;                       // k blocks per input chunk: one per stream wave
  constexpr int kChunkBytes = kChunkBlocks * MT * 1024;
  constexpr int kTileBytes = MT * 1024;                   // fp32 sums of one 16-column tile
  constexpr int kRedBytes = NSMAX * kTileBytes;
  constexpr int kDeltaBytes = Cfg<MT>::DELTA;
  constexpr int kTBytes = MT == 8 ? 2048 : 4096;                       // summed shrinks t of the rows expanded ahead of the stage end
  constexpr int kPool0 = kCtrlBytes + kRedBytes + kDeltaBytes + kTBytes;  // input chunks grow up from here, slots lie at the top
  static_assert(kSW % CHAIN == 0, "slots");
  static_assert(kLdsBytes - kSlots * kRedBytes - kPool0 >= 2 * kChunkBytes, "at least two input chunks next to the largest slots");
  extern __shared__ __align__(16) unsigned char smem[];
  Ctrl& c = *reinterpret_cast<Ctrl*>(smem);
  float* const red = reinterpret_cast<float*>(smem + kCtrlBytes);
  float* const delta = reinterpret_cast<float*>(smem + kCtrlBytes + kRedBytes);
  float* const t_lds = reinterpret_cast<float*>(smem + kCtrlBytes + kRedBytes + kDeltaBytes);
  unsigned char* const xreg = smem + kPool0;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x, G = gridDim.x;

  // ---- this workgroup's tiles in every stage -----------------------------------------------------------
  if (tid < kMaxStages * 8) {
    const int L = tid >> 3, a = tid & 7;
    if (L < p.n_stages && p.st[L].ksplit == 2) {
      // tiles 2 j, 2 j + 1 over half wg % 2 of the reduction; the tail waves see one tile: the one this workgroup finishes
      const Stage& s = p.st[L];
      const bool has = 2 * (wg >> 1) + 1 < s.units;
      if (a == 0) c.ns[L] = has ? 2 : 0;
      if (a < 2 && has) {
        const int tile = s.unit0 + 2 * (wg >> 1) + a;
        const unsigned long long kt_half = (unsigned long long)(s.K >> 6);
        c.tb_ptr[L][a] = (unsigned long long)(uintptr_t)s.W[0] + ((unsigned long long)tile * (s.K >> 5) + (wg & 1) * kt_half) * 1024ull;
        c.tb_seg[L][a] = a == 0 ? 0 : -1;
        c.tb_tile[L][a] = s.unit0 + 2 * (wg >> 1) + (wg & 1);
      }
    } else if (L < p.n_stages) {
      const Stage& s = p.st[L];
      const int f0 = wg * s.cap < s.units ? wg * s.cap : s.units, f1 = f0 + s.cap < s.units ? f0 + s.cap : s.units;
      const int u0 = s.unit0 + f0, u1 = s.unit0 + f1;
      const int ns = s.pair ? 2 * (u1 - u0) : (u1 - u0);
      int ns_pad = ns;  // the ring rounds serve the tile counts that divide NSMAX
      while (ns_pad > 0 && NSMAX % ns_pad != 0) ++ns_pad;
      if (a == 0) c.ns[L] = ns_pad;
      if (a >= ns && a < ns_pad) {  // filler: streams the first tile again (valid memory), result dropped
        c.tb_ptr[L][a] = (unsigned long long)(uintptr_t)s.W[0];
        c.tb_seg[L][a] = -1;
        c.tb_tile[L][a] = 0;
      }
      if (a < ns) {
        int seg, tile;
        if (s.pair) {
          seg = a & 1;
          tile = u0 + (a >> 1);
        } else {
          int u = u0 + a;
          seg = 0;
          while (seg + 1 < s.n_seg && u >= (s.N[seg] >> 4)) {
            u -= s.N[seg] >> 4;
            ++seg;
          }
          tile = u;
        }
        c.tb_ptr[L][a] = (unsigned long long)(uintptr_t)s.W[seg] + (unsigned long long)tile * (s.K >> 5) * 1024ull;
        c.tb_seg[L][a] = seg;
        c.tb_tile[L][a] = tile;
      }
    }
  }
  if (tid == 0) {
    c.x_ready[0] = 0;
    c.x_ready[1] = 0;
    c.part_cnt = 0;
    c.swap_done = 0;
    c.sum_cnt = 0;
    c.red_free = 0;
    c.tail_go = 0;
    c.tail_done = 0;
    c.s_flag = 0;
    c.epoch = (ld_agent(p.flags + wg) >> 4) + 1;
  }
  if (tid < 8) {
    c.x_done[tid] = 0;
    c.slot_turn[tid] = 0;
  }
  if (tid >= 64 && tid < 64 + kMaxRows) {
    const int m = tid - 64;
    int mask = 0, tenant = 0, r = 0;
    if (m < p.M && p.lora) {
      const int req = p.row_to_req ? p.row_to_req[m] : m;
      if (req >= 0 && req < p.Breq) {
        const uint8_t rb = p.route[req];
        for (int st = 0; st < MILORA_NUM_SITES; ++st)
          if (route_has(rb, st)) {
            r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, st, &tenant);  // the same for every chosen site
            if (r > 0) mask |= 1 << st;
          }
      }
    }
    c.r_mask[m] = mask;
    c.r_ten[m] = tenant;
    c.r_rank[m] = r;
  }
  __syncthreads();
  const int epoch = __builtin_amdgcn_readfirstlane(c.epoch);

  // A stage's reduction is cut into chunks of kSW k blocks, one per stream wave.  Every workgroup walks the
  // chunks in its own rotation (start_of): the workgroups of an XCD all read the same input rows, and in
  // lockstep they would all hit the same few L2 channels.
  // k blocks of a stage that this workgroup walks (half of them in a ksplit stage) and the first of them
  auto kt_of = [&](const Stage& sg) __attribute__((always_inline)) -> int { return sg.ksplit == 2 ? sg.K >> 6 : sg.K >> 5; };
  auto kb0_of = [&](const Stage& sg) __attribute__((always_inline)) -> int { return sg.ksplit == 2 ? (wg & 1) * (sg.K >> 6) : 0; };
  auto chunks_of = [&](int ns, int kt) __attribute__((always_inline)) -> int { return ns > 0 ? (kt + kSW - 1) / kSW : 0; };
  auto rounds_of = [&](int ns, int nch) __attribute__((always_inline)) -> int { return (ns * nch + D - 1) / D; };
  auto start_of = [&](int nch) __attribute__((always_inline)) -> int {
    const int per_xcd = (G + 7) >> 3;
    return nch > 0 ? (int)(((long)(wg >> 3) * nch) / per_xcd) % nch : 0;
  };
  // LDS of a stage in which the workgroup holds ns tiles: kSlots areas of ns tiles at the top, input chunk
  // buffers below them.
  auto slots_off = [&](int ns) __attribute__((always_inline)) -> int { return kLdsBytes - kSlots * ns * kTileBytes; };
  auto nbuf_of = [&](int ns) __attribute__((always_inline)) -> int { return (slots_off(ns) - kPool0) / kChunkBytes; };
  auto spin_until = [&](auto cond) __attribute__((always_inline)) {
    int spins = 0;
    while (!cond()) {
      if (++spins >= p.spin_limit) give_up(p.status);
      __builtin_amdgcn_s_sleep(1);
    }
    compiler_fence();
  };
  // one wave: LDS written by some lanes is read by others afterwards
  auto wave_sync = [&]() __attribute__((always_inline)) {
    compiler_fence();
    wait_lds();
    compiler_fence();
  };

  if (w < kSW) {
    // ===================================== stream waves =====================================
    // These waves wait for LDS words only and address memory through nothing they wait for: after a wait that ran
    // out (the loader or the LoRA wave has given up) they record it, skip every later wait and run to the end of
    // their loop on whatever the buffers hold.
    bool dead = false;
    auto spin_until = [&](auto cond) __attribute__((always_inline)) {
      int spins = 0;
      while (!dead && !cond()) {
        if (++spins >= p.spin_limit) {
          st_agent(p.status, 1);
          dead = true;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      compiler_fence();
    };
    u32x4 ring[D];
    f32x4 acc[NSMAX][MT];
    // producer state, uniform over the wave
    int p_stage = -1, p_a = 0, p_cur = 0, p_nch = 1, p_ns = 1, p_kt = 0, p_left = 0;
    uint32_t p_tlo = 0, p_thi = 0;  // lane a: pointer to the first block of tile a of the producer's stage
    unsigned long long p_last = (unsigned long long)(uintptr_t)p.st[0].W[0];
    auto prod_advance = [&]() __attribute__((always_inline)) {
      int ns = 1, kt = 0, left = 0, nch = 1;
      for (;;) {
        ++p_stage;
        if (p_stage >= p.n_stages) break;
        ns = __builtin_amdgcn_readfirstlane(c.ns[p_stage]);
        kt = kt_of(p.st[p_stage]);
        nch = chunks_of(ns, kt);
        left = rounds_of(ns, nch) * D;
        if (left > 0) break;
      }
      // past the last stage the producer keeps re-reading the last block (ring slots are always refilled)
      const bool live = p_stage < p.n_stages;
      const unsigned long long tp = c.tb_ptr[live ? p_stage : 0][lane & 7];
      p_ns = live ? ns : 1;
      p_kt = live ? kt : 0;
      p_left = live ? left : 0x7ffffff0;
      p_a = 0;
      p_nch = live ? nch : 1;
      p_cur = live ? start_of(nch) : 0;
      p_tlo = (uint32_t)tp;
      p_thi = (uint32_t)(tp >> 32);
    };
    auto prod_next = [&]() __attribute__((always_inline)) -> const gu32x4* {
      const int kb = w + kSW * p_cur;
      if (kb < p_kt) {
        const uint32_t lo = __builtin_amdgcn_readlane(p_tlo, p_a), hi = __builtin_amdgcn_readlane(p_thi, p_a);
        p_last = (((unsigned long long)hi << 32) | lo) + ((unsigned long long)kb << 10);
      }
      if (++p_a == p_ns) {
        p_a = 0;
        if (++p_cur == p_nch) p_cur = 0;
      }
      return reinterpret_cast<const gu32x4*>(p_last) + lane;
    };
    auto prod_round_end = [&]() __attribute__((always_inline)) {
      p_left -= D;
      if (p_left == 0) prod_advance();
    };
    prod_advance();
#pragma unroll
    for (int s = 0; s < D; ++s) {
      ring[s] = __builtin_nontemporal_load(prod_next());
      __builtin_amdgcn_sched_barrier(0);
    }
    prod_round_end();

    int nseq = 0;            // input chunks of the earlier stages
    int lbase[2] = {0, 0};   // ... and how many of them each loader wave brought
    for (int L = 0; L < p.n_stages; ++L) {
      const Stage& sg = p.st[L];
      const int KT = kt_of(sg);
      const int NS = __builtin_amdgcn_readfirstlane(c.ns[L]);
      const int NCH = chunks_of(NS, KT);
      const int NBUF = nbuf_of(NS);
      TS(0);
#pragma unroll
      for (int a = 0; a < NSMAX; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[a][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      // Sums of squares of the input rows over this wave's k blocks (normalisation).  Up to 32 rows the matrix cores
      // form them: the product of an operand block with itself has them on its diagonal, one instruction per row
      // tile and k block where the vector unit needs sixteen (the stream waves are bound by instruction issue).
      constexpr bool kGramSS = MT <= 2;
      float ss[MT];
      f32x4 ssg[kGramSS ? MT : 1];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) ss[mt] = 0.f;
#pragma unroll
      for (int mt = 0; mt < (kGramSS ? MT : 1); ++mt) ssg[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int rounds = rounds_of(NS, NCH);
      // Ring rounds.  Slot s of a round holds tile s % NS of the wave's next k block; NS divides NSMAX and the
      // accumulator of slot s is s % NSMAX, so one piece of code serves every NS that divides NSMAX, and
      // accumulators that met the same tile are added up afterwards.  The last round of a stage can hold slots
      // past the end of the reduction; there both operands are zeroed instead of branching around the matrix
      // instruction.
      if (rounds > 0) {
        static_assert(D % NSMAX == 0, "ring rounds must hold whole k blocks");
        u32x4 xb[MT], xn[MT];  // operand blocks of the current k block and, when it was there in time, the next one
        bool have_next = false;
        int seen[2] = {0, 0};  // input chunks known to have landed (cached copies of the loaders' counters)
        const bool norm = sg.norm != 0;
        // this lane's (row lane % 16, k group lane / 16) inside an input block: packed blocks hold it at slot
        // lane, gathered row-major blocks at slot row * 4 + k group
        const int rd_off = sg.x_packed ? lane * 16 : ((lane & 15) * 4 + (lane >> 4)) * 16;
        int i = 0, cur = start_of(NCH), ac = 0;  // chunks begun, chunk index in this workgroup's rotation, tile
        int bufi = 0;                            // i % NBUF, kept by counting: a division per chunk is paid in issue slots
        uint32_t wmask = 0xffffffffu;
        for (int r = 0; r < rounds; ++r) {
#pragma unroll
          for (int s = 0; s < D; ++s) {
            if (ac == 0) {
              const bool cvalid = i < NCH && (w + kSW * cur) < KT;
              if (i < NCH) {
                // next input chunk: report the previous ones finished, make sure this one has landed
                compiler_fence();
                st_lds(&c.x_done[w], nseq + i);
                if (!have_next) {
                  if (seen[i % kLoaders] <= lbase[i % kLoaders] + i / kLoaders) {
                    spin_until([&]() { return (seen[i % kLoaders] = ld_lds(&c.x_ready[i % kLoaders])) > lbase[i % kLoaders] + i / kLoaders; });
                  }
                  const unsigned char* xbuf = xreg + bufi * kChunkBytes;
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt)
                    xb[mt] = *reinterpret_cast<const u32x4*>(xbuf + ((w * MT + mt) << 10) + rd_off);
                } else {
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt) xb[mt] = xn[mt];
                }
                if (TRACE && i == 0) TS(1);
                // the chunk after it, if the loader is that far: its LDS reads overlap this k block's work
                have_next = i + 1 < NCH && seen[(i + 1) % kLoaders] > lbase[(i + 1) % kLoaders] + (i + 1) / kLoaders;
                if (have_next) {
                  const unsigned char* xbuf = xreg + (bufi + 1 == NBUF ? 0 : bufi + 1) * kChunkBytes;
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt)
                    xn[mt] = *reinterpret_cast<const u32x4*>(xbuf + ((w * MT + mt) << 10) + rd_off);
                }
              }
              wmask = cvalid ? 0xffffffffu : 0u;
              if (!cvalid) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) xb[mt] = u32x4{0u, 0u, 0u, 0u};
              }
              if (norm && cvalid) {
                if constexpr (kGramSS) {
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt)
                    ssg[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xb[mt]), __builtin_bit_cast(bf16x8, xb[mt]),
                                                                      ssg[mt], 0, 0, 0);
                } else {
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt) ss[mt] += sumsq8(xb[mt]);
                }
              }
            }
            // Between stage ends only kSteady loads per wave stay in flight (the rest of the ring holds blocks that
            // have landed): deeper queues of weight loads delay the input loader's loads behind them.  In the last
            // round of a stage the landed blocks are used up without this wait, so the ring is all in flight,
            // next stage's weights, when the stage end stalls this wave.
            if (r + 1 < rounds) wait_vm<kSteady - 1>();
            const u32x4 wv = ring[s] & wmask;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[s % NSMAX][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  __builtin_bit_cast(bf16x8, wv), __builtin_bit_cast(bf16x8, xb[mt]), acc[s % NSMAX][mt], 0, 0, 0);
            ring[s] = __builtin_nontemporal_load(prod_next());
            if (++ac == NS) {
              ac = 0;
              ++i;
              if (++bufi == NBUF) bufi = 0;
              if (++cur == NCH) cur = 0;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          prod_round_end();
        }
        // accumulators that met the same tile, added in a fixed order
#pragma unroll
        for (int q = 1; q < NSMAX; ++q)
#pragma unroll
          for (int t = 0; t < q; ++t)
            if (q % NS == t)
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) acc[t][mt] += acc[q][mt];
      }
      TS(2);
      compiler_fence();
      st_lds(&c.x_done[w], nseq + NCH);
      nseq += NCH;
      lbase[0] += (NCH + kLoaders - 1) / kLoaders;
      lbase[1] += kLoaders > 1 ? NCH / kLoaders : 0;

      // ---- stage end: the waves' partial tiles meet in LDS ------------------------------------------------
      // Wave w puts its partial tiles into slot w / CHAIN (the first wave of a slot stores, the others add in
      // wave order); when all have, each wave sums a sixth of the elements over the slots, in slot order, into
      // `red`.  Then the wave goes on to the next stage; the two other waves finish this one.
      if (NS > 0) {
        const int slot = w / CHAIN, pos = w % CHAIN;
        float* const sl = reinterpret_cast<float*>(smem + slots_off(NS) + slot * NS * kTileBytes);
        // the slots may overlap the previous stage's slots or input chunks: everything of that stage is summed
        spin_until([&]() { return ld_lds(&c.sum_cnt) >= L * kSW && ld_lds(&c.slot_turn[slot]) >= L * CHAIN + pos; });
#pragma unroll
        for (int a = 0; a < NSMAX; ++a)
          if (a < NS)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                float* e = sl + ((a * MT + mt) * 4 + q) * 64 + lane;
                *e = (pos == 0 ? 0.f : *e) + acc[a][mt][q];
              }
        if constexpr (kGramSS) {
          // a lane holds rows 4 (lane / 16) .. + 3 of column lane % 16 of the product: the diagonal element of row
          // j = lane % 16 lies in the lane with lane / 16 == j / 4, at index j % 4
          const int j = lane & 15;
          if ((lane >> 4) == (j >> 2)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              const f32x4 g = ssg[mt];
              const float lo = (j & 1) ? g[1] : g[0], hi = (j & 1) ? g[3] : g[2];
              c.ss_part[w][mt * 16 + j] = (j & 2) ? hi : lo;
            }
          }
        } else {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            float v = ss[mt];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (lane < 16) c.ss_part[w][mt * 16 + lane] = v;
          }
        }
        compiler_fence();
        wait_lds();
        st_lds(&c.slot_turn[slot], L * CHAIN + pos + 1);
        if (lane == 0) __hip_atomic_fetch_add(&c.part_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        // all partial tiles are in, and the tail waves are done with the sums of the previous stage
        spin_until([&]() { return ld_lds(&c.part_cnt) >= (L + 1) * kSW && ld_lds(&c.red_free) >= L; });
        const int E = NS * MT * 256, e0 = (E * w) / kSW, e1 = (E * (w + 1)) / kSW;
        const float* const s0 = reinterpret_cast<const float*>(smem + slots_off(NS));
        for (int e = e0 + lane; e < e1; e += 64) {
          float s = s0[e];
#pragma unroll
          for (int q = 1; q < kSlots; ++q) s += s0[q * E + e];
          red[e] = s;
        }
        compiler_fence();
        wait_lds();
      } else {
        spin_until([&]() { return ld_lds(&c.sum_cnt) >= L * kSW; });
        if (lane == 0) __hip_atomic_fetch_add(&c.part_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (lane == 0) __hip_atomic_fetch_add(&c.slot_turn[w / CHAIN], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      TS(3);
      if (lane == 0) __hip_atomic_fetch_add(&c.sum_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    return;
  }

  // ======================== the two tail waves: input loader and LoRA wave ========================
  // Stage end, run by these two waves while the stream waves already wait for the next stage's input: the LoRA
  // expand (formed by the LoRA wave during the stage, in `delta`) is added to the fp32 sums, then both waves
  // apply the layer glue to half of the outputs each and store them, and the LoRA wave raises the hand-over flag.
  auto red_idx = [&](int a, int m, int nl) __attribute__((always_inline)) {
    return ((a * MT + (m >> 4)) * 4 + (nl & 3)) * 64 + (m & 15) + 16 * (nl >> 2);
  };
  // LoRA expand of list entries [l0, l1): lane = (entry, tile, column quad); added to `red` or stored in `delta`
  // shrink t[c] of row m, as published by the wave that summed the row's partials
  auto t_sum = [&](const Stage& sg, int m, int s, int c) __attribute__((always_inline)) -> float {
    return ld_agent(p.tfin + (size_t)shrink_slot(sg, m, s) * p.ad.r_max + c);
  };
  auto expand = [&](const int L, const Stage& sg, const int NS, const int NC, int l0, int l1, bool to_red) __attribute__((always_inline)) {
    const int work = (l1 - l0) * NS * 4;
    for (int e = lane; e < work; e += 64) {
      const int q = e & 3, a = (e >> 2) % NS, li = l0 + (e >> 2) / NS;
      const int s = c.l_ms[li] >> 8;
      float d[4] = {0.f, 0.f, 0.f, 0.f};
      const bool mine = c.tb_seg[L][a] == s;
      const int m = c.l_ms[li] & 0xff;
      if (mine) {
        const int r = c.r_rank[m];
        const int n = c.tb_tile[L][a] * 16 + q * 4;
        const size_t ldb = (size_t)sg.N[s];
        const gbf16* Bm = (const gbf16*)p.ad.B[c.r_ten[m] * MILORA_NUM_SITES + sg.site[s]] + n;
        const float* tv = t_lds + (size_t)li * p.ad.r_max;  // entries formed ahead of the stage end have t in LDS
        if (((uintptr_t)Bm & 7) == 0 && (ldb & 3) == 0) {
          int cc = 0;
          for (; cc + 16 <= r; cc += 16) {
            u32x2 bb[16];
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
              bb[u] = *reinterpret_cast<const gu32x2*>(Bm + (size_t)(cc + u) * ldb);
              t[u] = to_red ? t_sum(sg, m, s, cc + u) : tv[cc + u];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
              d[0] += t[u] * __uint_as_float(bb[u][0] << 16);
              d[1] += t[u] * __uint_as_float(bb[u][0] & 0xffff0000u);
              d[2] += t[u] * __uint_as_float(bb[u][1] << 16);
              d[3] += t[u] * __uint_as_float(bb[u][1] & 0xffff0000u);
            }
          }
          for (; cc < r; ++cc) {
            const u32x2 bb = *reinterpret_cast<const gu32x2*>(Bm + (size_t)cc * ldb);
            const float t = to_red ? t_sum(sg, m, s, cc) : tv[cc];
            d[0] += t * __uint_as_float(bb[0] << 16);
            d[1] += t * __uint_as_float(bb[0] & 0xffff0000u);
            d[2] += t * __uint_as_float(bb[1] << 16);
            d[3] += t * __uint_as_float(bb[1] & 0xffff0000u);
          }
        } else {
          for (int cc = 0; cc < r; ++cc) {
            const float t = to_red ? t_sum(sg, m, s, cc) : tv[cc];
#pragma unroll
            for (int z = 0; z < 4; ++z) d[z] += t * bf16_to_f32(Bm[(size_t)cc * ldb + z]);
          }
        }
      }
      if (to_red) {
        if (mine)
#pragma unroll
          for (int z = 0; z < 4; ++z) red[red_idx(a, m, q * 4 + z)] += d[z];
      } else {
#pragma unroll
        for (int z = 0; z < 4; ++z) delta[(((li - l0) * NS + a) * 4 + q) * 4 + z] = d[z];
      }
    }
  };
  // bias + residual of a lane's first output item, fetched while the stage still runs (the stages that have them,
  // o and down, give a lane at most one item per tile and row tile: the loads are off the stage end's path)
  auto glue_prefetch = [&](const int L, const Stage& sg, const int NS, const int half, float (&pre)[8]) __attribute__((always_inline)) {
#pragma unroll
    for (int z = 0; z < 8; ++z) pre[z] = 0.f;
    const int nout = sg.pair ? NS >> 1 : NS;
    const int e = half * 64 + lane;
    if (e >= nout * p.M * 2) return;
    const int hf = e & 1, m = (e >> 1) % p.M, ao = (e >> 1) / p.M;
    const int a = sg.pair ? 2 * ao : ao;
    if (c.tb_seg[L][a] < 0) return;
    const int s = sg.pair ? 0 : c.tb_seg[L][a];
    const int n = c.tb_tile[L][a] * 16 + hf * 8;
    if (sg.bias[s]) {
      const u32x4 bb = *reinterpret_cast<const u32x4*>(sg.bias[s] + n);
#pragma unroll
      for (int z = 0; z < 4; ++z) {
        pre[2 * z] += __uint_as_float(bb[z] << 16);
        pre[2 * z + 1] += __uint_as_float(bb[z] & 0xffff0000u);
      }
    }
    if (sg.resid_bf16) {
      const u32x4 rr = *reinterpret_cast<const u32x4*>(sg.resid_bf16 + (size_t)m * sg.ld_resid + n);
#pragma unroll
      for (int z = 0; z < 4; ++z) {
        pre[2 * z] += __uint_as_float(rr[z] << 16);
        pre[2 * z + 1] += __uint_as_float(rr[z] & 0xffff0000u);
      }
    }
    if (sg.resid_f32) {
      const f32x4* rr = reinterpret_cast<const f32x4*>(sg.resid_f32 + (size_t)m * sg.ld_resid + n);
      const f32x4 r0 = rr[0], r1 = rr[1];
#pragma unroll
      for (int z = 0; z < 4; ++z) {
        pre[z] += r0[z];
        pre[4 + z] += r1[z];
      }
    }
  };
  // glue and stores of half of the outputs: lane = (output tile, row, half of the tile's 16 columns)
  auto glue = [&](const int L, const Stage& sg, const int NS, const int half, const float (&pre)[8]) __attribute__((always_inline)) {
    const int nout = sg.pair ? NS >> 1 : NS;
    const int work = nout * p.M * 2;
    for (int e = half * 64 + lane; e < work; e += 128) {
      const bool first = e < 128;
      const int hf = e & 1, m = (e >> 1) % p.M, ao = (e >> 1) / p.M;
      const int a = sg.pair ? 2 * ao : ao;
      if (c.tb_seg[L][a] < 0) continue;  // filler tile: streamed to keep the ring rounds whole, result dropped
      const int s = sg.pair ? 0 : c.tb_seg[L][a];
      const int n = c.tb_tile[L][a] * 16 + hf * 8;
      const float inv = c.inv_rows[m];
      float val[8];
#pragma unroll
      for (int z = 0; z < 8; ++z) {
        const float v0 = red[red_idx(a, m, hf * 8 + z)] * inv;
        if (sg.pair) val[z] = silu(v0) * (red[red_idx(a + 1, m, hf * 8 + z)] * inv);
        else val[z] = v0;
      }
      if (first) {
#pragma unroll
        for (int z = 0; z < 8; ++z) val[z] += pre[z];
      } else {
        if (sg.bias[s]) {
          const u32x4 bb = *reinterpret_cast<const u32x4*>(sg.bias[s] + n);
#pragma unroll
          for (int z = 0; z < 4; ++z) {
            val[2 * z] += __uint_as_float(bb[z] << 16);
            val[2 * z + 1] += __uint_as_float(bb[z] & 0xffff0000u);
          }
        }
        if (sg.resid_bf16) {
          const u32x4 rr = *reinterpret_cast<const u32x4*>(sg.resid_bf16 + (size_t)m * sg.ld_resid + n);
#pragma unroll
          for (int z = 0; z < 4; ++z) {
            val[2 * z] += __uint_as_float(rr[z] << 16);
            val[2 * z + 1] += __uint_as_float(rr[z] & 0xffff0000u);
          }
        }
        if (sg.resid_f32) {
          const f32x4* rr = reinterpret_cast<const f32x4*>(sg.resid_f32 + (size_t)m * sg.ld_resid + n);
          const f32x4 r0 = rr[0], r1 = rr[1];
#pragma unroll
          for (int z = 0; z < 4; ++z) {
            val[z] += r0[z];
            val[4 + z] += r1[z];
          }
        }
      }
      if (sg.out_f32) {
        f32x4* oo = reinterpret_cast<f32x4*>(sg.out_f32 + (size_t)m * sg.ld_f32 + n);
        st_through(oo, f32x4{val[0], val[1], val[2], val[3]});
        st_through(oo + 1, f32x4{val[4], val[5], val[6], val[7]});
      }
      u32x4 o;
#pragma unroll
      for (int z = 0; z < 4; ++z) o[z] = pack_bf16x2(val[2 * z], val[2 * z + 1]);
      if (sg.out[s]) *reinterpret_cast<u32x4*>(sg.out[s] + (size_t)m * sg.ld_out[s] + n) = o;
      if (sg.out_pk && (sg.pair || s == sg.n_seg - 1)) st_through(reinterpret_cast<u32x4*>(sg.out_pk + packed_x_offset(m, n, MT)), o);
    }
  };

  // ---- input copies of one stage by loader wave `lj` of kLoaders (it takes every kLoaders-th chunk) ------------
  int lcount = 0;  // chunks this wave has brought in the earlier stages
  auto load_input = [&](const int L, const Stage& sg, const int KT, const int NS, const int NCH, const int NBUF,
                        const int nseq, const int lj) __attribute__((always_inline)) {
    const int kb_first = kb0_of(sg);  // the stage's k blocks this workgroup walks are kb_first .. kb_first + KT - 1
    if (NS > 0) {
        // A block is the 1 KiB operand of one k block and one 16-row tile; lane l of the consumer holds
        // (row l % 16, k group l / 16).  The copies go from global memory straight into LDS (lane l of a wave load
        // lands at base + 16 l) and take no registers, so many chunks can be in flight; a chunk is announced once
        // the memory counter shows it has landed.  Packed inputs are read as they lie (1 KiB contiguous per
        // load); row-major inputs are gathered, lane l reading the 16 bytes of (row l / 4, k group l % 4): four
        // lanes cover 64 contiguous bytes of a row, which the memory pipeline takes in one piece, and the stream
        // waves read such a block with the matching lane order.
        constexpr int LPC = kSW * MT;  // wave loads per chunk
        // chunks in flight: two (with one the stream waves wait for every chunk, with three to six the copies get in
        // the way of the weight stream: 125.8, 122.7, 124.3 .. 125.2 us per layer step of the 7B shape at 32 rows)
        constexpr int kDepth = 2;
        static_assert(LPC * (kDepth - 1) <= 63, "chunk too large for the memory counter");
        const unsigned char* const Xb = reinterpret_cast<const unsigned char*>(sg.X);
        const bool xpk = sg.x_packed != 0;
        size_t loff[MT];  // byte offset of this lane's 16 bytes for row tile mt inside k block 0
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          int row = mt * 16 + (lane >> 2);
          if (row > p.M - 1) row = p.M - 1;  // rows past the batch repeat the last one; their results are dropped
          loff[mt] = xpk ? (size_t)mt * 1024 + lane * 16 : ((size_t)row * sg.ldx + (lane & 3) * 8) * sizeof(bf16_t);
        }
        const size_t kstep = xpk ? (size_t)MT * 1024 : 64;  // bytes from one k block to the next
        const int rot = start_of(NCH);
        const uint32_t done_off = lds_off(&c.x_done[lane < kSW ? lane : 0]), ready_off = lds_off(&c.x_ready[lj]);
        const uint32_t sum_off = lds_off(&c.sum_cnt);
        // the chunk buffers may overlap the previous stage's slots: all of its partial tiles have been summed
        spin_until([&]() { return lds_peek(sum_off) >= L * kSW; });
        const int depth = kDepth * kLoaders <= NBUF ? kDepth : (NBUF / kLoaders > 0 ? NBUF / kLoaders : 1);  // own chunks in flight
        int done_seen = 0, mine = 0;  // own chunks issued
        for (int ch = lj; ch < NCH; ch += kLoaders, ++mine) {
          // the buffer's previous chunk (of this stage, or any chunk of an earlier stage) has been consumed by
          // every stream wave
          const int need = nseq + (ch >= NBUF ? ch - NBUF + 1 : 0);
          if (done_seen < need) {  // a cached minimum over the stream waves: LDS is asked only when it does not suffice
            spin_until([&]() {
              int v = lds_peek(done_off);
              v = lane < kSW ? v : 0x7fffffff;
#pragma unroll
              for (int off = 1; off < 8; off <<= 1) {
                const int o = __shfl_xor(v, off, 64);
                v = o < v ? o : v;
              }
              done_seen = __builtin_amdgcn_readfirstlane(v);
              return done_seen >= need;
            });
          }
          int cur = ch + rot;
          if (cur >= NCH) cur -= NCH;
          const int kb0 = cur * kSW;
          unsigned char* dst = xreg + (ch % NBUF) * kChunkBytes;
          // a ragged last chunk re-reads the last k block (valid memory); the stream waves zero what lies past K
#pragma unroll
          for (int pos = 0; pos < kSW; ++pos) {
            const int kb = kb0 + pos < KT ? kb0 + pos : KT - 1;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xb + (size_t)(kb_first + kb) * kstep + loff[mt]),
                                               (__attribute__((address_space(3))) void*)(dst + ((pos * MT + mt) << 10)), 16, 0, 0);
          }
          // with `depth` chunks in flight the oldest has landed once at most (depth - 1) chunks of loads are out
          if (mine + 1 >= depth) {
            if (depth == kDepth) wait_vm<LPC * (kDepth - 1)>();
            else wait_vm<0>();
            lds_poke(ready_off, lcount + (depth == kDepth ? mine + 2 - depth : mine + 1));
            if (TRACE && mine + 1 == depth) TS(2);
          }
        }
        wait_vm<0>();
        lcount += mine;
        lds_poke(ready_off, lcount);
        TS(3);
      }
  };

  // The two tail waves issue ahead of the stream waves: their copies, polls and stores lie on the path of every stage
  // end, while a stream wave that waits a few cycles for an issue slot loses nothing its ring has not covered.
  __builtin_amdgcn_s_setprio(3);
  int nseq = 0;  // input chunks of the earlier stages
  if (w == kLoader) {
    // ===================================== input loader =====================================
    for (int L = 0; L < p.n_stages; ++L) {
      const Stage& sg = p.st[L];
      const int KT = kt_of(sg);
      const int NS = __builtin_amdgcn_readfirstlane(c.ns[L]);
      const int NSo = sg.ksplit == 2 ? NS >> 1 : NS;  // tiles this workgroup finishes
      const int NCH = chunks_of(NS, KT);
      const int NBUF = nbuf_of(NS);
      TS(0);
      if (sg.sync_before && L > 0) {
        if (!grid_wait(p.flags, G, epoch * 16 + L, lane, p.spin_limit)) give_up(p.status);
        st_lds(&c.s_flag, L);
      }
      TS(1);
      load_input(L, sg, KT, NS, NCH, NBUF, nseq, 0);
      nseq += NCH;
      // ---- stage end: the LoRA wave has added the LoRA terms to the sums ---------------------------------------
      float pre[8];
      glue_prefetch(L, sg, NSo, 0, pre);
      if (sg.ksplit == 2 && NS > 0) {
        // This wave has nothing else to do until the sums carry their LoRA terms, the LoRA wave is still forming
        // those: the exchange runs here, beside them.
        spin_until([&]() { return ld_lds(&c.sum_cnt) >= (L + 1) * kSW; });
        // `red` holds this workgroup's half of the sums of tiles 2 j and 2 j + 1.  The half of the tile the partner
        // finishes goes to memory, stored through and acknowledged before the flag; the partner's half of this
        // workgroup's tile comes back the same way.  Sum = first half of the reduction + second half, on both sides.
        constexpr int kTileF4 = MT * 64;  // 16-byte pieces of a tile's sums
        const int h = wg & 1, partner = wg ^ 1;
        const int tag = epoch * 16 + L + 1;
        f32x4* const mine = reinterpret_cast<f32x4*>(p.xpart) + (size_t)wg * kTileF4;
        const f32x4* const theirs = reinterpret_cast<const f32x4*>(p.xpart) + (size_t)partner * kTileF4;
        const f32x4* const send = reinterpret_cast<const f32x4*>(red) + (1 - h) * kTileF4;
        for (int e = lane; e < kTileF4; e += 64) st_through(mine + e, send[e]);
        wait_all_mem();
        if (lane == 0) st_agent(p.xflag + wg, tag);
        spin_until([&]() { return ld_agent(p.xflag + partner) == tag; });
        f32x4* const keep = reinterpret_cast<f32x4*>(red) + h * kTileF4;
        f32x4* const out = reinterpret_cast<f32x4*>(red);
        for (int e = lane; e < kTileF4; e += 64) {
          const f32x4 got = ld_through1(theirs + e);
          const f32x4 own = keep[e];
          out[e] = h == 0 ? own + got : got + own;
        }
        wave_sync();
        TS(8);
        st_lds(&c.swap_done, L + 1);
      }
      spin_until([&]() { return ld_lds(&c.tail_go) >= L + 1; });
      TS(4);
      glue(L, sg, NSo, 0, pre);
      wait_all_mem();
      TS(5);
      st_lds(&c.tail_done, L + 1);
    }
  } else {
    // ===================================== LoRA wave =====================================
    int lvl_tag = 0;
    for (int L = 0; L < p.n_stages; ++L) {
      const Stage& sg = p.st[L];
      const int K = sg.K;
      const int NSs = __builtin_amdgcn_readfirstlane(c.ns[L]);  // tiles this workgroup streams
      const int NS = sg.ksplit == 2 ? NSs >> 1 : NSs;           // tiles it finishes
      const int NC = shrink_chunks(K);
      TS(0);
      if (sg.lora_shrink) lvl_tag = epoch * 16 + L + 1;  // a slot can serve several levels of one launch
      if (p.lora && sg.lora_shrink) {
        if (sg.sync_before && L > 0) {
          spin_until([&]() { return ld_lds(&c.s_flag) >= L; });
        }
        TS(1);
        // the rows with a LoRA term at one of this level's sites, in row order (the same list in every workgroup)
        if (lane == 0) c.s_cnt = 0;
        wave_sync();
        for (int s = 0; s < sg.n_seg; ++s)
          for (int m0 = 0; m0 < p.M; m0 += 64) {
            const int m = m0 + lane;
            const bool has = m < p.M && ((c.r_mask[m] >> sg.site[s]) & 1);
            const unsigned long long mask = __ballot(has);
            const int base = c.s_cnt;
            if (has) c.s_rows[base + __popcll(mask & ((1ull << lane) - 1ull))] = m | (s << 8);
            wave_sync();
            if (lane == 0) c.s_cnt = base + __popcll(mask);
            wave_sync();
          }
        const int items = c.s_cnt * NC;
        // spread the items of consecutive rows over the grid, and of consecutive stages over different workgroups
        for (int it = (wg + 97 * L) % G; it < items; it += G) {
          const int ms = c.s_rows[it / NC], m = ms & 0xff;
          lora_shrink_item<MT>(p, sg, m, ms >> 8, c.r_ten[m], c.r_rank[m], it % NC, NC, lvl_tag, lane);
        }
        TS(2);
      }
      if (kLoaders > 1) {
        const int KT = kt_of(sg);
        if (sg.sync_before && L > 0 && !(p.lora && sg.lora_shrink)) {
          if (!grid_wait(p.flags, G, epoch * 16 + L, lane, p.spin_limit)) give_up(p.status);
        }
        load_input(L, sg, KT, NSs, chunks_of(NSs, KT), nbuf_of(NSs), nseq, 1);
        nseq += chunks_of(NSs, KT);
      }
      // ---- rows whose LoRA term lands in this workgroup's tiles; their expand is formed ahead of the stage end ----
      int cnt = 0, npre = 0;
      if (p.lora && NS > 0) {
        if (lane == 0) c.l_cnt = 0;
        wave_sync();
        for (int m = lane; m < p.M; m += 64) {
          const int sites = c.r_mask[m];
          if (sites) {
            for (int s = 0; s < sg.n_seg; ++s) {
              if (!((sites >> sg.site[s]) & 1)) continue;
              bool mine = false;  // does the workgroup hold a tile of this site?
              for (int a = 0; a < NS; ++a) mine = mine || c.tb_seg[L][a] == s;
              if (!mine) continue;
              c.l_ms[atomicAdd(&c.l_cnt, 1)] = m | (s << 8);
            }
          }
        }
        wave_sync();
        cnt = __builtin_amdgcn_readfirstlane(c.l_cnt);
        // the shrinks of these rows have been published: lane = entry
        {
          int spins = 0;
          for (int e = lane; e < ((cnt + 63) & ~63); e += 64) {
            const int ms = c.l_ms[e < cnt ? e : 0];
            const int* f = p.tready + shrink_slot(sg, ms & 0xff, ms >> 8);
            while (!__all(e >= cnt || ld_agent(f) == lvl_tag)) {
              if (++spins >= p.spin_limit) give_up(p.status);
              __builtin_amdgcn_s_sleep(2);
            }
          }
        }
        TS(3);
        const int cap_d = kDeltaBytes / (NS * 64), cap_t = kTBytes / (p.ad.r_max * 4);  // entries `delta` and t_lds hold
        npre = cnt < cap_d ? cnt : cap_d;
        npre = npre < cap_t ? npre : cap_t;
        for (int e = lane; e < npre * p.ad.r_max; e += 64) {
          const int li = e / p.ad.r_max, cc = e - li * p.ad.r_max;
          const int ms = c.l_ms[li];
          t_lds[e] = cc < c.r_rank[ms & 0xff] ? t_sum(sg, ms & 0xff, ms >> 8, cc) : 0.f;
        }
        wave_sync();
        expand(L, sg, NS, NC, 0, npre, false);
        wave_sync();
        TS(4);
      }
      float pre[8];
      glue_prefetch(L, sg, NS, 1, pre);
      // ---- stage end: all six stream waves have summed their part of the tiles ---------------------------------
      spin_until([&]() { return ld_lds(&c.sum_cnt) >= (L + 1) * kSW; });
      TS(5);
      // (o and down: the loader wave has swapped the halves of the sums with the partner workgroup meanwhile)
      if (sg.ksplit == 2 && NSs > 0) spin_until([&]() { return ld_lds(&c.swap_done) >= L + 1; });
      for (int m = lane; m < MT * 16; m += 64) {
        float ssq = 0.f;
#pragma unroll
        for (int ww = 0; ww < kSW; ++ww) ssq += c.ss_part[ww][m];
        c.inv_rows[m] = sg.norm ? rsqrtf(ssq / (float)K + 1e-5f) : 1.f;
      }
      if (npre > 0) {
        const int work = npre * NS * 4;
        for (int e = lane; e < work; e += 64) {
          const int q = e & 3, a = (e >> 2) % NS, li = (e >> 2) / NS;
          if (c.tb_seg[L][a] != (c.l_ms[li] >> 8)) continue;
          const int m = c.l_ms[li] & 0xff;
#pragma unroll
          for (int z = 0; z < 4; ++z) red[red_idx(a, m, q * 4 + z)] += delta[((li * NS + a) * 4 + q) * 4 + z];
        }
      }
      if (cnt > npre) expand(L, sg, NS, NC, npre, cnt, true);
      wave_sync();
      st_lds(&c.tail_go, L + 1);
      glue(L, sg, NS, 1, pre);
      wait_all_mem();
      TS(6);
      spin_until([&]() { return ld_lds(&c.tail_done) >= L + 1; });
      // `red` may be overwritten; the outputs of both waves are in memory: hand over to the stages that read them
      st_lds(&c.red_free, L + 1);
      if (lane == 0) st_agent(p.flags + wg, epoch * 16 + (L + 1 < p.n_stages ? L + 1 : 15));
      TS(7);
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

// =====================================================================================================================
// Wide batches (33..128 rows).  With this many rows the stage input is as large as a workgroup's share of the weights,
// and a workgroup that owns a few 16-column tiles over the whole reduction reads all of it: the input copies, not the
// weights, set the time.  Here a level (q,k,v | o | gate,up | down) is cut the other way: a group is kSW * TPW tiles
// wide (each stream wave holds TPW tiles of it, over all rows), the (group, k block) space of a level is laid out in a
// line and dealt to the workgroups in equal contiguous pieces, so a workgroup reads only its piece of the reduction
// of the input.  A piece that ends inside a group leaves a segment: its fp32 partial tiles go to memory, and when all
// segments of a group are there, the group's tiles are summed in segment order, get their LoRA term and the level's
// glue, and are stored - each (tile, row tile) by one wave of the workgroup it is dealt to.
// =====================================================================================================================
// ---- shrink items of the wide kernel, in two steps -------------------------------------------------------------
// W^A does not depend on the activations: the rows of a chunk (up to 32 wave loads, the whole chunk for ranks up to 32)
// can be asked for before the level's barrier has opened, and sit in registers when it does.  What is left behind the
// barrier is one round trip for the 512 inputs of the row (one 16-byte load per lane, handed round through 1 KiB of
// LDS), the sums, and the store of the partial with its flag.  For ranks that are a power of two times 8, up to 64,
// and 16-byte aligned W^A; everything else takes lora_shrink_item.
struct ShrinkJob {
  const gbf16* A;
  int m, pos, r, kc, k_lo, k_hi, slot;
  bool fast;
};

template <int MT>
__device__ __forceinline__ ShrinkJob shrink_job(const Params& p, const Stage& sg, int ms, int tenant, int r, int kc) {
  ShrinkJob j;
  j.m = ms & 0xff;
  j.pos = ms >> 8;
  j.r = r;
  j.kc = kc;
  j.k_lo = kc * kShrinkChunk;
  j.k_hi = j.k_lo + kShrinkChunk < sg.K ? j.k_lo + kShrinkChunk : sg.K;
  j.slot = shrink_slot(sg, j.m, j.pos);
  j.A = (const gbf16*)p.ad.A[tenant * MILORA_NUM_SITES + sg.site[j.pos]];
  const int lpr = r >> 3;
  j.fast = (r & 7) == 0 && (lpr & (lpr - 1)) == 0 && lpr <= 8 && ((uintptr_t)j.A & 15) == 0;
  return j;
}

// wave loads h * 32 .. h * 32 + 31 of the chunk's rows of W^A (a chunk is 8 * (r / 8) = r loads of 64 / (r / 8) rows)
__device__ __forceinline__ void shrink_load_A(const ShrinkJob& j, int h, int lane, u32x4 (&a)[32]) {
  const int lpr = j.r >> 3, kpl = 64 / lpr, cg = lane & (lpr - 1), kr = lane / lpr;
  const gu32x4* Ap = reinterpret_cast<const gu32x4*>(j.A) + cg;
#pragma unroll
  for (int u = 0; u < 32; ++u) {
    int k = j.k_lo + kr + (h * 32 + u) * kpl;
    k = k < j.k_hi ? k : j.k_hi - 1;  // past the end of a ragged chunk: a valid row, its input is zero
    a[u] = __builtin_nontemporal_load(Ap + (size_t)k * lpr);  // (loads past the chunk's r repeat its last row; not used)
  }
}

template <int MT>
__device__ __forceinline__ void shrink_finish(const Params& p, const Stage& sg, const ShrinkJob& j, int tag, int lane,
                                              u32x4 (&a)[32], bf16_t* xs) {
  const int lpr = j.r >> 3, kpl = 64 / lpr, kr = lane / lpr;
  // the row's inputs of this chunk: lane l takes k_lo + 8 l .. + 7, and the chunk goes through LDS in k order
  {
    const int k = j.k_lo + 8 * lane;
    u32x4 xv = {0u, 0u, 0u, 0u};
    if (k < j.k_hi) {  // (k_hi is a multiple of 32)
      const bf16_t* src = sg.x_packed ? sg.X + packed_x_offset(j.m, k, MT) : sg.X + (size_t)j.m * sg.ldx + k;
      xv = *(const gu32x4*)src;
    }
    *reinterpret_cast<u32x4*>(xs + 8 * lane) = xv;
  }
  compiler_fence();
  wait_lds();
  compiler_fence();
  float acc[8];
#pragma unroll
  for (int v = 0; v < 8; ++v) acc[v] = 0.f;
  for (int h = 0; h * 32 < j.r; ++h) {
    if (h > 0) shrink_load_A(j, h, lane, a);
#pragma unroll
    for (int u = 0; u < 32; ++u) {
      if (h * 32 + u < j.r) {
        const float x = bf16_to_f32(xs[kr + (h * 32 + u) * kpl]);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          acc[2 * v] += x * __uint_as_float(a[u][v] << 16);
          acc[2 * v + 1] += x * __uint_as_float(a[u][v] & 0xffff0000u);
        }
      }
    }
  }
  // lanes with equal column group hold partial sums over different rows: fixed butterfly over the row bits
  for (int off = lpr; off < 64; off <<= 1)
#pragma unroll
    for (int v = 0; v < 8; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
  float* out = p.tpart + ((size_t)j.slot * p.nc_max + j.kc) * p.ad.r_max;
  if (lane < lpr)
#pragma unroll
    for (int v = 0; v < 8; ++v) st_agent(out + lane * 8 + v, acc[v]);
  wait_all_mem();
  st_agent(p.tpflag + j.slot * kTpStride + j.kc, tag);  // (by every lane: see shrink_items)
}

template <int MT> struct WCfg;
// (Two k steps of weight loads in flight per wave: deeper rings - three, four, six, eight steps were timed - only
// lengthen every other round trip of the launch - flags, partial tiles, LoRA items - which queue behind them in the
// memory system.  Chunks of two k blocks halve the stream waves' look-ups of the loader's word.
// Two tiles per wave at 64 rows as at 128, not four: groups of 12 tiles instead of 24 cut the reduction of a level into
// half as many pieces, so half as many partial tiles go through memory, and the input copies - twice as many k blocks
// per workgroup, 4 KiB each - are still small beside the weights: 163 -> 145 us per layer step of the 7B shape.
// One tile per wave: 2 us less at 64 rows with four k steps in flight, 10-15 us more at 128 rows; not used.)
template <> struct WCfg<4> { static constexpr int TPW = 2, D = 2, CKB = 2; };
template <> struct WCfg<8> { static constexpr int TPW = 2, D = 2, CKB = 2; };
constexpr int kWideGridMax = 256;   // workgroups the segment tables are sized for

__device__ __forceinline__ void st_through(u32x2* p, u32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
// Eight 16-byte loads that bypass the caches (the partial tiles are written by other workgroups in this launch, into
// memory that earlier levels and launches have used), complete when the function returns.
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

// The same with two more (the LoRA term tiles of a unit travel with its first eight partial tiles).
__device__ __forceinline__ void ld_through10(const f32x4* const (&q)[10], f32x4 (&v)[10]) {
  asm volatile(
      "global_load_dwordx4 %0, %10, off sc0 sc1\n\t"
      "global_load_dwordx4 %1, %11, off sc0 sc1\n\t"
      "global_load_dwordx4 %2, %12, off sc0 sc1\n\t"
      "global_load_dwordx4 %3, %13, off sc0 sc1\n\t"
      "global_load_dwordx4 %4, %14, off sc0 sc1\n\t"
      "global_load_dwordx4 %5, %15, off sc0 sc1\n\t"
      "global_load_dwordx4 %6, %16, off sc0 sc1\n\t"
      "global_load_dwordx4 %7, %17, off sc0 sc1\n\t"
      "global_load_dwordx4 %8, %18, off sc0 sc1\n\t"
      "global_load_dwordx4 %9, %19, off sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]), "=&v"(v[8]),
        "=&v"(v[9])
      : "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]), "v"(q[4]), "v"(q[5]), "v"(q[6]), "v"(q[7]), "v"(q[8]), "v"(q[9])
      : "memory");
}

// units (tiles, or gate/up tile pairs) and groups of a level
// Weight ring of the wide kernel: a load the compiler does not count, and the wait that makes a ring row usable
// (at most N loads still out; the row's registers pass through the statement so that nothing that reads them moves
// above it).
__device__ __forceinline__ void ring_load(u32x4& dst, const gu32x4* src) {
  asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(dst) : "v"(src) : "memory");
}
template <int N>
__device__ __forceinline__ void ring_wait_n(u32x4& a) {
  static_assert(N >= 0 && N < 64, "memory counter");
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void ring_wait_n(u32x4& a, u32x4& b) {
  static_assert(N >= 0 && N < 64, "memory counter");
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void ring_wait_n(u32x4& a, u32x4& b, u32x4& c2, u32x4& d) {
  static_assert(N >= 0 && N < 64, "memory counter");
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c2), "+v"(d) : "n"(N) : "memory");
}

__device__ __host__ __forceinline__ int wide_units(const Stage& s) {
  if (s.pair) return s.N[0] >> 4;
  int t = 0;
  for (int i = 0; i < s.n_seg; ++i) t += s.N[i] >> 4;
  return t;
}
__device__ __host__ __forceinline__ int wide_groups(const Stage& s, int NT) {
  const int upg = s.pair ? NT / 2 : NT;
  return (wide_units(s) + upg - 1) / upg;
}

template <int MT, bool TRACE>
__global__ void __launch_bounds__(kThreads) decode_wide_kernel(const Params p) {
  constexpr int TPW = WCfg<MT>::TPW, D = WCfg<MT>::D, CKB = WCfg<MT>::CKB, NT = kSW * TPW;
  constexpr int kChunk = CKB * MT * 1024;                         // bytes of an input chunk: CKB k blocks, all rows
  constexpr int NBUF = (kLdsBytes - kCtrlBytes) / kChunk;         // chunk buffers
  constexpr int LPC = CKB * MT;                                   // wave loads per chunk
  constexpr int kDepth = 16384 / kChunk > 1 ? 16384 / kChunk : 1;  // chunks the loader keeps in flight: 16 KB (64 KB cost 2.5 us per layer step)
  static_assert(D % CKB == 0 && LPC * kDepth <= 63 && NBUF >= 4 && kDepth < NBUF, "chunks");
  extern __shared__ __align__(16) unsigned char smem[];
  Ctrl& c = *reinterpret_cast<Ctrl*>(smem);
  unsigned char* const xreg = smem + kCtrlBytes;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x, G = gridDim.x;

  if (tid == 0) {
    c.x_ready[0] = 0;
    c.shr_ready = 0;
    c.bar_seen = 0;
    c.epoch = (ld_agent(p.flags + wg) >> 4) + 1;
  }
  if (tid < 8) {
    c.x_done[tid] = 0;
    c.seg_arr[tid] = 0;
  }
  if (tid < kMaxStages) { c.shr_next[tid] = 0; c.lvl_arr[tid] = 0; c.exp_next[tid] = 0; }
  if (tid >= 64 && tid < 64 + kMaxRows) {
    const int m = tid - 64;
    int mask = 0, tenant = 0, r = 0;
    if (m < p.M && p.lora) {
      const int req = p.row_to_req ? p.row_to_req[m] : m;
      if (req >= 0 && req < p.Breq) {
        const uint8_t rb = p.route[req];
        for (int st = 0; st < MILORA_NUM_SITES; ++st)
          if (route_has(rb, st)) {
            r = routed_rank(p.ad, p.tenant_id, p.route, req, p.Breq, st, &tenant);  // the same for every chosen site
            if (r > 0) mask |= 1 << st;
          }
      }
    }
    c.r_mask[m] = mask;
    c.r_ten[m] = tenant;
    c.r_rank[m] = r;
  }
  __syncthreads();
  const int epoch = __builtin_amdgcn_readfirstlane(c.epoch);

  // A wait that runs out is recorded in the status word and leaves the wave `dead`: it waits for nothing any more,
  // draws no LoRA items and builds no lists (their inputs may not be there), and otherwise runs through its levels on
  // whatever the buffers hold - every address it forms comes from the launch parameters, not from what it waited for.
  // (No wave ends early here: an s_endpgm inside the item loops below made the compiler re-run an item for ever.)
  // cond() is the same in every lane (an __all, or a word every lane reads): the loop is kept scalar.
  bool dead = false;
  // (The status word is stored from assembly: a store the compiler sees inside the weight loop makes it wait for
  // every outstanding load at each use of the weight ring - loads and stores share the memory counter and may
  // complete out of order, so with a store possibly pending it waits for the count to reach zero.)
  auto spin_until = [&](auto cond) __attribute__((always_inline)) {
    int spins = 0;
    while (!dead && !__builtin_amdgcn_readfirstlane((int)cond())) {
      if (++spins >= p.spin_limit) {
        if (lane == 0) asm volatile("global_store_dword %0, %1, off sc1" : : "v"(p.status), "v"(1) : "memory");
        dead = true;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    compiler_fence();
  };
  auto barrier_wait = [&](int target) __attribute__((always_inline)) {
    if (!dead && !grid_wait(p.flags, G, target, lane, p.spin_limit)) {
      if (lane == 0) st_agent(p.status, 1);
      dead = true;
    }
  };
  auto wave_sync = [&]() __attribute__((always_inline)) {
    compiler_fence();
    wait_lds();
    compiler_fence();
  };

  // 1 KiB per tail wave for the inputs of a shrink item (the few-row kernel's sums of squares lie there; unused here)
  static_assert(sizeof(c.ss_part) >= 2 * kShrinkChunk * sizeof(bf16_t), "input staging of the shrink items");
  bf16_t* const xstage = reinterpret_cast<bf16_t*>(&c.ss_part[0][0]) + (w == kLora ? kShrinkChunk : 0);
  // The level's shrink items (row with a LoRA term at a site of the level, k chunk) are spread over the grid; those
  // of this workgroup are drawn one by one by its LoRA wave and, once its copies are out, its loader wave.
  auto shrink_items = [&](const int L, const Stage& sg) __attribute__((always_inline)) {
    const int NC = shrink_chunks(sg.K);
    const int items = __builtin_amdgcn_readfirstlane(ld_lds(&c.s_cnt)) * NC;
    for (;;) {
      // (The barrier keeps the compiler from fusing the one-lane store that ends an item with the one-lane ticket
      // draw of the next: fused, lanes 1..63 went round the loop on their own, with ticket 0, for ever.)
      __builtin_amdgcn_wave_barrier();
      int k = 0;
      if (lane == 0) k = __hip_atomic_fetch_add(&c.shr_next[L], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      k = __builtin_amdgcn_readfirstlane(k);
      const int it = (wg + 97 * L) % G + k * G;
      if (it >= items) break;
      const int ms = __builtin_amdgcn_readfirstlane(c.s_rows[it / NC]), m = ms & 0xff;
      const ShrinkJob job = shrink_job<MT>(p, sg, ms, __builtin_amdgcn_readfirstlane(c.r_ten[m]),
                                           __builtin_amdgcn_readfirstlane(c.r_rank[m]), it % NC);
      if (job.fast) {
        u32x4 a[32];
        shrink_load_A(job, 0, lane, a);
        shrink_finish<MT>(p, sg, job, epoch * 16 + L + 1, lane, a, xstage);
      } else {
        lora_shrink_item<MT, true, 16>(p, sg, m, ms >> 8, c.r_ten[m], c.r_rank[m], it % NC, NC, epoch * 16 + L + 1, lane);
      }
    }
  };
  // The level's expand items: the LoRA term t W^B of one routed row at one site for a slab of 256 columns (four per
  // lane), stored as fp32 tiles in the layout of the partial tiles, so that the sums below take it in like one more
  // segment.  An item waits for the row's shrink partials (one flag per k chunk), adds them in chunk order, takes
  // 32 ranks of W^B per round trip, stores, and publishes one word per (slab, row).  Drawn like the shrink items.
  auto expand_items = [&](const int L, const Stage& sg) __attribute__((always_inline)) {
    const int NC = shrink_chunks(sg.K);
    const int N = sg.N[0];  // the sites of a level are equally wide
    const int slabs = (N + 255) >> 8;
    // (what is read from LDS below is the same in every lane; it is made scalar, so that the loops and waits of an
    // item are plain scalar control flow)
    const int items = __builtin_amdgcn_readfirstlane(ld_lds(&c.s_cnt)) * slabs;
    const int lvl_tag = epoch * 16 + L + 1;
    f32x4* const dtab = reinterpret_cast<f32x4*>(p.delta) + (size_t)((L & 1) ? p.delta_odd : 0) * (MT * 64);
    int* const drd = p.dready + (size_t)(L & 1) * 3 * p.slabs_max * kMaxRows;
    const int rmax = p.ad.r_max;
    for (;;) {
      __builtin_amdgcn_wave_barrier();  // (as in shrink_items)
      int k = 0;
      if (lane == 0) k = __hip_atomic_fetch_add(&c.exp_next[L], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      k = __builtin_amdgcn_readfirstlane(k);
      const int it = (wg + 131 * L) % G + k * G;
      if (it >= items) break;
      const int e = it / slabs, j = it - e * slabs;
      const int ms = __builtin_amdgcn_readfirstlane(c.s_rows[e]), m = ms & 0xff, sp = ms >> 8;
      const int r = __builtin_amdgcn_readfirstlane(c.r_rank[m]), slot = shrink_slot(sg, m, sp);
      const int tenant = __builtin_amdgcn_readfirstlane(c.r_ten[m]);
      const int n = j * 256 + 4 * lane;
      const bool inb = n < N;
      const size_t ldb = (size_t)N;
      const gbf16* const Bbase = (const gbf16*)p.ad.B[tenant * MILORA_NUM_SITES + sg.site[sp]];
      const gbf16* const Bm = Bbase + (inb ? n : 0);
      const float* tp = p.tpart + (size_t)slot * p.nc_max * rmax;
      const bool vec = ((uintptr_t)Bbase & 7) == 0;  // (N is a multiple of 16: every row and every lane's quad is 8-byte aligned with it)
      // rows c0 .. c0 + 31 of W^B, this lane's four columns
      auto load_B = [&](int c0, u32x2 (&bb)[32]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 32; ++u) bb[u] = *reinterpret_cast<const gu32x2*>(Bm + (size_t)(c0 + u < r ? c0 + u : r - 1) * ldb);
      };
      u32x2 bb[32];
      if (vec) load_B(0, bb);  // W^B does not wait for the shrink: asked for before the flags are polled
      {  // the row's shrink partials are there: one flag per k chunk
        const int* f = p.tpflag + slot * kTpStride + (lane < NC ? lane : 0);
        spin_until([&]() { return __all(lane >= NC || ld_agent(f) == lvl_tag); });
      }
      float d[4] = {0.f, 0.f, 0.f, 0.f};
      for (int c0 = 0; c0 < r; c0 += 64) {
        // lane u sums rank c0 + u over the k chunks, in chunk order, 16 loads in flight per pass
        const int cu = c0 + lane;
        float tl = 0.f;
        for (int k0 = 0; k0 < NC; k0 += 16) {
          float v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u)
            v[u] = ld_agent(tp + (size_t)(k0 + u < NC ? k0 + u : NC - 1) * rmax + (cu < r ? cu : 0));
#pragma unroll
          for (int u = 0; u < 16; ++u) tl += k0 + u < NC ? v[u] : 0.f;
        }
        if (vec) {
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            if (c0 + 32 * h >= r) break;
            if (c0 + h > 0) load_B(c0 + 32 * h, bb);
#pragma unroll
            for (int u = 0; u < 32; ++u) {
              const float t = c0 + 32 * h + u < r ? __shfl(tl, 32 * h + u, 64) : 0.f;
              d[0] += t * __uint_as_float(bb[u][0] << 16);
              d[1] += t * __uint_as_float(bb[u][0] & 0xffff0000u);
              d[2] += t * __uint_as_float(bb[u][1] << 16);
              d[3] += t * __uint_as_float(bb[u][1] & 0xffff0000u);
            }
          }
        } else {
          for (int u = 0; u < 64 && c0 + u < r; ++u) {
            const float t = __shfl(tl, u, 64);
#pragma unroll
            for (int z = 0; z < 4; ++z) d[z] += t * bf16_to_f32(Bm[(size_t)(c0 + u) * ldb + z]);
          }
        }
      }
      if (inb) st_through(dtab + ((size_t)(sp * (N >> 4) + (n >> 4)) * MT + (m >> 4)) * 64 + (m & 15) + 16 * ((n >> 2) & 3),
                          f32x4{d[0], d[1], d[2], d[3]});
      wait_all_mem();
      st_agent(drd + (sp * p.slabs_max + j) * kMaxRows + m, lvl_tag);  // (by every lane, as the shrink flags)
    }
  };

  if (w >= kSW) __builtin_amdgcn_s_setprio(3);  // the loader and LoRA waves issue ahead of the stream waves
  int xs = 0;      // input chunks of the segments so far (the same count in every wave)
  int segord = 0;  // segments so far
  int seen = 0;    // stream waves: chunks known to have landed

  for (int L = 0; L < p.n_stages; ++L) {
    const Stage& sg = p.st[L];
    const int KT = sg.K >> 5;
    const int T = wide_units(sg), upg = sg.pair ? NT / 2 : NT, groups = (T + upg - 1) / upg;
    const long Wt = (long)groups * KT;
    const int act = Wt < (long)G ? (int)Wt : G;  // workgroups that get a piece of the level
    const int tag = epoch * 16 + L;
    TS(0);
    // Segment tables of even and odd levels lie apart: a level that follows another without a barrier (o after q,k,v
    // when the caller supplies the attention output) must not touch what that one's sums still read.
    const int sbase = (L & 1) * p.wsegs;
    // the workgroup that owns position x of the line: the last one whose piece starts at or before x
    auto owner = [&](long x) __attribute__((always_inline)) -> int { return (int)(((x + 1) * act - 1) / Wt); };
    long lo = 0, hi = 0;
    if (wg < act) {
      lo = (long)wg * Wt / act;
      hi = (long)(wg + 1) * Wt / act;
    }
    // the tiles this workgroup sums and stores: consecutive ones (they lie in one group, two at most)
    const int tpg = (T + G - 1) / G;
    const int t0 = wg * tpg < T ? wg * tpg : T, t1 = t0 + tpg < T ? t0 + tpg : T;
    const int lvl_tag = epoch * 16 + L + 1;
    // unit (tile, or gate/up pair) -> site position and tile inside the site's matrix
    auto unit_tile = [&](int ti, int& sp) __attribute__((always_inline)) -> int {
      sp = 0;
      if (sg.pair) return ti;
      int u = ti;
      while (sp + 1 < sg.n_seg && u >= (sg.N[sp] >> 4)) {
        u -= sg.N[sp] >> 4;
        ++sp;
      }
      return u;
    };
    if (w < kSW) {
      // ===================================== stream waves =====================================
      const int rd_off = sg.x_packed ? lane * 16 : ((lane & 15) * 4 + (lane >> 4)) * 16;
      const bool norm = sg.norm != 0;
      for (long pos = lo; pos < hi;) {
        const int g = (int)(pos / KT), kb0 = (int)(pos - (long)g * KT);
        const long gend = (long)(g + 1) * KT;
        const int len = (int)((hi < gend ? hi : gend) - pos);
        const int sid = sbase + wg + g;
        const int nch = (len + CKB - 1) / CKB;
        // this wave's tiles of the group
        const gu32x4* wp[TPW];
        bool tval[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
          int seg = 0, tile;
          if (sg.pair) {
            tile = g * upg + ((w * TPW + j) >> 1);  // slot w TPW + j of the group: gate and up tiles alternate
            seg = (w * TPW + j) & 1;
            tval[j] = tile < T;
          } else {
            int u = g * NT + w * TPW + j;
            tval[j] = u < T;
            if (!tval[j]) u = 0;
            while (seg + 1 < sg.n_seg && u >= (sg.N[seg] >> 4)) {
              u -= sg.N[seg] >> 4;
              ++seg;
            }
            tile = u;
          }
          if (!tval[j]) { seg = 0; tile = 0; }  // streams valid memory, result dropped
          wp[j] = (const gu32x4*)sg.W[seg] + ((size_t)tile * KT + kb0) * 64 + lane;
        }
        u32x4 ring[D][TPW];
        auto ring_wait = [&](u32x4 (&row)[TPW]) __attribute__((always_inline)) {
          if constexpr (TPW == 1) ring_wait_n<(D - 1) * TPW>(row[0]);
          else if constexpr (TPW == 2) ring_wait_n<(D - 1) * TPW>(row[0], row[1]);
          else ring_wait_n<(D - 1) * TPW>(row[0], row[1], row[2], row[3]);
        };
        auto ring_drain = [&](u32x4 (&row)[TPW]) __attribute__((always_inline)) {
          if constexpr (TPW == 1) ring_wait_n<0>(row[0]);
          else if constexpr (TPW == 2) ring_wait_n<0>(row[0], row[1]);
          else ring_wait_n<0>(row[0], row[1], row[2], row[3]);
        };
        static_assert(TPW == 1 || TPW == 2 || TPW == 4, "ring_wait is written for one, two or four tiles per wave");
        f32x4 acc[TPW][MT];
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[j][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        float ss[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ss[mt] = 0.f;
#pragma unroll
        for (int s = 0; s < D; ++s)
#pragma unroll
          for (int j = 0; j < TPW; ++j) ring_load(ring[s][j], wp[j] + (size_t)(s < len ? s : len - 1) * 64);
        for (int i0 = 0; i0 < len; i0 += D) {
#pragma unroll
          for (int s = 0; s < D; ++s) {
            const int i = i0 + s;
            const bool valid = i < len;
            if (s % CKB == 0) {
              // next chunk: the ones before it are consumed; it has landed
              const int chn = i / CKB;
              compiler_fence();
              st_lds(&c.x_done[w], xs + (chn < nch ? chn : nch));
              if (valid && seen <= xs + chn) spin_until([&]() { return (seen = ld_lds(&c.x_ready[0])) > xs + chn; });
              if (TRACE && pos == lo && i == 0) TS(1);
            }
            const uint32_t mask = valid ? 0xffffffffu : 0u;
            const int chn = valid ? i / CKB : nch - 1;
            const unsigned char* xbuf = xreg + ((xs + chn) % NBUF) * kChunk + (s % CKB) * (MT * 1024) + rd_off;
            u32x4 xb[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xb[mt] = *reinterpret_cast<const u32x4*>(xbuf + mt * 1024) & mask;
            if (norm && w == 0) {
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) ss[mt] += sumsq8(xb[mt]);
            }
            // The weight blocks of this slot have landed once all but the (D - 1) TPW loads issued after them have.
            // Loads and wait are written as assembly: with loads it can see the compiler drains every outstanding
            // load once per pass of the ring, which leaves the ring empty at every pass.
            ring_wait(ring[s]);
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
              const u32x4 wv = ring[s][j] & mask;
#pragma unroll
              for (int mt = 0; mt < MT; ++mt)
                acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv), __builtin_bit_cast(bf16x8, xb[mt]),
                                                                    acc[j][mt], 0, 0, 0);
            }
            const int nx = i + D < len ? i + D : len - 1;
#pragma unroll
            for (int j = 0; j < TPW; ++j) ring_load(ring[s][j], wp[j] + (size_t)nx * 64);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        compiler_fence();
        st_lds(&c.x_done[w], xs + nch);
        // the segment's partial tiles, as the matrix cores leave them: lane = (row lane % 16, columns 4 (lane / 16) ..)
        f32x4* const P = reinterpret_cast<f32x4*>(p.wpart) + ((size_t)sid * NT + w * TPW) * (MT * 64) + lane;
#pragma unroll
        for (int j = 0; j < TPW; ++j)
          if (tval[j])
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) st_through(P + (j * MT + mt) * 64, acc[j][mt]);
        if (norm && w == 0) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            float v = ss[mt];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (lane < 16) st_agent(p.wss + (size_t)sid * (MT * 16) + mt * 16 + lane, v);
          }
        }
        // the ring's last, clamped loads still write their registers: those stay reserved until they have
#pragma unroll
        for (int s = 0; s < D; ++s) ring_drain(ring[s]);
        wait_all_mem();
        // the last of the six waves announces the segment
        int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(&c.seg_arr[segord & 7], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old + 1 == kSW * ((segord >> 3) + 1) && lane == 0) st_agent(p.segflag + sid, tag);
        xs += nch;
        ++segord;
        pos += len;
      }
      TS(2);
    } else if (w == kLoader) {
      // ===================================== input loader =====================================
      if (sg.sync_before && L > 0) {
        barrier_wait(epoch * 16 + L);
        st_lds(&c.bar_seen, L);  // the LoRA wave waits for this word instead of polling the flags too
      }
      TS(1);
      const unsigned char* const Xb = reinterpret_cast<const unsigned char*>(sg.X);
      const bool xpk = sg.x_packed != 0;
      size_t loff[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        int row = mt * 16 + (lane >> 2);
        if (row > p.M - 1) row = p.M - 1;
        loff[mt] = xpk ? (size_t)mt * 1024 + lane * 16 : ((size_t)row * sg.ldx + (lane & 3) * 8) * sizeof(bf16_t);
      }
      const size_t kstep = xpk ? (size_t)MT * 1024 : 64;
      const uint32_t done_off = lds_off(&c.x_done[lane < kSW ? lane : 0]), ready_off = lds_off(&c.x_ready[0]);
      int issued = 0;  // chunks of this level
      for (long pos = lo; pos < hi;) {
        const int g = (int)(pos / KT), kb0 = (int)(pos - (long)g * KT);
        const long gend = (long)(g + 1) * KT;
        const int len = (int)((hi < gend ? hi : gend) - pos);
        const int nch = (len + CKB - 1) / CKB;
        for (int ch = 0; ch < nch; ++ch) {
          const int n = xs + issued;  // this chunk's number; it reuses the buffer of chunk n - NBUF
          spin_until([&]() { return __all(lds_peek(done_off) >= n - NBUF + 1); });
          unsigned char* const dst = xreg + (n % NBUF) * kChunk;
#pragma unroll
          for (int kk = 0; kk < CKB; ++kk) {
            int kb = ch * CKB + kk;
            kb = kb0 + (kb < len ? kb : len - 1);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xb + (size_t)kb * kstep + loff[mt]),
                                               (__attribute__((address_space(3))) void*)(dst + ((kk * MT + mt) << 10)), 16, 0, 0);
          }
          ++issued;
          if (issued >= kDepth) {
            wait_vm<LPC * (kDepth - 1)>();
            lds_poke(ready_off, xs + issued - kDepth + 1);
          }
        }
        pos += len;
      }
      wait_vm<0>();
      lds_poke(ready_off, xs + issued);
      xs += issued;
      TS(2);
      if (p.lora) spin_until([&]() { return ld_lds(&c.shr_ready) >= L + 1; });  // the copies are out: help with the LoRA items
    } else {
      // ===================================== LoRA wave: the level's shrinks =====================================
      if (p.lora) {
        // the level's rows with a LoRA term, in row order (the same list in every workgroup): it follows from the
        // route table alone and is built before the barrier; the loader wave may still be drawing the previous
        // level's items from the list
        if (L > 0) spin_until([&]() { return ld_lds(&c.lvl_arr[L - 1]) >= kWaves; });
        if (lane == 0 && !dead) c.s_cnt = 0;
        wave_sync();
        for (int s = 0; s < sg.n_seg && !dead; ++s)
          for (int m0 = 0; m0 < p.M; m0 += 64) {
            const int m = m0 + lane;
            const bool has = m < p.M && ((c.r_mask[m < p.M ? m : 0] >> sg.site[s]) & 1);
            const unsigned long long mask = __ballot(has);
            const int base = c.s_cnt;
            if (has) c.s_rows[base + __popcll(mask & ((1ull << lane) - 1ull))] = m | (s << 8);
            wave_sync();
            if (lane == 0) c.s_cnt = base + __popcll(mask);
            wave_sync();
          }
        if (lane == 0 && !dead) st_lds(&c.shr_ready, L + 1);
        TS(2);
        // the wave's first shrink item: its rows of W^A are asked for now and travel while the barrier is closed
        const int NC = shrink_chunks(sg.K);
        const int items = dead ? 0 : __builtin_amdgcn_readfirstlane(ld_lds(&c.s_cnt)) * NC;
        int k = 0;
        if (lane == 0) k = __hip_atomic_fetch_add(&c.shr_next[L], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        k = __builtin_amdgcn_readfirstlane(k);
        const int it = (wg + 97 * L) % G + k * G;
        const bool have = it < items;
        ShrinkJob job;
        job.fast = false;
        uint32_t pf[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};  // one word of every 128-byte line of the chunk of W^A
        int ms = 0;
        if (have) {
          ms = __builtin_amdgcn_readfirstlane(c.s_rows[it / NC]);
          const int m = ms & 0xff;
          job = shrink_job<MT>(p, sg, ms, __builtin_amdgcn_readfirstlane(c.r_ten[m]), __builtin_amdgcn_readfirstlane(c.r_rank[m]),
                               it % NC);
          if (job.fast) {
            const unsigned char* base = (const unsigned char*)(uintptr_t)job.A + (size_t)job.k_lo * job.r * 2;
            const int bytes = (job.k_hi - job.k_lo) * job.r * 2;
            int lane_here = lane;  // (opaque: otherwise the eight offsets are kept, and spilled, for the whole kernel)
            asm volatile("" : "+v"(lane_here));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const int off = (i * 64 + lane_here) * 128;
              if (off < bytes) pf[i] = __builtin_nontemporal_load((const __attribute__((address_space(1))) uint32_t*)(base + off));
            }
          }
        }
        if (sg.sync_before && L > 0) spin_until([&]() { return ld_lds(&c.bar_seen) >= L; });
        asm volatile("" : : "v"(pf[0]), "v"(pf[1]), "v"(pf[2]), "v"(pf[3]), "v"(pf[4]), "v"(pf[5]), "v"(pf[6]), "v"(pf[7]));
        TS(1);
        if (have && !dead) {
          TS(8);
          if (job.fast) {
            u32x4 a[32];
            shrink_load_A(job, 0, lane, a);
            shrink_finish<MT>(p, sg, job, epoch * 16 + L + 1, lane, a, xstage);
          } else lora_shrink_item<MT, true, 16>(p, sg, ms & 0xff, ms >> 8, c.r_ten[ms & 0xff], c.r_rank[ms & 0xff], it % NC, NC,
                                              epoch * 16 + L + 1, lane);
          TS(9);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
    if (p.lora && !dead) {
      // loader and LoRA wave: the level's shrinks, then the expands.  The stream waves, their segments stored, help
      // with the expands: with many routed rows and large ranks (the sums wait for the last expand item) two waves
      // per workgroup are few.
      if (w >= kSW) {
        shrink_items(L, sg);
        TS(6);
      } else {
        spin_until([&]() { return ld_lds(&c.shr_ready) >= L + 1; });
      }
      expand_items(L, sg);
      TS(3);
    }
    // ===================================== all waves: sum, LoRA term, glue, store =====================================
    {
      // A wave's units lie in one group (two at most): a flag that has been seen stays, so the segment flags of a
      // group are polled once per wave.
      int g_seen = -1;
      int uc = 0;
      const f32x4* const dtab = reinterpret_cast<const f32x4*>(p.delta) + (size_t)((L & 1) ? p.delta_odd : 0) * (MT * 64);
      const int* const drd = p.dready + (size_t)(L & 1) * 3 * p.slabs_max * kMaxRows;
      TS(4);
      for (int ti = t0; ti < t1; ++ti)
        for (int mt = 0; mt < MT; ++mt, ++uc) {
          if ((uc & 7) != w) continue;
          int s;
          const int tile = unit_tile(ti, s);
          int g, a0;
          if (sg.pair) {
            g = ti / upg;
            const int pi = ti - g * upg;
            a0 = 2 * pi;
          } else {
            g = ti / NT;
            a0 = ti - g * NT;
          }
          const long x0 = (long)g * KT;
          const int wf = owner(x0), wl = owner(x0 + KT - 1), n = wl - wf + 1, sid0 = sbase + wf + g;
          const int m = mt * 16 + (lane & 15), q = lane >> 4;
          const int ncol = tile * 16 + q * 4;
          // The LoRA terms of the unit's rows (stored by the expand items as tiles of this layout) and the group's
          // segments are there: one poll loop over both kinds of flags.
          const int mm = m < p.M ? m : 0;
          const bool has_a = p.lora && m < p.M && ((c.r_mask[mm] >> sg.site[s]) & 1);
          const bool has_b = sg.pair && p.lora && m < p.M && ((c.r_mask[mm] >> sg.site[1]) & 1);
          const int* const fa = drd + (s * p.slabs_max + (tile >> 4)) * kMaxRows + mm;
          const int* const fb = drd + (1 * p.slabs_max + (tile >> 4)) * kMaxRows + mm;
          {
            const int* const fs = p.segflag + sid0 + (lane < n ? lane : 0);
            const bool poll_seg = g != g_seen;
            spin_until([&]() {  // (the three words asked for together: one round trip per poll)
              const int va = ld_agent(fa), vb = ld_agent(fb), vs = ld_agent(fs);
              const bool ok = (!has_a || va == lvl_tag) & (!has_b || vb == lvl_tag) & (!poll_seg || lane >= n || vs == tag);
              return __all(ok);
            });
            for (int b = 64; poll_seg && b < n; b += 64) {  // (more than 64 segments per group: tiny levels on a large grid)
              const int i = b + lane;
              const int* f = p.segflag + sid0 + (i < n ? i : 0);
              spin_until([&]() { return __all(i >= n || ld_agent(f) == tag); });
            }
            g_seen = g;
          }
          f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
          float ssq = 0.f;
          if (sg.norm) {  // lane = (row, segment % 4): the sums of squares of 16 segments per round trip, added in order
            for (int b = 0; b < n; b += 16) {
              float v[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int i = b + 4 * u + q;
                v[u] = ld_agent(p.wss + (size_t)(sid0 + (i < n ? i : 0)) * (MT * 16) + m);
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) ssq += b + 4 * u + q < n ? v[u] : 0.f;
            }
          }
          const size_t sstride = (size_t)NT * MT * 64;
          const f32x4* const P0 = reinterpret_cast<const f32x4*>(p.wpart) + ((size_t)sid0 * NT + a0) * (MT * 64) + mt * 64 + lane;
          const f32x4* const Da = dtab + ((size_t)(s * (sg.N[0] >> 4) + tile) * MT + mt) * 64 + lane;
          const f32x4* const Db = dtab + ((size_t)((sg.N[0] >> 4) + tile) * MT + mt) * 64 + lane;
          // bias and residual travel with the partial tiles
          u32x2 g_bias = {0u, 0u}, g_rb = {0u, 0u};
          f32x4 g_rf = {0.f, 0.f, 0.f, 0.f};
          if (m < p.M) {
            if (sg.bias[s]) g_bias = *reinterpret_cast<const u32x2*>(sg.bias[s] + ncol);
            if (sg.resid_bf16) g_rb = *reinterpret_cast<const u32x2*>(sg.resid_bf16 + (size_t)m * sg.ld_resid + ncol);
            if (sg.resid_f32) g_rf = *reinterpret_cast<const f32x4*>(sg.resid_f32 + (size_t)m * sg.ld_resid + ncol);
          }
          f32x4 da = {0.f, 0.f, 0.f, 0.f}, db = {0.f, 0.f, 0.f, 0.f};
          if (sg.pair) {  // gate and up tiles of four segments per round trip, the LoRA term tiles with the first
            for (int i = 0; i < n; i += 4) {
              const f32x4* q10[10];
              f32x4 v[10];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int iu = i + u < n ? i + u : n - 1;
                q10[u] = P0 + iu * sstride;
                q10[4 + u] = P0 + iu * sstride + MT * 64;
              }
              q10[8] = has_a ? Da : P0;
              q10[9] = has_b ? Db : P0;
              if (i == 0) {
                ld_through10(q10, v);
                if (has_a) da = v[8];
                if (has_b) db = v[9];
              } else {
                const f32x4* q8[8];
                f32x4 v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) q8[u] = q10[u];
                ld_through8(q8, v8);
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = v8[u];
              }
#pragma unroll
              for (int u = 0; u < 4; ++u)
                if (i + u < n) {
                  sa += v[u];
                  sb += v[4 + u];
                }
            }
          } else {  // eight segments per round trip
            for (int i = 0; i < n; i += 8) {
              const f32x4* q10[10];
              f32x4 v[10];
#pragma unroll
              for (int u = 0; u < 8; ++u) q10[u] = P0 + (i + u < n ? i + u : n - 1) * sstride;
              q10[8] = has_a ? Da : P0;
              q10[9] = P0;
              if (i == 0) {
                ld_through10(q10, v);
                if (has_a) da = v[8];
              } else {
                const f32x4* q8[8];
                f32x4 v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) q8[u] = q10[u];
                ld_through8(q8, v8);
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = v8[u];
              }
#pragma unroll
              for (int u = 0; u < 8; ++u)
                if (i + u < n) sa += v[u];
            }
          }
          if (sg.norm) {
            ssq += __shfl_xor(ssq, 16, 64);
            ssq += __shfl_xor(ssq, 32, 64);
          }
          if (m < p.M) {
            const float inv = sg.norm ? rsqrtf(ssq / (float)sg.K + 1e-5f) : 1.f;
            float val[4];
#pragma unroll
            for (int z = 0; z < 4; ++z) {
              const float v0 = (sa[z] + da[z]) * inv;
              val[z] = sg.pair ? silu(v0) * ((sb[z] + db[z]) * inv) : v0;
            }
            if (sg.bias[s]) {
              val[0] += __uint_as_float(g_bias[0] << 16);
              val[1] += __uint_as_float(g_bias[0] & 0xffff0000u);
              val[2] += __uint_as_float(g_bias[1] << 16);
              val[3] += __uint_as_float(g_bias[1] & 0xffff0000u);
            }
            if (sg.resid_bf16) {
              val[0] += __uint_as_float(g_rb[0] << 16);
              val[1] += __uint_as_float(g_rb[0] & 0xffff0000u);
              val[2] += __uint_as_float(g_rb[1] << 16);
              val[3] += __uint_as_float(g_rb[1] & 0xffff0000u);
            }
            if (sg.resid_f32) {
#pragma unroll
              for (int z = 0; z < 4; ++z) val[z] += g_rf[z];
            }
            if (sg.out_f32) st_through(reinterpret_cast<f32x4*>(sg.out_f32 + (size_t)m * sg.ld_f32 + ncol), f32x4{val[0], val[1], val[2], val[3]});
            const u32x2 o = {pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3])};
            if (sg.out[s]) *reinterpret_cast<u32x2*>(sg.out[s] + (size_t)m * sg.ld_out[s] + ncol) = o;
            if (sg.out_pk && (sg.pair || s == sg.n_seg - 1)) st_through(reinterpret_cast<u32x2*>(sg.out_pk + packed_x_offset(m, ncol, MT)), o);
          }
        }
    }
    // ---- level end: the last wave to get here hands the level over ----
    wait_all_mem();
    TS(5);
    {
      int old = 0;
      if (lane == 0) old = __hip_atomic_fetch_add(&c.lvl_arr[L], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      old = __builtin_amdgcn_readfirstlane(old);
      if (old + 1 == kWaves && lane == 0) st_agent(p.flags + wg, epoch * 16 + (L + 1 < p.n_stages ? L + 1 : 15));
    }
  }
}

int mt_for(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : (M <= 64 ? 4 : 8)); }
int ns_max_for(int MT) { return MT <= 2 ? Cfg<2>::NS : (MT == 4 ? Cfg<4>::NS : Cfg<8>::NS); }


// One workgroup per compute unit, all resident at once (the grid barrier relies on that).
template <int MT>
int stream_grid() {
  static int cached = 0;
  if (cached) return cached;
  int dev = 0, cus = 0, occ = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_stream_kernel<MT, false>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
    return 0;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_stream_kernel<MT, true>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
    return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, decode_stream_kernel<MT, false>, kThreads, kLdsBytes) != hipSuccess)
    return 0;
  if (occ < 1 || cus < 1) return 0;
  cached = cus > kMaxGrid ? kMaxGrid : cus;
  return cached;
}

int grid_for(int MT) {
  switch (MT) {
    case 1: return stream_grid<1>();
    case 2: return stream_grid<2>();
    case 4: return stream_grid<4>();
    default: return stream_grid<8>();
  }
}

template <bool TRACE>
void launch_stream_t(const Params& p, int MT, int G, hipStream_t st) {
  switch (MT) {
    case 1: hipLaunchKernelGGL((decode_stream_kernel<1, TRACE>), dim3(G), dim3(kThreads), kLdsBytes, st, p); break;
    case 2: hipLaunchKernelGGL((decode_stream_kernel<2, TRACE>), dim3(G), dim3(kThreads), kLdsBytes, st, p); break;
    case 4: hipLaunchKernelGGL((decode_stream_kernel<4, TRACE>), dim3(G), dim3(kThreads), kLdsBytes, st, p); break;
    default: hipLaunchKernelGGL((decode_stream_kernel<8, TRACE>), dim3(G), dim3(kThreads), kLdsBytes, st, p); break;
  }
}

int launch_stream(const Params& p, int MT, int G, hipStream_t st) {
  if (p.trace) launch_stream_t<true>(p, MT, G, st);
  else launch_stream_t<false>(p, MT, G, st);
  return check_launch();
}

// The wide kernel's grid: one workgroup per compute unit, at most as many as the segment tables hold.
template <int MT>
int wide_grid() {
  static int cached = 0;
  if (cached) return cached;
  int dev = 0, cus = 0, occ = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_wide_kernel<MT, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kLdsBytes) != hipSuccess)
    return 0;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_wide_kernel<MT, true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kLdsBytes) != hipSuccess)
    return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, decode_wide_kernel<MT, false>, kThreads, kLdsBytes) != hipSuccess) return 0;
  if (occ < 1 || cus < 1) return 0;
  cached = cus > kWideGridMax ? kWideGridMax : cus;
  return cached;
}

int wide_tiles_per_group(int MT) { return kSW * (MT == 4 ? WCfg<4>::TPW : WCfg<8>::TPW); }

// Segments a launch can leave: every workgroup's piece ends one, and so does every group.
int wide_segments(int MT, int d, int F) {
  const int NT = wide_tiles_per_group(MT);
  const int g_qkv = (3 * (d >> 4) + NT - 1) / NT, g_gu = ((F >> 4) + NT / 2 - 1) / (NT / 2);
  return kWideGridMax + (g_qkv > g_gu ? g_qkv : g_gu);
}

void reset_stage(Stage& s) {
  s.X = nullptr; s.ldx = 0; s.K = 0; s.x_packed = 0; s.out_pk = nullptr; s.n_seg = 0; s.pair = 0; s.norm = 0; s.sync_before = 0; s.lora_shrink = 0; s.tpos0 = 0;
  s.unit0 = 0; s.units = 0; s.cap = 1; s.ksplit = 1;
  for (int i = 0; i < 3; ++i) {
    s.W[i] = nullptr; s.N[i] = 0; s.site[i] = -1; s.bias[i] = nullptr; s.out[i] = nullptr; s.ld_out[i] = 0;
  }
  s.resid_bf16 = nullptr; s.resid_f32 = nullptr; s.ld_resid = 0; s.out_f32 = nullptr; s.ld_f32 = 0;
}

// Cut `left` units into stages: a stage hands every workgroup the same number `cap` of units, cap * per_unit
// being a tile count the ring rounds serve (a divisor of ns_max).  Minimises the summed caps (the time,
// in units of one tile column per workgroup), then the number of stages.  caps[] receives the choice.
int plan_level(int left, int G, int per_unit, int ns_max, int depth, int* caps, int* n_caps) {
  if (left <= 0) { *n_caps = 0; return 0; }
  int best = 1 << 30, best_n = 1 << 30;
  if (depth >= kMaxStages) return best;
  for (int c = 1; c * per_unit <= ns_max; ++c) {
    if (ns_max % (c * per_unit) != 0) continue;
    int sub[kMaxStages], n_sub = 0;
    const long rest = (long)left - (long)c * G;
    const int t = plan_level(rest > 0 ? (int)rest : 0, G, per_unit, ns_max, depth + 1, sub, &n_sub);
    if (t >= (1 << 30)) continue;
    if (c + t < best || (c + t == best && n_sub + 1 < best_n)) {
      best = c + t;
      best_n = n_sub + 1;
      caps[0] = c;
      for (int i = 0; i < n_sub; ++i) caps[1 + i] = sub[i];
      *n_caps = best_n;
    }
  }
  return best;
}

// Append the stages of one level.  In a stage workgroup g takes units [g * cap, (g + 1) * cap) of the stage's
// range (the last workgroup with work may get fewer, the ones after it none: they spend the stage prefetching
// the weights of their next one).  Returns false when the launch would need more stages than it has.
bool push_level(Params& p, const Stage& level, int units_total, int G, int ns_max) {
  const int per_unit = level.pair ? 2 : 1;
  if (level.ksplit == 2) {
    // one stage: pairs of workgroups share pairs of tiles, each taking one half of the reduction
    const bool fits = level.n_seg == 1 && !level.pair && !level.norm && units_total % 2 == 0 && units_total <= (G & ~1) && units_total <= kMaxSplitGrid &&
                      (level.K >> 5) % 2 == 0 && ns_max % 2 == 0 && p.xpart != nullptr;
    if (fits) {
      if (p.n_stages >= kMaxStages) return false;
      Stage& s = p.st[p.n_stages++];
      s = level;
      s.unit0 = 0;
      s.units = units_total;
      s.cap = 1;
      s.lora_shrink = 1;
      return true;
    }
  }
  int caps[kMaxStages], n_caps = 0;
  if (plan_level(units_total, G, per_unit, ns_max, 0, caps, &n_caps) >= (1 << 30)) return false;
  int left = units_total, u = 0;
  for (int i = 0; i < n_caps; ++i) {
    if (p.n_stages >= kMaxStages) return false;
    Stage& s = p.st[p.n_stages++];
    s = level;
    s.ksplit = 1;
    s.unit0 = u;
    s.units = left < caps[i] * G ? left : caps[i] * G;
    s.cap = caps[i];
    s.sync_before = i == 0 ? level.sync_before : 0;
    s.lora_shrink = i == 0 ? 1 : 0;
    u += s.units;
    left -= s.units;
  }
  return true;
}

// ---- workspace layout ------------------------------------------------------------------------------------
struct DecodeWs {
  int* flags;      // [kMaxGrid] barrier flags; zero before the first launch, then owned by the kernels
  int* status;
  int* xflag;      // [kMaxGrid] flags of the partial tiles swapped inside ksplit stages; zero before the first launch
  float* xpart;    // [kMaxSplitGrid][row tiles][256] those tiles
  int* tready;     // [kSlotsPerRow kMaxRows] per shrink slot: epoch of the launch that published it
  int* tcount;     // [kSlotsPerRow kMaxRows] partials written so far (zero between launches)
  float* tfin;     // [kSlotsPerRow M][r_max] published shrinks
  float* tpart;    // [kSlotsPerRow M][NCmax][r_max] shrink partials
  float* h_f32;    // [M][d]
  bf16_t* v_pk;    // a = v as operand blocks   (K = d)
  bf16_t* h_pk;    // h as operand blocks       (K = d)
  bf16_t* m_pk;    // m = silu(g) * u as operand blocks (K = F)
  int* segflag;    // wide kernel, layer decode of more than 32 rows only: see Params
  float* wss;
  float* wpart;
  int* tpflag;
  int* dready;
  float* delta;
  int delta_odd, slabs_max;
  size_t bytes;
};

DecodeWs carve_decode_ws(void* base, int M, int d, int F, int r_max, bool wide = false) {
  const int big = F > d ? F : d;
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += align_up(n, 256); return o; };
  const size_t o_fl = take((size_t)(2 * kMaxGrid + 64) * sizeof(int));
  const size_t o_p = take((size_t)kMaxRows * 2 * kSlotsPerRow * sizeof(int));  // at a fixed place whatever M is: the counters must read zero
  const size_t o_tf = take((size_t)kSlotsPerRow * M * r_max * sizeof(float));
  const size_t o_t = take((size_t)kSlotsPerRow * M * shrink_chunks(big) * r_max * sizeof(float));
  const size_t o_h = take((size_t)M * d * sizeof(float));
  const int rows = mt_for(M) * 16;
  const size_t o_v = take((size_t)rows * d * sizeof(bf16_t));
  const size_t o_hb = take((size_t)rows * d * sizeof(bf16_t));
  const size_t o_m = take((size_t)rows * F * sizeof(bf16_t));
  const size_t o_xp = M <= 32 ? take((size_t)kMaxSplitGrid * rows * 16 * sizeof(float)) : 0;  // ksplit stages: up to 32 rows only
  size_t o_sf = 0, o_ss = 0, o_wp = 0, o_tp = 0, o_dr = 0, o_dt = 0;
  // LoRA term tiles of the wide kernel: the sites of an even level (q,k,v or gate,up) side by side, then those of an
  // odd level (o or down); 256-column slabs of the widest site
  const int tiles_even = 3 * (d >> 4) > 2 * (F >> 4) ? 3 * (d >> 4) : 2 * (F >> 4), tiles_odd = d >> 4;
  const int slabs_max = (big + 255) >> 8;
  if (wide) {
    const int MT = mt_for(M), segs = 2 * wide_segments(MT, d, F);
    o_sf = take((size_t)segs * sizeof(int));
    o_ss = take((size_t)segs * rows * sizeof(float));
    o_wp = take((size_t)segs * wide_tiles_per_group(MT) * MT * 1024);
    o_tp = take((size_t)kSlotsPerRow * kMaxRows * kTpStride * sizeof(int));
    o_dr = take((size_t)2 * 3 * slabs_max * kMaxRows * sizeof(int));
    o_dt = take((size_t)(tiles_even + tiles_odd) * MT * 1024);
  }
  char* b = (char*)base;
  int* fl = (int*)(b + o_fl);
  return DecodeWs{fl, fl + kMaxGrid, fl + kMaxGrid + 64, M <= 32 ? (float*)(b + o_xp) : nullptr, (int*)(b + o_p), (int*)(b + o_p) + kSlotsPerRow * kMaxRows, (float*)(b + o_tf), (float*)(b + o_t), (float*)(b + o_h),
                  (bf16_t*)(b + o_v), (bf16_t*)(b + o_hb), (bf16_t*)(b + o_m), (int*)(b + o_sf), (float*)(b + o_ss), (float*)(b + o_wp),
                  (int*)(b + o_tp), (int*)(b + o_dr), (float*)(b + o_dt), tiles_even, slabs_max, off};
}

void fill_common(Params& p, const DecodeWs& ws, int M, int Breq, int Kmax, const AdapterView& ad, const int32_t* tenant_id,
                 const uint8_t* route, const int32_t* row_to_req) {
  p.n_stages = 0; p.M = M; p.Breq = Breq; p.ad = ad; p.tenant_id = tenant_id; p.route = route; p.row_to_req = row_to_req;
  p.lora = 1;
  p.tpart = ws.tpart; p.tfin = ws.tfin; p.tcount = ws.tcount; p.tready = ws.tready; p.nc_max = shrink_chunks(Kmax);
  p.flags = ws.flags; p.status = ws.status; p.xflag = ws.xflag; p.xpart = ws.xpart; p.spin_limit = g_wait_limit.load(std::memory_order_relaxed);
  p.trace = nullptr;
  p.wpart = ws.wpart; p.wss = ws.wss; p.segflag = ws.segflag; p.wsegs = 0;
  p.tpflag = ws.tpflag; p.dready = ws.dready; p.delta = ws.delta; p.delta_odd = ws.delta_odd; p.slabs_max = ws.slabs_max;
}

}  // namespace

int set_wait_limit(int polls) {
  return g_wait_limit.exchange(polls > 0 ? polls : kSpinLimit, std::memory_order_relaxed);
}

size_t decode_packed_workspace_bytes(int M, int d, int F, int r_max) { return carve_decode_ws(nullptr, M, d, F, r_max, M > 32).bytes; }

// The word the stream kernels set when one of their bounded waits ran out (it lies at the same place in every
// workspace of the packed paths).  Waits for the stream's work, then copies the word to the host.
int decode_workspace_status(const void* workspace, int* status, hipStream_t st) {
  const DecodeWs ws = carve_decode_ws(const_cast<void*>(workspace), 1, 32, 32, 1);
  MILORA_HIP(hipMemcpyAsync(status, ws.status, sizeof(int), hipMemcpyDeviceToHost, st));
  MILORA_HIP(hipStreamSynchronize(st));
  return MILORA_OK;
}


// One decode step of a layer on packed weights: one launch over the stages q,k,v | o | gate,up | down.
int layer_decode_packed(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                        const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                        bf16_t* y, bf16_t* qkv_out, void* workspace, hipStream_t st, LaunchMarks* marks) {
  const int MT = mt_for(B);
  const bool wide = MT >= 4;  // more than 32 rows: the kernel that cuts the reduction over the workgroups
  const int G = wide ? (MT == 4 ? wide_grid<4>() : wide_grid<8>()) : grid_for(MT);
  if (G <= 0) return hip_fail(hipGetLastError());
  const int nsm = ns_max_for(MT);
  DecodeWs ws = carve_decode_ws(workspace, B, d, F, ad.r_max, B > 32);
  const int norm = (flags & MILORA_LAYER_RMSNORM) ? 1 : 0;
  Params p;
  fill_common(p, ws, B, B, F > d ? F : d, ad, tenant_id, route, nullptr);
  Stage lv[4];
  int units[4];
  // level 0: q, k, v from x
  {
    Stage& l = lv[0];
    reset_stage(l);
    l.X = x; l.ldx = d; l.K = d; l.n_seg = 3; l.norm = norm;
    for (int s = 0; s < 3; ++s) {
      l.W[s] = (const bf16_t*)wts->W[s]; l.N[s] = d; l.site[s] = s;
      if (qkv_out) { l.out[s] = qkv_out + (size_t)s * d; l.ld_out[s] = 3 * d; }
    }
    if (!attn_out) l.out_pk = ws.v_pk;  // a = v goes to the next stage as operand blocks
    units[0] = 3 * (d >> 4);
  }
  // level 1: h = x + L_o(a)
  {
    Stage& l = lv[1];
    reset_stage(l);
    if (attn_out) { l.X = attn_out; l.ldx = d; }
    else { l.X = ws.v_pk; l.x_packed = 1; l.sync_before = 1; }
    l.K = d; l.n_seg = 1;
    l.W[0] = (const bf16_t*)wts->W[3]; l.N[0] = d; l.site[0] = 3;
    l.resid_bf16 = x; l.ld_resid = d;
    l.out_f32 = ws.h_f32; l.ld_f32 = d;
    l.out_pk = ws.h_pk;
    l.tpos0 = 3;
    l.ksplit = 2;
    units[1] = d >> 4;
  }
  // level 2: m = silu(L_gate(n(h))) * L_up(n(h))
  {
    Stage& l = lv[2];
    reset_stage(l);
    l.X = ws.h_pk; l.x_packed = 1; l.K = d; l.n_seg = 2; l.pair = 1; l.norm = norm; l.sync_before = 1;
    for (int s = 0; s < 2; ++s) { l.W[s] = (const bf16_t*)wts->W[4 + s]; l.N[s] = F; l.site[s] = 4 + s; }
    l.out_pk = ws.m_pk;
    units[2] = F >> 4;
  }
  // level 3: y = h + L_down(m)
  {
    Stage& l = lv[3];
    reset_stage(l);
    l.X = ws.m_pk; l.x_packed = 1; l.K = F; l.n_seg = 1; l.sync_before = 1;
    l.W[0] = (const bf16_t*)wts->W[6]; l.N[0] = d; l.site[0] = 6;
    l.resid_f32 = ws.h_f32; l.ld_resid = d;
    l.out[0] = y; l.ld_out[0] = d;
    l.tpos0 = 3;
    l.ksplit = 2;
    units[3] = d >> 4;
  }
  if (marks && marks->trace) p.trace = marks->trace;
  if (wide) {
    for (int L = 0; L < 4; ++L) {
      p.st[L] = lv[L];
      p.st[L].ksplit = 1;
      p.st[L].lora_shrink = 1;
    }
    p.n_stages = 4;
    if (marks) { marks->grid = G; marks->stages = 4; }
    p.wsegs = wide_segments(MT, d, F);
    if (MT == 4 && !p.trace) hipLaunchKernelGGL((decode_wide_kernel<4, false>), dim3(G), dim3(kThreads), kLdsBytes, st, p);
    else if (MT == 4) hipLaunchKernelGGL((decode_wide_kernel<4, true>), dim3(G), dim3(kThreads), kLdsBytes, st, p);
    else if (!p.trace) hipLaunchKernelGGL((decode_wide_kernel<8, false>), dim3(G), dim3(kThreads), kLdsBytes, st, p);
    else hipLaunchKernelGGL((decode_wide_kernel<8, true>), dim3(G), dim3(kThreads), kLdsBytes, st, p);
    const int rcw = check_launch();
    if (rcw) return rcw;
    if (marks && marks->n > 0) (void)hipEventRecord(marks->ev[0], st);
    return MILORA_OK;
  }
  for (int L = 0; L < 4; ++L)
    if (!push_level(p, lv[L], units[L], G, nsm)) return MILORA_ERANGE;
  if (marks) { marks->grid = G; marks->stages = p.n_stages; }
  int rc = launch_stream(p, MT, G, st);
  if (rc) return rc;
  if (marks && marks->n > 0) (void)hipEventRecord(marks->ev[0], st);
  return MILORA_OK;
}

size_t decode_trace_bytes() { return (size_t)kMaxGrid * kMaxStages * kWaves * kTraceSlots * sizeof(long long); }
int decode_trace_dims(int* stages_max, int* waves, int* slots) {
  *stages_max = kMaxStages; *waves = kWaves; *slots = kTraceSlots;
  return kMaxGrid;
}

// ---- layer decode on scratch memory the library itself holds ----------------------------------------------------
// For callers that can neither allocate nor hand over a workspace.  The array lives in every GPU the library runs
// on, from the first use of the library on it to the end of the process; each GPU has its own copy at its own
// address, looked up once per device.  In host code the array's name is only a handle for that lookup: what the
// kernels get is the looked-up address.
constexpr size_t kStaticScratchBytes = (size_t)MILORA_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];

static int static_scratch(void** out) {
  int dev = -1;
  MILORA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MILORA_ERANGE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    MILORA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MILORA_OK;
}

__global__ void __launch_bounds__(256) clear_words_kernel(uint32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Bytes at the start of a decode workspace that must read zero before its first launch: barrier flags, status word,
// shrink counters and ready words.
static size_t control_bytes() {
  static char base;
  const DecodeWs ws = carve_decode_ws(&base, 1, 32, 32, 1);
  return (size_t)((const char*)ws.tfin - &base);
}

int layer_decode_packed_static(const bf16_t* x, int B, int d, int F, const milora_layer_weights* wts, const AdapterView& ad,
                               const int32_t* tenant_id, const uint8_t* route, uint32_t flags, const bf16_t* attn_out,
                               bf16_t* y, bf16_t* qkv_out, hipStream_t st) {
  if (B > 32) return MILORA_ERANGE;  // more rows take the kernel whose partial-tile tables need tens of MB
  if (carve_decode_ws(nullptr, B, d, F, ad.r_max, false).bytes > kStaticScratchBytes) return MILORA_ERANGE;
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc) return rc;
  // The array keeps what the last call left, and that call may have had other sizes or may have run out of a wait:
  // the control words start from zero in every call (a fill kernel, so that the call can be captured in a graph).
  const int words = (int)(control_bytes() / sizeof(uint32_t));
  hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, st, (uint32_t*)ptr, words);
  if ((rc = check_launch())) return rc;
  return layer_decode_packed(x, B, d, F, wts, ad, tenant_id, route, flags, attn_out, y, qkv_out, ptr, st, nullptr);
}

int static_scratch_status(int* status, hipStream_t st) {
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc) return rc;
  return decode_workspace_status(ptr, status, st);
}

// ---- one routed linear of M <= 128 rows on a packed weight ------------------------------------------
size_t routed_linear_packed_workspace_bytes(int M, int d1, int d2, int r_max) {
  (void)d2;
  return carve_decode_ws(nullptr, M, 32, d1, r_max).bytes;
}

int routed_linear_packed(const bf16_t* X, int M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                         const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                         const uint8_t* route, int B, bf16_t* Y, void* workspace, hipStream_t st) {
  const int MT = mt_for(M);
  const int G = grid_for(MT);
  if (G <= 0) return hip_fail(hipGetLastError());
  DecodeWs ws = carve_decode_ws(workspace, M, 32, d1, ad.r_max);
  Params p;
  fill_common(p, ws, M, B, d1, ad, tenant_id, route, row_to_req);
  Stage l;
  reset_stage(l);
  l.X = X; l.ldx = d1; l.K = d1; l.n_seg = 1;
  l.W[0] = W; l.N[0] = d2; l.site[0] = site; l.bias[0] = bias;
  l.out[0] = Y; l.ld_out[0] = d2;
  if (!push_level(p, l, d2 >> 4, G, ns_max_for(MT))) return MILORA_ERANGE;
  return launch_stream(p, MT, G, st);
}

int pack_weight(const void* src, void* dst, int d1, int d2, hipStream_t st) {
  const size_t groups = (size_t)d1 * d2 / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, (const u32x4*)src,
                     (u32x4*)dst, d1, d2);
  return check_launch();
}

}  // namespace milora
