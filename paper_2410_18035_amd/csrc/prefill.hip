// Many-row (prefill) routed LoRA linear on row-major bf16 weights (paper Eq. 1 with the layer-level gate of
// Sec. 3.3): Y = X W^T + bias + (X W^A) W^B for the rows whose request is routed to this site.
//
// One workgroup of four waves computes a 256 x 256 tile of Y with the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulators, 128 x 128 per wave; a kernel of nothing but this instruction
// sustains 2.3-2.4 PFLOP/s on the chip, one of nothing but the 16x16x32 form 1.45-1.5).  X and W are both contiguous along the
// reduction index: 16-row x 64-k blocks of either are copied from global memory straight into LDS
// (global_load_lds_dwordx4, no registers; whole 128-byte lines per row), in a ring of five half steps of
// 32 KB, and read back as matrix-core operands with one conflict-free 16-byte LDS load per lane, pair of blocks
// and 16 k.  A step's operands are all in registers after a quarter of its matrix work; its ring slots are
// refilled from there on, so that nearly the whole LDS is data on its way (the copies are bound by latency:
// bytes in flight over about two microseconds).
// The LoRA term enters as extra k steps: t = X W^A (fp32, computed beforehand) split into two bf16 halves
// (hi + lo, so nothing of t's precision is lost) against W^B of the tenant, masked to that tenant's rows.
// Bias is added and the result rounded once at the store.
#include "common.h"

namespace milora {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// Adapter matrices are reached through pointer tables read at run time; telling the compiler that they lie in
// global memory keeps their loads off the counter the LDS reads wait on.
typedef __attribute__((address_space(1))) const bf16_t gbf16;
__device__ __forceinline__ gbf16* in_global(const void* p) { return (gbf16*)p; }

constexpr int kTM = 256, kTN = 256, kTK = 64;
constexpr int kThreadsP = 256;
constexpr int kBlocksM = kTM / 16, kBlocksN = kTN / 16;
constexpr int kBlockBytes = 16 * kTK * 2;                 // 16 rows x 64 k: 2 KiB, a row is one 128-byte line
constexpr int kHalfBytes = (kBlocksM + kBlocksN) / 2 * kBlockBytes;  // 8 X blocks + 8 W blocks: 32 KiB
constexpr int kHalves = 5;                                // ring of half steps
constexpr int kLdsBytesP = kHalves * kHalfBytes;
constexpr int kAccTilesRows = 3;
// Where the sixteen copy instructions of a k step sit among its 64 matrix instructions: those of the first half
// after instructions 0, kCopyAStride, ..., those of the second half from instruction kCopyB0 on (16 or later: the
// slot they fill is read until then).
#ifndef PF_CA
#define PF_CA 2
#define PF_CB0 16
#define PF_CBS 3
#endif
constexpr int kCopyAStride = PF_CA, kCopyB0 = PF_CB0, kCopyBStride = PF_CBS;
static_assert(kCopyB0 >= 16 && 7 * kCopyAStride < kCopyB0 && kCopyB0 + 7 * kCopyBStride < 64, "copy positions");
constexpr int kShrinkSplit = kPrefillShrinkParts;  // the shrink's reduction is cut into this many parts, one workgroup each
constexpr int kGroupM = 4;  // consecutive workgroups of an XCD walk 4 row tiles of one column tile

struct PParams {
  const bf16_t* X;
  const bf16_t* W;
  const bf16_t* bias;
  bf16_t* Y;
  const float* t;     // kShrinkSplit partial shrinks [part][rows of the whole call][r_max], to be added in part order
  size_t t_stride;    // floats from one part to the next
  const int32_t* row_to_req;
  const int32_t* tenant_id;
  const uint8_t* route;
  AdapterView ad;
  int64_t M;         // rows of this launch
  int64_t row_base;  // index of its first row in the caller's matrix (requests of unmapped rows)
  int d1, d2, site, B;
  int tilesM, tilesN;
};

// Which of the eight 16-byte pieces of its 128-byte LDS line holds k group kg of row r (0..15) of a block:
// kg ^ swz(r).  Eight neighbouring rows get eight different pieces, and rows r and r + 8 (which lie 1 KiB apart, on
// the same banks) differ too, so a 16-byte operand read of 16 rows at one k group touches every bank once.
__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// 16 bytes per lane from base + voff (global) to LDS at dst + lane * 16, asynchronously; counted by vmcnt.
// Written as assembly so that the compiler does not order its own LDS reads behind the copy.
__device__ __forceinline__ void copy_to_lds(const void* base, uint32_t voff, uint32_t dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(dst), "v"(voff), "s"(base)
               : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

__global__ void __launch_bounds__(kThreadsP, 1) prefill_kernel(PParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  // workgroup -> tile: workgroup ids go round-robin over the 8 XCDs; each XCD takes a contiguous run of the
  // tile order, which walks kGroupM row tiles per column tile so that the XCD's L2 serves the re-reads
  // (the 32 workgroups resident on an XCD then cover 4 row tiles x 8 column tiles)
  const int total = p.tilesM * p.tilesN;
  const int per = (total + 7) / 8;
  const int id = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  if (id >= total) return;
  const int gspan = kGroupM * p.tilesN;
  const int first = id / gspan * kGroupM;
  const int gsz = p.tilesM - first < kGroupM ? p.tilesM - first : kGroupM;
  const int in_group = id % gspan;
  const int64_t m0 = (int64_t)(first + in_group % gsz) * kTM;
  const int n0 = in_group / gsz * kTN;

  const int KT = p.d1 / kTK;
  const uint32_t lds0 = lds_addr(lds);

  // copies.  A k step of 64 is brought in two halves: half 0 = X rows 0..127 and W rows 0..127 of the tile,
  // half 1 = the other rows; a half is 8 + 8 blocks of 16 rows, a block two copy instructions of 8 rows each
  // (8 lanes take the 128-byte line of a row, so every request is for whole cache lines).  Waves 0,1 bring
  // the X blocks of a half (4 each), waves 2,3 the W blocks.  Which 16 bytes of the line a lane takes is
  // permuted by the row so that the operand reads below spread over all LDS banks.
  const bool is_w = wave >= 2;
  const unsigned char* src = is_w ? (const unsigned char*)p.W : (const unsigned char*)p.X;
  const int64_t row0 = is_w ? (int64_t)n0 : m0;
  const int64_t rlim = is_w ? (int64_t)p.d2 : p.M;
  uint32_t voff[2][8];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int rr = lane >> 3;
      int64_t r = row0 + (hh * 8 + (wave & 1) * 4 + (j >> 1)) * 16 + (j & 1) * 8 + rr;
      r = r < rlim ? r : rlim - 1;
      voff[hh][j] = (uint32_t)((uint64_t)r * (uint32_t)p.d1 * 2u + (uint32_t)((lane & 7) ^ swz((j & 1) * 8 + rr)) * 16u);
    }
  const uint32_t dst_in_half = (uint32_t)((is_w ? 8 : 0) + (wave & 1) * 4) * kBlockBytes;
  // half H = 2 * (k step) + hh lives in ring slot H % kHalves
  // copy j (0..7) of a half; a wave's eight copies of a half are spread between its matrix instructions: issued
  // back to back they would hold the wave at the issue of the memory instructions while the matrix cores idle
  auto issue_one = [&](int kt, int hh, int slot, int j) __attribute__((always_inline)) {
    const int kk = kt < KT ? kt : KT - 1;  // past the end: re-read the last step into a slot nobody reads
    const unsigned char* b = src + (size_t)kk * (kTK * 2);
    const uint32_t dst = lds0 + slot * kHalfBytes + dst_in_half;
    copy_to_lds(b, voff[hh][j], dst + j * 1024);
  };
  auto issue = [&](int kt, int hh, int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 8; ++j) issue_one(kt, hh, slot, j);
  };

  // acc[i][j]: rows 32 i .. 32 i + 31 of the wave's X part against rows 32 j .. of its W part
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand read: lane l takes row l % 32 of a pair of 16-row blocks and the 16 bytes of k group 2 ks + l / 32
  // (ks = 0..3: the four 16-k sub-steps of a block's 64 k)
  const int rrow = lane & 31;
  int rd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    rd[ks] = (rrow >> 4) * kBlockBytes + (rrow & 15) * 128 + (((2 * ks + (lane >> 5)) ^ swz(rrow & 15)) << 4);
  const unsigned char* wbase = lds + (kBlocksM / 2) * kBlockBytes;
  // One k step of 64 for the wave's 128 x 128 part: 64 matrix instructions, number q = 16 ks + 4 i + j.  The
  // operand reads come early: the sixteen of the first two sub-steps, then the other sixteen between the matrix
  // instructions of the first sub-step.  `mid` runs after instruction 15, once every wave of the workgroup has
  // its operands in registers: the step's two ring slots are free from there on.  copy(q) runs after instruction q.
  auto mma64 = [&](int slot_x, int slot_w, auto mid, auto copy) __attribute__((always_inline)) {
    const unsigned char* sa = lds + slot_x * kHalfBytes;
    const unsigned char* sb = wbase + slot_w * kHalfBytes;
    bf16x8 a[4][4], b[4][4];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < 4; ++i) a[ks][i] = *(const bf16x8*)(sa + rd[ks] + i * 2 * kBlockBytes);
#pragma unroll
      for (int j = 0; j < 4; ++j) b[ks][j] = *(const bf16x8*)(sb + rd[ks] + j * 2 * kBlockBytes);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0][q & 3], a[0][q >> 2], acc[q >> 2][q & 3], 0, 0, 0);
      const int ks = 2 + (q >> 3), e = q & 3;
      if (q & 4) b[ks][e] = *(const bf16x8*)(sb + rd[ks] + e * 2 * kBlockBytes);
      else a[ks][e] = *(const bf16x8*)(sa + rd[ks] + e * 2 * kBlockBytes);
      copy(q);
      __builtin_amdgcn_sched_barrier(0);
    }
    mid();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 16; q < 64; ++q) {
      acc[(q >> 2) & 3][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[q >> 4][q & 3], a[q >> 4][(q >> 2) & 3],
                                                                         acc[(q >> 2) & 3][q & 3], 0, 0, 0);
      copy(q);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  issue(0, 0, 0);
  issue(0, 1, 1);
  issue(1, 0, 2);
  issue(1, 1, 3);
  // 12 of the 16 accumulator tiles in the accumulation registers, 4 in ordinary ones: with all 256 in the
  // accumulation file the compiler has no spare tile there and shuffles tiles between the files in the loop
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (i < kAccTilesRows) asm volatile("" : "+a"(acc[i][j]));
      else asm volatile("" : "+v"(acc[i][j]));
    }
  // The ring: halves 2 kt and 2 kt + 1 (this step) are read, the two of the next step are on their way, the
  // fifth slot takes the first half of the step after next at once and the second half goes into this step's
  // first slot as soon as every wave has taken its operands out: a copy has between one and three quarters and
  // two whole steps of matrix work to arrive.
  int h0 = 0;  // ring slot of half 0 of the current step
  for (int kt = 0; kt < KT; ++kt) {
    const int h1 = h0 + 1 >= kHalves ? h0 + 1 - kHalves : h0 + 1;
    const int h2 = h0 + 2 >= kHalves ? h0 + 2 - kHalves : h0 + 2;
    const int h4 = h0 + 4 >= kHalves ? h0 + 4 - kHalves : h0 + 4;
    wait_vm<16>();                  // all but the two halves issued last have landed: both halves of this step
    __builtin_amdgcn_s_barrier();   // for every wave
    asm volatile("" ::: "memory");
    mma64(
        wm ? h1 : h0, wn ? h1 : h0,
        [&]() __attribute__((always_inline)) {
          __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's operand reads have returned
          __builtin_amdgcn_s_barrier();        // and every other wave's
          asm volatile("" ::: "memory");
        },
        [&](int q) __attribute__((always_inline)) {
          // first half of the step after next into the free slot, second half into this step's first slot
          if (q < kCopyB0) {
            if (q % kCopyAStride == 0 && q / kCopyAStride < 8) issue_one(kt + 2, 0, h4, q / kCopyAStride);
          } else if ((q - kCopyB0) % kCopyBStride == 0 && (q - kCopyB0) / kCopyBStride < 8) {
            issue_one(kt + 2, 1, h0, (q - kCopyB0) / kCopyBStride);
          }
        });
    asm volatile("" ::: "memory");
    h0 = h2;
  }
  wait_vm<0>();
  __syncthreads();

  // ---- LoRA term of the routed rows as one more k step per 32 ranks ----------------------------------------
  // t = X W^A (fp32) goes in as bf16 hi + lo: hi in the first k half of a block, lo in the second, against the
  // same 32 rows of the tenant's W^B in both halves; rows of other tenants and unrouted rows enter as zeros.
  int* ctl = (int*)(lds + 2 * kHalfBytes);  // ring slots 0 and 1 hold the operand blocks
  int my_ten = -1;
  {
    const int64_t m = m0 + tid;
    if (m < p.M) {
      const int64_t req = p.row_to_req ? (int64_t)p.row_to_req[m] : p.row_base + m;
      int tenant = 0;
      const int r = (req >= 0 && req < p.B) ? routed_rank(p.ad, p.tenant_id, p.route, (int)req, p.B, p.site, &tenant) : 0;
      if (r) my_ten = tenant;
    }
  }
  int last = -1;
  for (;;) {
    if (tid == 0) ctl[0] = 0x7fffffff;
    __syncthreads();
    int cand = my_ten > last ? my_ten : 0x7fffffff;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_xor(cand, off, 64);
      cand = o < cand ? o : cand;
    }
    if (lane == 0) atomicMin(&ctl[0], cand);
    __syncthreads();
    const int cur = ctl[0];
    if (cur == 0x7fffffff) break;
    const int r = p.ad.rank[cur];
    gbf16* Bm = in_global(p.ad.B[cur * MILORA_NUM_SITES + p.site]);
    const int64_t m = m0 + tid;
    const int n = n0 + tid;
    // thread tid fills row tid of the X side and row tid of the W side
    const uint32_t rb = (uint32_t)(tid & 15);
    const uint32_t blk = (uint32_t)(tid >> 7) * kHalfBytes + (uint32_t)((tid >> 4) & 7) * kBlockBytes + rb * 128;
    for (int c0 = 0; c0 < r; c0 += 32) {
      // t of the tile's 256 rows for these 32 ranks, the shrink's parts added in part order, through LDS: eight
      // lanes read the 128 bytes of a row (whole lines), then every thread picks up its own row
      float* const ts = reinterpret_cast<float*>(lds + 2 * kHalfBytes + 1024);  // [256][33]
      const bool vec = (p.ad.r_max & 3) == 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (tid >> 3) + 32 * i, cq = c0 + (tid & 7) * 4;
        const int64_t mr = m0 + row;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (mr < p.M) {
          const float* q = p.t + (size_t)mr * p.ad.r_max + cq;
          if (vec && cq + 3 < p.ad.r_max) {
#pragma unroll
            for (int part = 0; part < kShrinkSplit; ++part) {
              const f32x4 x = *reinterpret_cast<const f32x4*>(q + part * p.t_stride);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += x[e];
            }
          } else {
            for (int e = 0; e < 4; ++e)
              if (cq + e < p.ad.r_max)
                for (int part = 0; part < kShrinkSplit; ++part) v[e] += q[part * p.t_stride + e];
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) ts[row * 33 + (tid & 7) * 4 + e] = v[e];
      }
      __syncthreads();
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x4 hi, lo, wb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float tv[2];
          uint32_t bw[2];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int c = c0 + g * 8 + e * 2 + h;
            tv[h] = (my_ten == cur && c < r) ? ts[tid * 33 + (c - c0)] : 0.f;
            bw[h] = (c < r && n < p.d2) ? (uint32_t)Bm[(size_t)c * p.d2 + n] : 0u;
          }
          const bf16_t h0b = f32_to_bf16(tv[0]), h1b = f32_to_bf16(tv[1]);
          hi[e] = (uint32_t)h0b | ((uint32_t)h1b << 16);
          lo[e] = pack_bf16x2(tv[0] - bf16_to_f32(h0b), tv[1] - bf16_to_f32(h1b));
          wb[e] = bw[0] | (bw[1] << 16);
        }
        const uint32_t o_hi = blk + (((uint32_t)g ^ (uint32_t)swz(rb)) << 4);
        const uint32_t o_lo = blk + (((uint32_t)(g + 4) ^ (uint32_t)swz(rb)) << 4);
        *(u32x4*)(lds + o_hi) = hi;
        *(u32x4*)(lds + o_lo) = lo;
        *(u32x4*)(lds + (kBlocksM / 2) * kBlockBytes + o_hi) = wb;
        *(u32x4*)(lds + (kBlocksM / 2) * kBlockBytes + o_lo) = wb;
      }
      __syncthreads();
      mma64(wm, wn, []() {}, [](int) {});
      __syncthreads();
    }
    last = cur;
  }

  // ---- bias, one rounding, store: of a 32 x 32 tile a lane holds row l % 32 and, in registers 4 g .. 4 g + 3, the
  // columns 8 g + 4 (l / 32) .. + 3
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = n0 + wn * 128 + j * 32 + g * 8 + (lane >> 5) * 4;
      if (n >= p.d2) continue;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (p.bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[e] = bf16_to_f32(p.bias[n + e]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + wm * 128 + i * 32 + (lane & 31);
        if (m >= p.M) continue;
        u32x2 v;
        v[0] = pack_bf16x2(acc[i][j][4 * g] + bv[0], acc[i][j][4 * g + 1] + bv[1]);
        v[1] = pack_bf16x2(acc[i][j][4 * g + 2] + bv[2], acc[i][j][4 * g + 3] + bv[3]);
        *(u32x2*)(p.Y + (size_t)m * p.d2 + n) = v;
      }
    }
  }
}

// ---- LoRA shrink for many rows: t[m][0..r) = X[m] . W^A of the row's tenant, routed rows only --------------
// One workgroup per 64 rows, 16 per wave.  W^A is [d1][r] (reduction index outermost), the matrix cores
// want 8 consecutive reduction indices per lane, so 256-row chunks of W^A go through LDS and are read back
// column-wise; X rows come straight from global memory as operands, a chunk's worth at a time.  A tile
// whose rows belong to several tenants is computed once per tenant and each row keeps its own tenant's
// result.  Needs d1 % 32 == 0.
constexpr int kShrinkRows = 64, kShrinkK = 256, kShrinkC = 64;
constexpr int kShrinkLd = 66;  // LDS row of 64 columns padded: the 4 k groups of a column read hit distinct banks

__global__ void __launch_bounds__(256, 2) shrink_tiles_kernel(const bf16_t* __restrict__ X, int64_t M, int64_t row_base,
                                                              int d1, const int32_t* __restrict__ row_to_req,
                                                              AdapterView ad, int site,
                                                              const int32_t* __restrict__ tenant_id,
                                                              const uint8_t* __restrict__ route, int B,
                                                              float* __restrict__ t, size_t t_stride) {
  __shared__ bf16_t As[kShrinkK][kShrinkLd];
  __shared__ int row_ten[kShrinkRows];
  __shared__ int next_ten;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t m0 = (int64_t)blockIdx.x * kShrinkRows;
  if (tid < kShrinkRows) {
    const int64_t m = m0 + tid;
    int ten = -1;
    if (m < M) {
      const int64_t req = row_to_req ? (int64_t)row_to_req[m] : row_base + m;
      int tenant = 0;
      if (req >= 0 && req < B && routed_rank(ad, tenant_id, route, (int)req, B, site, &tenant)) ten = tenant;
    }
    row_ten[tid] = ten;
  }
  __syncthreads();
  // this workgroup's part of the reduction (whole chunks; the last parts may be empty and then write zeros)
  const int per_part = ((d1 + kShrinkSplit * kShrinkK - 1) / (kShrinkSplit * kShrinkK)) * kShrinkK;
  const int k_begin = (int)blockIdx.y * per_part < d1 ? (int)blockIdx.y * per_part : d1;
  const int k_end = k_begin + per_part < d1 ? k_begin + per_part : d1;
  t += (size_t)blockIdx.y * t_stride;
  const int my_row = wave * 16 + (lane & 15);
  int64_t xrow = m0 + my_row;
  xrow = xrow < M ? xrow : M - 1;
  const bf16_t* xp = X + (size_t)xrow * d1 + (lane >> 4) * 8;
  int last = -1;
  for (;;) {
    if (tid == 0) next_ten = 0x7fffffff;
    __syncthreads();
    if (tid < kShrinkRows && row_ten[tid] > last) atomicMin(&next_ten, row_ten[tid]);
    __syncthreads();
    const int cur = next_ten;
    if (cur == 0x7fffffff) break;
    const int r = ad.rank[cur];
    gbf16* A = in_global(ad.A[cur * MILORA_NUM_SITES + site]);
    for (int cb = 0; cb < r; cb += kShrinkC) {
      const int rc = r - cb < kShrinkC ? r - cb : kShrinkC;
      const int ntile = (rc + 15) >> 4;
      f32x4 acc[4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      // this thread stages column c of every fourth row of a chunk; columns past the rank and rows past d1
      // read a valid element instead (what they produce is never stored / never used)
      const int c = tid & 63;
      gbf16* ap = A + cb + (c < rc ? c : 0);
      for (int k0 = k_begin; k0 < k_end; k0 += kShrinkK) {
        const int steps = k_end - k0 < kShrinkK ? (k_end - k0) / 32 : kShrinkK / 32;
        bf16x8 xf[kShrinkK / 32];
#pragma unroll
        for (int ks = 0; ks < kShrinkK / 32; ++ks) xf[ks] = *(const bf16x8*)(xp + k0 + (ks < steps ? ks : 0) * 32);
        __syncthreads();  // the chunk before has been read
#pragma unroll 16
        for (int i = 0; i < kShrinkK / 4; ++i) {
          int k = k0 + (tid >> 6) + 4 * i;
          k = k < k_end ? k : k_end - 1;
          As[(tid >> 6) + 4 * i][c] = ap[(size_t)k * r];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < kShrinkK / 32; ++ks) {
          if (ks < steps) {
            const int kk0 = ks * 32 + (lane >> 4) * 8;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
              if (nt < ntile) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  w[e] = (uint32_t)As[kk0 + 2 * e][nt * 16 + (lane & 15)] |
                         ((uint32_t)As[kk0 + 2 * e + 1][nt * 16 + (lane & 15)] << 16);
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), xf[ks], acc[nt], 0, 0, 0);
              }
            }
          }
        }
      }
      __syncthreads();
      // lane holds row lane % 16 of the wave, columns (lane / 16) * 4 .. + 4 of each 16-column tile
      const int64_t m = m0 + my_row;
      if (m < M && row_ten[my_row] == cur) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int cc = cb + nt * 16 + (lane >> 4) * 4 + e;
            if (nt < ntile && cc < r) t[(size_t)m * ad.r_max + cc] = acc[nt][e];
          }
      }
    }
    last = cur;
  }
}

}  // namespace

bool prefill_supported(int64_t M, int d1, int d2, const void* X, const void* W, const void* Y) {
  if (M < 64 || d1 % kTK != 0 || d2 % 16 != 0) return false;
  if ((((uintptr_t)X | (uintptr_t)W) & 15) != 0 || ((uintptr_t)Y & 7) != 0) return false;
  return (uint64_t)d2 * (uint64_t)d1 * 2u < (1ull << 32);  // 32-bit byte offsets inside W (X is cut into row slices)
}

int routed_linear_prefill(const bf16_t* X, int64_t M, int d1, int d2, const int32_t* row_to_req, const bf16_t* W,
                          const bf16_t* bias, const AdapterView& ad, int site, const int32_t* tenant_id,
                          const uint8_t* route, int B, const float* t, bf16_t* Y, hipStream_t stream) {
  static thread_local int lds_set_for = -1;
  int dev = 0;
  MILORA_HIP(hipGetDevice(&dev));
  if (lds_set_for != dev) {
    MILORA_HIP(hipFuncSetAttribute((const void*)prefill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesP));
    lds_set_for = dev;
  }
  // rows are independent: slices whose byte offsets inside X fit 32 bits and whose tile count fits a launch
  int64_t slice = (int64_t)(((1ull << 32) - 1) / ((uint64_t)d1 * 2u)) / kTM * kTM;
  const int tilesN = (d2 + kTN - 1) / kTN;
  const int64_t by_grid = (int64_t)((1 << 24) / tilesN) * kTM;
  if (slice > by_grid) slice = by_grid;
  if (slice < kTM) return MILORA_EUNSUPPORTED;
  for (int64_t r0 = 0; r0 < M; r0 += slice) {
    PParams p;
    p.M = M - r0 < slice ? M - r0 : slice;
    p.X = X + (size_t)r0 * d1;
    p.W = W;
    p.bias = bias;
    p.Y = Y + (size_t)r0 * d2;
    p.t = t + (size_t)r0 * ad.r_max;
    p.t_stride = (size_t)M * ad.r_max;
    p.row_to_req = row_to_req ? row_to_req + r0 : nullptr;
    p.row_base = r0;
    p.tenant_id = tenant_id;
    p.route = route;
    p.ad = ad;
    p.d1 = d1;
    p.d2 = d2;
    p.site = site;
    p.B = B;
    p.tilesM = (int)((p.M + kTM - 1) / kTM);
    p.tilesN = tilesN;
    const int total = p.tilesM * p.tilesN;
    const int per = (total + 7) / 8;
    hipLaunchKernelGGL(prefill_kernel, dim3(8 * per), dim3(kThreadsP), kLdsBytesP, stream, p);
    const int rc = check_launch();
    if (rc) return rc;
  }
  return MILORA_OK;
}

// LoRA shrink of the rows the tile kernel serves (same conditions as prefill_supported): t receives
// kPrefillShrinkParts partial results [part][M][r_max] that routed_linear_prefill adds in part order.
int launch_shrink_tiles(const bf16_t* X, int64_t M, int d1, const int32_t* row_to_req, const AdapterView& ad, int site,
                        const int32_t* tenant_id, const uint8_t* route, int B, float* t, hipStream_t stream) {
  const int64_t slice = (int64_t)1 << 30;  // rows per launch: the grid index stays well inside 32 bits
  for (int64_t r0 = 0; r0 < M; r0 += slice) {
    const int64_t mc = M - r0 < slice ? M - r0 : slice;
    hipLaunchKernelGGL(shrink_tiles_kernel, dim3((unsigned)((mc + kShrinkRows - 1) / kShrinkRows), kShrinkSplit), dim3(256), 0,
                       stream, X + (size_t)r0 * d1, mc, r0, d1, row_to_req ? row_to_req + r0 : nullptr, ad, site, tenant_id,
                       route, B, t + (size_t)r0 * ad.r_max, (size_t)M * ad.r_max);
    const int rc = check_launch();
    if (rc) return rc;
  }
  return MILORA_OK;
}

}  // namespace milora
