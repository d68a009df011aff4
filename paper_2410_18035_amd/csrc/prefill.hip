// Many-row (prefill) routed LoRA linear on row-major bf16 weights (paper Eq. 1 with the layer-level gate of
// Sec. 3.3): Y = X W^T + bias + (X W^A) W^B for the rows whose request is routed to this site.
//
// One workgroup of four waves computes a 256 x 256 tile of Y with the bf16 matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulators, 128 x 128 per wave).  X and W are both contiguous along the
// reduction index, so a 16-row x 32-k block of either is what one matrix-core operand takes; the blocks are
// copied from global memory straight into LDS (global_load_lds_dwordx4, no registers) in that operand order,
// four k steps deep (4 x 32 KB), and read back with one conflict-free 16-byte LDS load per lane and block.
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

constexpr int kTM = 256, kTN = 256, kTK = 32;
constexpr int kStages = 4;
constexpr int kThreadsP = 256;
constexpr int kBlocksM = kTM / 16, kBlocksN = kTN / 16;
constexpr int kStageBytes = (kBlocksM + kBlocksN) * 1024;
constexpr int kCtlBytes = 1024;
constexpr int kLdsBytesP = kStages * kStageBytes + kCtlBytes;
constexpr int kAccTilesRows = 6;
constexpr int kGroupM = 8;  // consecutive workgroups of an XCD walk 8 row tiles of one column tile

struct PParams {
  const bf16_t* X;
  const bf16_t* W;
  const bf16_t* bias;
  bf16_t* Y;
  const float* t;
  const int32_t* row_to_req;
  const int32_t* tenant_id;
  const uint8_t* route;
  AdapterView ad;
  int64_t M;
  int d1, d2, site, B;
  int tilesM, tilesN;
};

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

// One k step of 32 for the wave's 128 x 128 part: operand blocks from LDS, 64 matrix-core instructions.
__device__ __forceinline__ void mma_step(const unsigned char* sa, const unsigned char* sb, f32x4 (&acc)[8][8]) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = *(const bf16x8*)(sa + i * 1024);
#pragma unroll
  for (int j = 0; j < 8; ++j) b[j] = *(const bf16x8*)(sb + j * 1024);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
}

__global__ void __launch_bounds__(kThreadsP, 1) prefill_kernel(PParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  // workgroup -> tile: workgroup ids go round-robin over the 8 XCDs; each XCD takes a contiguous run of the
  // tile order, which walks kGroupM row tiles per column tile so that the XCD's L2 serves the re-reads
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

  // copies: waves 0,1 bring the 16 row blocks of X, waves 2,3 the 16 row blocks of W, 8 blocks each per k step
  const bool is_w = wave >= 2;
  const unsigned char* src = is_w ? (const unsigned char*)p.W : (const unsigned char*)p.X;
  const int64_t row0 = is_w ? (int64_t)n0 : m0;
  const int64_t rlim = is_w ? (int64_t)p.d2 : p.M;
  uint32_t voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    // four consecutive lanes take the 64 bytes of one row (coalesced); which 16 of them a lane takes is
    // permuted by the row so that the operand reads below spread over all LDS banks
    const int rr = lane >> 2;
    int64_t r = row0 + ((wave & 1) * 8 + j) * 16 + rr;
    r = r < rlim ? r : rlim - 1;
    voff[j] = (uint32_t)((uint64_t)r * (uint32_t)p.d1 * 2u + (uint32_t)((lane & 3) ^ ((rr >> 1) & 3)) * 16u);
  }
  auto issue = [&](int kt, int slot) __attribute__((always_inline)) {
    const int kk = kt < KT ? kt : KT - 1;  // past the end: re-read the last step into a slot nobody reads
    const unsigned char* b = src + (size_t)kk * (kTK * 2);
    const uint32_t dst = lds0 + slot * kStageBytes + (wave * 8) * 1024;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      copy_to_lds(b, voff[j], dst + j * 1024);
    }
  };

  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // operand read: lane l takes row l % 16, k group l / 16 of a block stored as 16 rows x 64 bytes
  const int rd_off = (lane & 15) * 64 + (((lane >> 4) ^ ((lane >> 1) & 3)) << 4);
  const unsigned char* sa0 = lds + (wm * 8) * 1024 + rd_off;
  const unsigned char* sb0 = lds + (kBlocksM + wn * 8) * 1024 + rd_off;

  issue(0, 0);
  issue(1, 1);
  issue(2, 2);
  auto step = [&](int kt, int slot) __attribute__((always_inline)) {
    wait_vm<16>();                  // this wave's copies of step kt have landed
    __builtin_amdgcn_s_barrier();   // so have the other waves'; and all waves are done reading step kt-1
    asm volatile("" ::: "memory");
    issue(kt + 3, (slot + 3) & 3);
    mma_step(sa0 + slot * kStageBytes, sb0 + slot * kStageBytes, acc);
    asm volatile("" ::: "memory");
  };
  // 48 of the 64 accumulator tiles in the accumulation registers, 16 in ordinary ones: with all 256 in the
  // accumulation file the compiler has no spare tile there and shuffles tiles between the files in the loop
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (i < kAccTilesRows) asm volatile("" : "+a"(acc[i][j]));
      else asm volatile("" : "+v"(acc[i][j]));
    }
  int kt = 0;
  for (; kt + 4 <= KT; kt += 4) {
    step(kt, 0);
    step(kt + 1, 1);
    step(kt + 2, 2);
    step(kt + 3, 3);
  }
  for (int s = 0; kt < KT; ++kt, ++s) step(kt, s);
  wait_vm<0>();
  __syncthreads();

  // ---- LoRA term of the routed rows as extra k steps ---------------------------------------------------
  int* ctl = (int*)(lds + kStages * kStageBytes);
  int my_ten = -1;
  {
    const int64_t m = m0 + tid;
    if (m < p.M) {
      const int64_t req = p.row_to_req ? (int64_t)p.row_to_req[m] : m;
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
    const bf16_t* Bm = (const bf16_t*)p.ad.B[cur * MILORA_NUM_SITES + p.site];
    const int64_t m = m0 + tid;
    const int n = n0 + tid;
    for (int c0 = 0; c0 < r; c0 += 32) {
      const uint32_t blk = (uint32_t)(tid >> 4) * 1024 + (uint32_t)(tid & 15) * 64;
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
            tv[h] = (my_ten == cur && c < r) ? p.t[(size_t)m * p.ad.r_max + c] : 0.f;
            bw[h] = (c < r && n < p.d2) ? (uint32_t)Bm[(size_t)c * p.d2 + n] : 0u;
          }
          const bf16_t h0 = f32_to_bf16(tv[0]), h1 = f32_to_bf16(tv[1]);
          hi[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
          lo[e] = pack_bf16x2(tv[0] - bf16_to_f32(h0), tv[1] - bf16_to_f32(h1));
          wb[e] = bw[0] | (bw[1] << 16);
        }
        const uint32_t o = blk + ((g ^ ((tid >> 1) & 3)) << 4);
        *(u32x4*)(lds + o) = hi;                              // slot 0, X side
        *(u32x4*)(lds + kStageBytes + o) = lo;                // slot 1, X side
        *(u32x4*)(lds + kBlocksM * 1024 + o) = wb;            // slot 0, W side
        *(u32x4*)(lds + kStageBytes + kBlocksM * 1024 + o) = wb;  // slot 1, W side
      }
      __syncthreads();
      mma_step(sa0, sb0, acc);
      mma_step(sa0 + kStageBytes, sb0 + kStageBytes, acc);
      __syncthreads();
    }
    last = cur;
  }

  // ---- bias, one rounding, store: a lane holds 4 consecutive columns of one row per 16 x 16 tile ----------
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int n = n0 + wn * 128 + j * 16 + (lane >> 4) * 4;
    if (n >= p.d2) continue;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) {
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[e] = bf16_to_f32(p.bias[n + e]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t m = m0 + wm * 128 + i * 16 + (lane & 15);
      if (m >= p.M) continue;
      u32x2 v;
      v[0] = pack_bf16x2(acc[i][j][0] + bv[0], acc[i][j][1] + bv[1]);
      v[1] = pack_bf16x2(acc[i][j][2] + bv[2], acc[i][j][3] + bv[3]);
      *(u32x2*)(p.Y + (size_t)m * p.d2 + n) = v;
    }
  }
}

}  // namespace

bool prefill_supported(int64_t M, int d1, int d2, const void* X, const void* W, const void* Y) {
  if (M < 64 || d1 % kTK != 0 || d2 % 16 != 0) return false;
  if ((((uintptr_t)X | (uintptr_t)W) & 15) != 0 || ((uintptr_t)Y & 7) != 0) return false;
  const uint64_t rows = (uint64_t)(M > d2 ? M : d2);
  if (rows * (uint64_t)d1 * 2u >= (1ull << 32)) return false;  // 32-bit byte offsets inside X and W
  const int64_t tiles = ((M + kTM - 1) / kTM) * ((d2 + kTN - 1) / kTN);
  return tiles < (1 << 28);
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
  PParams p;
  p.X = X; p.W = W; p.bias = bias; p.Y = Y; p.t = t;
  p.row_to_req = row_to_req; p.tenant_id = tenant_id; p.route = route; p.ad = ad;
  p.M = M; p.d1 = d1; p.d2 = d2; p.site = site; p.B = B;
  p.tilesM = (int)((M + kTM - 1) / kTM);
  p.tilesN = (d2 + kTN - 1) / kTN;
  const int total = p.tilesM * p.tilesN;
  const int per = (total + 7) / 8;
  hipLaunchKernelGGL(prefill_kernel, dim3(8 * per), dim3(kThreadsP), kLdsBytesP, stream, p);
  return check_launch();
}

}  // namespace milora
