// Any-shape, any-dtype routed LoRA linear (paper Eq. 1 with the layer-level gate of Sec. 3.3).
// This is the path for fp32 tensors, row-major weights with unaligned sizes and for whatever the
// matrix-core kernels do not cover.  Two kernels: the LoRA shrink t = x W^A for routed rows, and a
// tiled fp32 GEMM whose epilogue adds bias and t W^B before the single rounding to the output type.
#include "common.h"

namespace milora {

namespace {

constexpr int kThreads = 256;

// One workgroup per row m: t[m][c] = sum_k X[m][k] * A[k][c], c < r.  Threads are laid out with the
// rank index fastest (coalesced reads of A's rows); the k-lanes are summed through LDS in a fixed order.
template <typename T>
__global__ void __launch_bounds__(kThreads) shrink_rows_kernel(const T* __restrict__ X, int64_t M, int d1,
                                                               const int32_t* __restrict__ row_to_req, AdapterView ad,
                                                               int site, const int32_t* __restrict__ tenant_id,
                                                               const uint8_t* __restrict__ route, int B,
                                                               float* __restrict__ t) {
  __shared__ float red[kThreads];
  const int64_t m = blockIdx.x;
  const int64_t req = row_to_req ? (int64_t)row_to_req[m] : m;
  int tenant = 0;
  const int r = (req >= 0 && req < B) ? routed_rank(ad, tenant_id, route, (int)req, B, site, &tenant) : 0;
  if (r == 0) return;
  const T* A = (const T*)ad.A[tenant * MILORA_NUM_SITES + site];
  int rpad = 1;
  while (rpad < r) rpad <<= 1;
  const int c = threadIdx.x % rpad, krow = threadIdx.x / rpad, rpp = kThreads / rpad;
  float acc = 0.f;
  if (c < r)
    for (int k = krow; k < d1; k += rpp) acc += Elem<T>::load(X, (size_t)m * d1 + k) * Elem<T>::load(A, (size_t)k * r + c);
  red[threadIdx.x] = acc;
  __syncthreads();
  if (krow == 0 && c < r) {
    float s = 0.f;
    for (int j = 0; j < rpp; ++j) s += red[j * rpad + c];
    t[(size_t)m * ad.r_max + c] = s;
  }
}

// 64x64 output tile per workgroup, 16-deep k slices through LDS, 4x4 outputs per thread, fp32 FMA.
// W is row-major [d2][d1].  Epilogue: + bias, + t[m] . B for rows that carry a LoRA term at `site`.
template <typename T>
__global__ void __launch_bounds__(kThreads) linear_tile_kernel(const T* __restrict__ X, int64_t M, int d1, int d2,
                                                               const int32_t* __restrict__ row_to_req,
                                                               const T* __restrict__ W, const T* __restrict__ bias,
                                                               AdapterView ad, int site,
                                                               const int32_t* __restrict__ tenant_id,
                                                               const uint8_t* __restrict__ route, int B,
                                                               const float* __restrict__ t, T* __restrict__ Y) {
  constexpr int TM = 64, TN = 64, TK = 16;
  __shared__ float xs[TK][TM + 1];
  __shared__ float ws[TK][TN + 1];
  const int64_t m0 = (int64_t)blockIdx.y * TM;
  const int n0 = blockIdx.x * TN;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < d1; k0 += TK) {
    // 64 rows x 16 k of X and of W: 1024 elements each, 4 per thread, k fastest (contiguous in memory)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = threadIdx.x + e * kThreads;
      const int kk = idx % TK, rr = idx / TK;
      const int k = k0 + kk;
      const int64_t m = m0 + rr;
      const int n = n0 + rr;
      xs[kk][rr] = (m < M && k < d1) ? Elem<T>::load(X, (size_t)m * d1 + k) : 0.f;
      ws[kk][rr] = (n < d2 && k < d1) ? Elem<T>::load(W, (size_t)n * d1 + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = xs[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
    const int64_t req = row_to_req ? (int64_t)row_to_req[m] : m;
    int tenant = 0;
    const int r = (req >= 0 && req < B) ? routed_rank(ad, tenant_id, route, (int)req, B, site, &tenant) : 0;
    const T* Bm = r ? (const T*)ad.B[tenant * MILORA_NUM_SITES + site] : nullptr;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= d2) continue;
      float v = acc[i][j];
      if (bias) v += Elem<T>::load(bias, n);
      if (r) {
        float delta = 0.f;
        for (int c = 0; c < r; ++c) delta += t[(size_t)m * ad.r_max + c] * Elem<T>::load(Bm, (size_t)c * d2 + n);
        v += delta;
      }
      Elem<T>::store(Y, (size_t)m * d2 + n, v);
    }
  }
}

}  // namespace

int launch_shrink(const void* X, int64_t M, int d1, int dtype, const int32_t* row_to_req, const AdapterView& ad,
                  int site, const int32_t* tenant_id, const uint8_t* route, int B, float* t, hipStream_t stream) {
  if (dtype == MILORA_BF16)
    hipLaunchKernelGGL((shrink_rows_kernel<bf16_t>), dim3((unsigned)M), dim3(kThreads), 0, stream, (const bf16_t*)X, M,
                       d1, row_to_req, ad, site, tenant_id, route, B, t);
  else
    hipLaunchKernelGGL((shrink_rows_kernel<float>), dim3((unsigned)M), dim3(kThreads), 0, stream, (const float*)X, M,
                       d1, row_to_req, ad, site, tenant_id, route, B, t);
  return check_launch();
}

int launch_linear_generic(const void* X, int64_t M, int d1, int d2, int dtype, const int32_t* row_to_req,
                          const void* W, const void* bias, const AdapterView& ad, int site,
                          const int32_t* tenant_id, const uint8_t* route, int B, const float* t, void* Y,
                          hipStream_t stream) {
  dim3 grid((unsigned)((d2 + 63) / 64), (unsigned)((M + 63) / 64));
  if (grid.y > 65535) return MILORA_ERANGE;
  if (dtype == MILORA_BF16)
    hipLaunchKernelGGL((linear_tile_kernel<bf16_t>), grid, dim3(kThreads), 0, stream, (const bf16_t*)X, M, d1, d2,
                       row_to_req, (const bf16_t*)W, (const bf16_t*)bias, ad, site, tenant_id, route, B, t,
                       (bf16_t*)Y);
  else
    hipLaunchKernelGGL((linear_tile_kernel<float>), grid, dim3(kThreads), 0, stream, (const float*)X, M, d1, d2,
                       row_to_req, (const float*)W, (const float*)bias, ad, site, tenant_id, route, B, t, (float*)Y);
  return check_launch();
}

}  // namespace milora
