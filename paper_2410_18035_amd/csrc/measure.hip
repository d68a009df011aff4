// Measurement helpers, not part of the method: what this GPU sustains on the two resources the kernels of
// this library are bound by, so that their rates can be put beside a measured ceiling as well as the
// vendor's figures.  One kernel issues nothing but bf16 matrix-core instructions on independent
// accumulators; the other reads a buffer once with 16-byte loads.
#include "common.h"

namespace milora {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kAccs = 32;

// Operand values: small integers (few bits change between lanes and elements), or, with `mixed`, values spread
// over [-1, 1) with every mantissa bit in use - what weights and activations look like, and what the matrix cores
// draw more power for.
__device__ __forceinline__ void rate_operands(bf16x8& a, bf16x8& b, int mixed) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (mixed) {
      const uint32_t ha = (threadIdx.x * 8u + i + 1u) * 2654435761u, hb = (threadIdx.x * 8u + i + 77u) * 2246822519u;
      a[i] = (__bf16)((float)(int)(ha >> 8) * (1.0f / 8388608.0f) - 1.0f);
      b[i] = (__bf16)((float)(int)(hb >> 8) * (1.0f / 8388608.0f) - 1.0f);
    } else {
      a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
      b[i] = (__bf16)(float)(i & 1);
    }
  }
}

__global__ void __launch_bounds__(256, 1) mfma_rate_kernel(float* out, int iters, int mixed) {
  f32x4 acc[kAccs];
#pragma unroll
  for (int i = 0; i < kAccs; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 a, b;
  rate_operands(a, b, mixed);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kAccs; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < kAccs; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, a, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kAccs; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kAccs32 = 8;

// The same with v_mfma_f32_32x32x16_bf16: twice the flops per instruction and per operand register read.
__global__ void __launch_bounds__(256, 1) mfma32_rate_kernel(float* out, int iters, int mixed) {
  f32x16 acc[kAccs32];
#pragma unroll
  for (int i = 0; i < kAccs32; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a, b;
  rate_operands(a, b, mixed);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
      for (int i = 0; i < kAccs32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < kAccs32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[i], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kAccs32; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int kReadUnroll>
__global__ void __launch_bounds__(256) read_rate_kernel(const u32x4* __restrict__ buf, size_t n16, uint32_t* out) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t s = 0;
  for (; i + (kReadUnroll - 1) * stride < n16; i += kReadUnroll * stride) {
    u32x4 v[kReadUnroll];
#pragma unroll
    for (int u = 0; u < kReadUnroll; ++u) v[u] = __builtin_nontemporal_load(buf + i + u * stride);
#pragma unroll
    for (int u = 0; u < kReadUnroll; ++u) s ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(buf + i);
    s ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (s == 0x9e3779b9u) out[0] = s;  // keeps the loads alive; practically never taken
}

}  // namespace
}  // namespace milora

using namespace milora;

extern "C" size_t milora_measure_workspace_bytes(void) { return (size_t)1024 * 256 * sizeof(float); }

extern "C" int milora_measure_matrix_rate(int shape, int iters, void* workspace, size_t workspace_bytes, double* tflops,
                                        void* stream) {
  if (iters < 1 || !tflops || shape < 0 || shape > 3) return MILORA_EINVAL;
  const int mixed = shape >> 1;
  shape &= 1;
  if (!workspace || workspace_bytes < milora_measure_workspace_bytes()) return MILORA_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, cus = 0;
  MILORA_HIP(hipGetDevice(&dev));
  MILORA_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int grid = cus < 1 ? 256 : (cus > 512 ? 1024 : 2 * cus);
  hipEvent_t e0, e1;
  MILORA_HIP(hipEventCreate(&e0));
  MILORA_HIP(hipEventCreate(&e1));
  auto* kernel = shape == 0 ? mfma_rate_kernel : mfma32_rate_kernel;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, (float*)workspace, iters < 64 ? iters : 64, mixed);
  (void)hipEventRecord(e0, st);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, (float*)workspace, iters, mixed);
  (void)hipEventRecord(e1, st);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_fail(e);
  // both kernels issue 64 instructions' worth of 16x16x32 per wave and iteration: 32 of twice the size in the second
  const double flops = (double)grid * 4.0 * (double)iters * (2.0 * kAccs) * (2.0 * 16 * 16 * 32);
  static_assert(2 * 2 * kAccs32 * 32 * 32 * 16 == 2 * kAccs * 16 * 16 * 32, "same flops per iteration");
  *tflops = flops / ((double)ms * 1e-3) / 1e12;
  return check_launch();
}

namespace {
template <int U>
int time_read(const void* buf, size_t n16, int reps, int grid, void* workspace, hipStream_t st, double* gbs) {
  hipEvent_t e0, e1;
  MILORA_HIP(hipEventCreate(&e0));
  MILORA_HIP(hipEventCreate(&e1));
  hipLaunchKernelGGL(read_rate_kernel<U>, dim3(grid), dim3(256), 0, st, (const u32x4*)buf, n16, (uint32_t*)workspace);
  (void)hipEventRecord(e0, st);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(read_rate_kernel<U>, dim3(grid), dim3(256), 0, st, (const u32x4*)buf, n16, (uint32_t*)workspace);
  (void)hipEventRecord(e1, st);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_fail(e);
  *gbs = (double)(n16 * 16) * reps / ((double)ms * 1e-3) / 1e9;
  return check_launch();
}
}  // namespace

extern "C" int milora_measure_read_rate(const void* buf, size_t bytes, int reps, void* workspace, size_t workspace_bytes,
                                        double* gbs, void* stream) {
  if (!buf || bytes < 16 || reps < 1 || !gbs || ((uintptr_t)buf & 15) != 0) return MILORA_EINVAL;
  if (!workspace || workspace_bytes < milora_measure_workspace_bytes()) return MILORA_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const size_t n16 = bytes / 16;
  // the best of a few launch shapes (workgroups per launch x loads in flight per thread)
  double best = 0.0;
  for (int grid = 1024; grid <= 8192; grid *= 2) {
    double g8 = 0.0, g16 = 0.0;
    int rc = time_read<8>(buf, n16, reps, grid, workspace, st, &g8);
    if (rc) return rc;
    rc = time_read<16>(buf, n16, reps, grid, workspace, st, &g16);
    if (rc) return rc;
    best = g8 > best ? g8 : best;
    best = g16 > best ? g16 : best;
  }
  *gbs = best;
  return MILORA_OK;
}
