// Two micro-benchmarks that put the measured kernels next to what this very GPU sustains (boards differ, and
// the chip lowers its clock under matrix load):
//   stream copy      16-byte loads and stores over a large buffer: the HBM rate a memory-bound kernel can reach
//   MFMA loop        back-to-back 16x16x32 bf16 MFMAs on register operands (no LDS, no memory): the matrix rate
//                    the chip sustains under its power limit, the practical ceiling of any bf16 GEMM here
#include <algorithm>

#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

// a workgroup moves contiguous 16 KB pieces, four 16-byte loads in flight per lane before the first store
__global__ void __launch_bounds__(256)
stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  const size_t n_pieces = n16 / 1024;
  for (size_t p = blockIdx.x; p < n_pieces; p += gridDim.x) {
    const size_t i = p * 1024 + threadIdx.x;
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256);
    const u32x4 c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + 256);
    __builtin_nontemporal_store(c, dst + i + 512);
    __builtin_nontemporal_store(d, dst + i + 768);
  }
  for (size_t i = n_pieces * 1024 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// operands with random signs and mantissas, magnitudes below 1 (what normalised activations and weights look like;
// the sustained clock depends on how much the operand bits toggle)
__device__ inline bf16x8 pseudo_random_operand(unsigned s) {
  bf16x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    s = s * 1664525u + 1013904223u;
    v[i] = (__bf16)(((int)(s >> 16) % 2001 - 1000) * 0.001f);
  }
  return v;
}

static constexpr int kLoopWaves = 8;          // per workgroup, two per SIMD as in the GEMM kernel
static constexpr int kMfmaPerIter = 32;       // a 64 x 128 x 32 wavefront sub-tile step

__global__ void __launch_bounds__(64 * kLoopWaves, 1)
mfma_loop_kernel(float* __restrict__ out, int iters) {
  bf16x8 a[4], b[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = pseudo_random_operand(threadIdx.x * 17 + i + blockIdx.x);
#pragma unroll
  for (int j = 0; j < 8; ++j) b[j] = pseudo_random_operand(threadIdx.x * 31 + j + 7 * blockIdx.x);
  f32x4 acc[4][8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;   // keeps the loop alive
}

hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  const unsigned blocks = (unsigned)std::min<size_t>((n16 + 1023) / 1024, 256 * 16);
  stream_copy_kernel<<<blocks, 256, 0, st>>>(reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

size_t mfma_loop_out_floats(int n_workgroups) { return (size_t)n_workgroups * 64 * kLoopWaves; }
double mfma_loop_flops(int n_workgroups, int iters) {
  return (double)n_workgroups * kLoopWaves * iters * kMfmaPerIter * (2.0 * 16 * 16 * 32);
}
hipError_t launch_mfma_loop(float* out, int n_workgroups, int iters, hipStream_t st) {
  mfma_loop_kernel<<<n_workgroups, 64 * kLoopWaves, 0, st>>>(out, iters);
  return hipGetLastError();
}

}  // namespace rc
