// bf16 projection GEMM for very few rows (decoding: one row per sequence, M <= 32).
//
// With so few rows the product is bound by streaming the weights once from HBM, so the kernel is laid out for
// bytes in flight rather than for tile reuse: a workgroup of 8 wavefronts owns 16 output columns (16 weight
// rows); each wavefront takes one eighth of K and walks it in 32-element steps with one 16x16x32 MFMA per
// step (operands go straight from global memory into the MFMA lane layout: lane l holds row l % 16,
// elements 8 (l / 16) .. +7 of the step); the eight partial 16x16 tiles are added through LDS in a fixed
// order and the epilogue is applied.  Rows 16..31 use a second accumulator.
#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8s;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4s;

static constexpr int kSkinnyWaves = 8;
static constexpr int kSkinnyUnroll = 4;

__device__ inline float silu_s(float x) { return x / (1.0f + __expf(-x)); }

template <bool DUAL>
__global__ void __launch_bounds__(kSkinnyWaves * 64)
gemm_skinny_kernel(const bf16* __restrict__ a, const bf16* __restrict__ w, const bf16* __restrict__ w2,
                   const bf16* __restrict__ w3, int ns1, int ns2, void* __restrict__ c, int m, int n, int k, int ldc,
                   int epi, const int* __restrict__ m_live) {
  __shared__ float part[kSkinnyWaves][4][64][4];   // [wave][tile: gate/rows 0-15, gate/16-31, up/0-15, up/16-31][lane][e]
  m = live_count(m, m_live);
  if (m <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = (int)blockIdx.x * 16;
  const int col = n0 + (lane & 15);
  const int kw = k / kSkinnyWaves;
  const size_t koff = (size_t)wave * kw + 8 * (lane >> 4);
  const bf16* pw;
  const bf16* pu = nullptr;
  if (DUAL) {
    pw = w + (size_t)col * k + koff;
    pu = w2 + (size_t)col * k + koff;
  } else {
    pw = (col < ns1 ? w + (size_t)col * k : (col < ns2 ? w2 + (size_t)(col - ns1) * k : w3 + (size_t)(col - ns2) * k)) + koff;
  }
  const bool two = m > 16;
  const bf16* pa0 = a + (size_t)min(lane & 15, m - 1) * k + koff;
  const bf16* pa1 = a + (size_t)min(16 + (lane & 15), m - 1) * k + koff;
  f32x4s g0 = {0.f, 0.f, 0.f, 0.f}, g1 = g0, u0 = g0, u1 = g0;
  for (int ks = 0; ks < kw; ks += 32 * kSkinnyUnroll) {
    bf16x8s fb[kSkinnyUnroll], fu[kSkinnyUnroll], fa0[kSkinnyUnroll], fa1[kSkinnyUnroll];
#pragma unroll
    for (int s = 0; s < kSkinnyUnroll; ++s) {
      const int o = ks + 32 * s;
      if (o < kw) {
        fb[s] = *reinterpret_cast<const bf16x8s*>(pw + o);
        if (DUAL) fu[s] = *reinterpret_cast<const bf16x8s*>(pu + o);
        fa0[s] = *reinterpret_cast<const bf16x8s*>(pa0 + o);
        if (two) fa1[s] = *reinterpret_cast<const bf16x8s*>(pa1 + o);
      }
    }
#pragma unroll
    for (int s = 0; s < kSkinnyUnroll; ++s) {
      if (ks + 32 * s < kw) {
        g0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa0[s], fb[s], g0, 0, 0, 0);
        if (two) g1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa1[s], fb[s], g1, 0, 0, 0);
        if (DUAL) {
          u0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa0[s], fu[s], u0, 0, 0, 0);
          if (two) u1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa1[s], fu[s], u1, 0, 0, 0);
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    part[wave][0][lane][e] = g0[e];
    part[wave][1][lane][e] = g1[e];
    if (DUAL) {
      part[wave][2][lane][e] = u0[e];
      part[wave][3][lane][e] = u1[e];
    }
  }
  __syncthreads();
  // wavefront 0 finishes rows 0-15, wavefront 1 rows 16-31
  if (wave > 1 || (wave == 1 && !two)) return;
  float gs[4] = {0.f, 0.f, 0.f, 0.f}, us[4] = {0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < kSkinnyWaves; ++p) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      gs[e] += part[p][wave][lane][e];
      if (DUAL) us[e] += part[p][2 + wave][lane][e];
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int row = wave * 16 + 4 * (lane >> 4) + e;
    if (row >= m) continue;
    const size_t o = (size_t)row * ldc + col;
    if (DUAL) reinterpret_cast<bf16*>(c)[o] = f32_to_bf16(silu_s(gs[e]) * us[e]);
    else if (epi == EPI_STORE_F32) reinterpret_cast<float*>(c)[o] = gs[e];
    else if (epi == EPI_ADD_F32) reinterpret_cast<float*>(c)[o] += gs[e];
    else reinterpret_cast<bf16*>(c)[o] = f32_to_bf16(gs[e]);
  }
}

bool gemm_skinny_applies(int m, int n, int k, int ns1, int ns2) {
  return m >= 1 && m <= 32 && n % 16 == 0 && k % (kSkinnyWaves * 32) == 0 && ns1 % 16 == 0 && ns2 % 16 == 0;
}

hipError_t launch_gemm_skinny_bf16(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2,
                                   void* c, int m, int n, int k, int ldc, GemmEpilogue epi, hipStream_t st,
                                   const int* m_live) {
  const dim3 grid((unsigned)(n / 16));
  if (epi == EPI_SWIGLU_T)
    gemm_skinny_kernel<true><<<grid, kSkinnyWaves * 64, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, (int)epi, m_live);
  else
    gemm_skinny_kernel<false><<<grid, kSkinnyWaves * 64, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, (int)epi, m_live);
  return hipGetLastError();
}

}  // namespace rc
