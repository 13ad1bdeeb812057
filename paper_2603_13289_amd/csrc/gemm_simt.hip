// Projection GEMM for the float configuration: C[M][N] = A[M][K] * W[N][K]^T on the vector ALUs,
// 64x64 output tile per workgroup, 4x4 outputs per thread, float accumulation.
// (bf16 models run on the matrix cores instead: gemm_mfma.hip.)
#include "common.h"

namespace rc {

static constexpr int BM = 64, BN = 64, BK = 16, PAD = 4;

__device__ inline float silu_f(float x) { return x / (1.0f + __expf(-x)); }

template <typename T, bool DUAL>
__global__ void __launch_bounds__(256)
gemm_simt_kernel(const T* __restrict__ a, const T* __restrict__ w, const T* __restrict__ w2, void* __restrict__ c,
                 int m, int n, int k, int ldc, int epi, const int* __restrict__ m_live) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int LPR = BK / VEC;  // 16-byte loads per tile row
  m = live_count(m, m_live);
  if ((int)blockIdx.y * BM >= m) return;   // uniform: the grid may be sized for an upper bound of the row count
  __shared__ float As[BK][BM + PAD];
  __shared__ float Bs[BK][BN + PAD];
  __shared__ float Bs2[DUAL ? BK : 1][BN + PAD];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  float acc[4][4] = {}, acc2[4][4] = {};
  const int lrow = tid / LPR, lk = (tid % LPR) * VEC;
  const bool loader = tid < BM * LPR;
  for (int k0 = 0; k0 < k; k0 += BK) {
    if (loader) {
      float va[VEC], vb[VEC], vb2[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) va[e] = vb[e] = vb2[e] = 0.f;
      const bool kin = k0 + lk < k;
      if (kin && m0 + lrow < m) Vec16<T>::load(a + (size_t)(m0 + lrow) * k + k0 + lk, va);
      if (kin && n0 + lrow < n) {
        Vec16<T>::load(w + (size_t)(n0 + lrow) * k + k0 + lk, vb);
        if (DUAL) Vec16<T>::load(w2 + (size_t)(n0 + lrow) * k + k0 + lk, vb2);
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        As[lk + e][lrow] = va[e];
        Bs[lk + e][lrow] = vb[e];
        if (DUAL) Bs2[lk + e][lrow] = vb2[e];
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const float4 av = *reinterpret_cast<const float4*>(&As[kk][ty * 4]);
      const float4 bv = *reinterpret_cast<const float4*>(&Bs[kk][tx * 4]);
      const float ar[4] = {av.x, av.y, av.z, av.w}, br[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], br[j], acc[i][j]);
      if (DUAL) {
        const float4 b2 = *reinterpret_cast<const float4*>(&Bs2[kk][tx * 4]);
        const float b2r[4] = {b2.x, b2.y, b2.z, b2.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc2[i][j] = fmaf(ar[i], b2r[j], acc2[i][j]);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= m) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= n) continue;
      const size_t o = (size_t)row * ldc + col;
      if (epi == EPI_STORE_F32) reinterpret_cast<float*>(c)[o] = acc[i][j];
      else if (epi == EPI_ADD_F32) reinterpret_cast<float*>(c)[o] += acc[i][j];
      else if (epi == EPI_STORE_T) reinterpret_cast<T*>(c)[o] = from_f32<T>(acc[i][j]);
      else reinterpret_cast<T*>(c)[o] = from_f32<T>(silu_f(acc[i][j]) * acc2[i][j]);
    }
  }
}

template <typename T>
hipError_t launch_gemm_simt(const T* a, const T* w, const T* w2, void* c, int m, int n, int k, int ldc,
                            GemmEpilogue epi, hipStream_t st, const int* m_live) {
  if (m <= 0 || n <= 0) return hipSuccess;
  dim3 grid((unsigned)((n + BN - 1) / BN), (unsigned)((m + BM - 1) / BM));
  if (epi == EPI_SWIGLU_T)
    gemm_simt_kernel<T, true><<<grid, 256, 0, st>>>(a, w, w2, c, m, n, k, ldc, (int)epi, m_live);
  else
    gemm_simt_kernel<T, false><<<grid, 256, 0, st>>>(a, w, w2, c, m, n, k, ldc, (int)epi, m_live);
  return hipGetLastError();
}

template <>
hipError_t launch_gemm<float>(const float* a, const float* w, const float* w2, void* c, int m, int n, int k,
                              int ldc, GemmEpilogue epi, hipStream_t st, const int* m_live) {
  return launch_gemm_simt<float>(a, w, w2, c, m, n, k, ldc, epi, st, m_live);
}

template <>
hipError_t launch_gemm_qkv<float>(const float* a, const float* wq, int nq, const float* wk, const float* wv, int nkv,
                                  float* c, int m, int k, hipStream_t st, const int* m_live) {
  const int n = nq + 2 * nkv;
  hipError_t e = launch_gemm_simt<float>(a, wq, nullptr, c, m, nq, k, n, EPI_STORE_F32, st, m_live);
  if (e != hipSuccess) return e;
  e = launch_gemm_simt<float>(a, wk, nullptr, c + nq, m, nkv, k, n, EPI_STORE_F32, st, m_live);
  if (e != hipSuccess) return e;
  return launch_gemm_simt<float>(a, wv, nullptr, c + nq + nkv, m, nkv, k, n, EPI_STORE_F32, st, m_live);
}

}  // namespace rc
