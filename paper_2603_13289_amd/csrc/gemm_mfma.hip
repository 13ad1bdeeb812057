// K3: projection GEMMs of the active rows on the matrix cores (bf16 in, float accumulate).
//
//   C[M][N] (op)= A[M][K] * W[N][K]^T        A: compact activation rows, W: weights [out][in]
//
// Both operands are K-contiguous, which is exactly what the MFMA operand registers want (8
// consecutive k per lane), so tiles go global -> LDS -> registers without any transpose.
//
// Workgroup tile BM x BN, K step 64.  LDS holds one A tile [BM][64] and one B tile [BN][64] as rows of
// eight 16-byte chunks; chunk c of row r is stored at slot c ^ ((r >> 1) & 7).  With 64 LDS banks of
// 4 bytes a 128-byte row covers half the banks, so 16 lanes reading the same chunk of 16 consecutive
// rows (one MFMA operand fetch) touch 16 different (row parity, slot) pairs = all 64 banks once, and
// the row-contiguous fill is conflict free as well.  No padding is needed.
// The next K step is fetched into registers while the current one is multiplied.
// Each wavefront owns a (BM/WAVES_M) x (BN/WAVES_N) sub-tile built from 32x32x16 MFMA blocks.
//
// SwiGLU epilogue (DUAL): the B tile stacks BN/2 rows of W_gate on BN/2 rows of W_up for the same
// output columns, every wavefront holds matching gate/up accumulators and writes silu(gate)*up.
//
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids congruent mod 8) walk
// all row tiles of the same few weight-column tiles: a weight tile is then fetched from HBM once
// per XCD-L2 instead of once per row tile.
#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int BK = 64;
static constexpr int XCDS = 8;

__device__ inline float silu_mf(float x) { return x / (1.0f + __expf(-x)); }

template <int BM, int BN, int WAVES_M, int WAVES_N, bool DUAL, int OCC>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64, OCC)
gemm_mfma_kernel(const bf16* __restrict__ a, const bf16* __restrict__ w, const bf16* __restrict__ w2,
                 const bf16* __restrict__ w3, int ns1, int ns2, void* __restrict__ c, int m, int n, int k, int ldc,
                 int epi, int tiles_m, int total_tiles, int per_xcd) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int A_PER = BM * 8 / NT, B_PER = BN * 8 / NT;
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  static_assert(A_PER * NT == BM * 8 && B_PER * NT == BN * 8, "tile/threads mismatch");
  static_assert(!DUAL || (FN % 2 == 0), "dual tiles need an even number of column fragments");

  __shared__ uint4 lds_a[BM * 8];
  __shared__ uint4 lds_b[BN * 8];

  const int logical = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
  if (logical >= total_tiles) return;
  const int tile_m = logical % tiles_m, tile_n = logical / tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN_OUT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // per-thread global sources of the tile fill: chunk (row, ch) with row = idx / 8, ch = idx % 8
  const bf16* pa[A_PER];
  const bf16* pb[B_PER];
  const int ch = tid & 7;
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int row = (tid + i * NT) >> 3;
    pa[i] = (m0 + row < m) ? a + (size_t)(m0 + row) * k + ch * 8 : nullptr;
  }
#pragma unroll
  for (int i = 0; i < B_PER; ++i) {
    const int row = (tid + i * NT) >> 3;
    if (DUAL) {
      const int half = row >= BN / 2;
      const int col = n0 + row - half * (BN / 2);
      pb[i] = (col < n) ? (half ? w2 : w) + (size_t)col * k + ch * 8 : nullptr;
    } else {
      // output columns [0, ns1) come from w, [ns1, ns2) from w2, [ns2, n) from w3 (fused q|k|v projection)
      const int col = n0 + row;
      const bf16* src = col < ns1 ? w + (size_t)col * k : (col < ns2 ? w2 + (size_t)(col - ns1) * k
                                                                     : w3 + (size_t)(col - ns2) * k);
      pb[i] = (col < n) ? src + ch * 8 : nullptr;
    }
  }

  uint4 ra[A_PER], rb[B_PER];
  auto fetch = [&](int k0) {
    const bool kin = k0 + ch * 8 < k;
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      ra[i] = (pa[i] && kin) ? *reinterpret_cast<const uint4*>(pa[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      rb[i] = (pb[i] && kin) ? *reinterpret_cast<const uint4*>(pb[i] + k0) : make_uint4(0, 0, 0, 0);
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // LDS rows this lane reads its MFMA operands from
  int arow[FM], brow[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) arow[i] = wm * WTM + i * 32 + (lane & 31);
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    if (DUAL) brow[j] = (j < FN / 2 ? wn * (WTN / 2) + j * 32 : BN / 2 + wn * (WTN / 2) + (j - FN / 2) * 32) + (lane & 31);
    else brow[j] = wn * WTN + j * 32 + (lane & 31);
  }
  const int khalf = lane >> 5;

  fetch(0);
  for (int k0 = 0; k0 < k; k0 += BK) {
    __syncthreads();   // everyone is done reading the previous tile
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      const int row = (tid + i * NT) >> 3;
      lds_a[row * 8 + (ch ^ ((row >> 1) & 7))] = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      const int row = (tid + i * NT) >> 3;
      lds_b[row * 8 + (ch ^ ((row >> 1) & 7))] = rb[i];
    }
    __syncthreads();
    if (k0 + BK < k) fetch(k0 + BK);
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      bf16x8 fa[FM], fb[FN];
      const int chunk = 2 * s + khalf;
#pragma unroll
      for (int i = 0; i < FM; ++i)
        fa[i] = __builtin_bit_cast(bf16x8, lds_a[arow[i] * 8 + (chunk ^ ((arow[i] >> 1) & 7))]);
#pragma unroll
      for (int j = 0; j < FN; ++j)
        fb[j] = __builtin_bit_cast(bf16x8, lds_b[brow[j] * 8 + (chunk ^ ((brow[j] >> 1) & 7))]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: accumulator element e of a 32x32 block sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
  constexpr int FN_OUT = DUAL ? FN / 2 : FN;
  constexpr int WTN_OUT = DUAL ? WTN / 2 : WTN;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN_OUT; ++j) {
      const int col = n0 + wn * WTN_OUT + j * 32 + (lane & 31);
      if (col >= n) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm * WTM + i * 32 + 8 * (e / 4) + 4 * khalf + (e % 4);
        if (row >= m) continue;
        const size_t o = (size_t)row * ldc + col;
        const float v = acc[i][j][e];
        if (DUAL) {
          reinterpret_cast<bf16*>(c)[o] = f32_to_bf16(silu_mf(v) * acc[i][j + FN_OUT][e]);
        } else if (epi == EPI_STORE_F32) {
          reinterpret_cast<float*>(c)[o] = v;
        } else if (epi == EPI_ADD_F32) {
          reinterpret_cast<float*>(c)[o] += v;
        } else {
          reinterpret_cast<bf16*>(c)[o] = f32_to_bf16(v);
        }
      }
    }
  }
}

static int g_gemm_tile = 0;   // 0: choose by shape; 1: 128x256; 2: 256x256; 3: 128x128
void set_gemm_tile(int t) { g_gemm_tile = t; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int OCC>
static hipError_t launch_cfg(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2, void* c,
                             int m, int n, int k, int ldc, GemmEpilogue epi, hipStream_t st) {
  const bool dual = epi == EPI_SWIGLU_T;
  const int bn_out = dual ? BN / 2 : BN;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + bn_out - 1) / bn_out;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + XCDS - 1) / XCDS;
  const dim3 grid((unsigned)(per_xcd * XCDS));
  constexpr int NT = WAVES_M * WAVES_N * 64;
  if (dual)
    gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, true, OCC><<<grid, NT, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc,
                                                                              (int)epi, tiles_m, total, per_xcd);
  else
    gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, false, OCC><<<grid, NT, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc,
                                                                               (int)epi, tiles_m, total, per_xcd);
  return hipGetLastError();
}

static hipError_t dispatch(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2, void* c,
                           int m, int n, int k, int ldc, GemmEpilogue epi, hipStream_t st) {
  if (m <= 0 || n <= 0) return hipSuccess;
  int tile = g_gemm_tile;
  if (tile == 0) {
    // enough 128x256 tiles to fill the chip twice over -> big tiles; otherwise smaller ones
    const int bn_out = epi == EPI_SWIGLU_T ? 128 : 256;
    const long t1 = (long)((m + 127) / 128) * ((n + bn_out - 1) / bn_out);
    tile = t1 >= 400 ? 1 : 3;
  }
  switch (tile) {
    case 2: return launch_cfg<256, 256, 4, 2, 1>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st);
    case 3: return launch_cfg<128, 128, 2, 2, 2>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st);
    default: return launch_cfg<128, 256, 2, 2, 2>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st);
  }
}

template <>
hipError_t launch_gemm<bf16>(const bf16* a, const bf16* w, const bf16* w2, void* c, int m, int n, int k, int ldc,
                             GemmEpilogue epi, hipStream_t st) {
  return dispatch(a, w, w2, nullptr, n, n, c, m, n, k, ldc, epi, st);
}

// q | k | v projections of the same rows as one GEMM over the concatenated output columns
template <>
hipError_t launch_gemm_qkv<bf16>(const bf16* a, const bf16* wq, int nq, const bf16* wk, const bf16* wv, int nkv,
                                 float* c, int m, int k, hipStream_t st) {
  const int n = nq + 2 * nkv;
  return dispatch(a, wq, wk, wv, nq, nq + nkv, c, m, n, k, n, EPI_STORE_F32, st);
}

}  // namespace rc
