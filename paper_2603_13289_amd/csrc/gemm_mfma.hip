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
// The register-staged kernel fetches the next K step into registers while the current one is multiplied;
// the direct-to-LDS kernel keeps two K steps in flight in two LDS buffers.
// Each wavefront owns a (BM/WAVES_M) x (BN/WAVES_N) sub-tile, built from 32x32x16 MFMA blocks in the
// register-staged kernel (any K) and from 16x16x32 blocks in the direct-to-LDS kernel (K a multiple of 64).
//
// SwiGLU epilogue (DUAL): the B tile stacks BN/2 rows of W_gate on BN/2 rows of W_up for the same
// output columns, every wavefront holds matching gate/up accumulators and writes silu(gate)*up.
//
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids congruent mod 8) walk
// all row tiles of the same few weight-column tiles: a weight tile is then fetched from HBM once
// per XCD-L2 instead of once per row tile.
#include <algorithm>
#include <vector>

#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int BK = 64;
static constexpr int XCDS = 8;
static int g_xcd_remap = 1;
void set_gemm_xcd_remap(int on) { g_xcd_remap = on; }

__device__ inline float silu_mf(float x) { return x / (1.0f + __expf(-x)); }

// Accumulator element e of the 32x32 block (i, j) of a wavefront sits at row 8*(e/4) + 4*(lane/32) + e%4,
// column lane%32 of that block.
template <int FM, int FN, int WTM, int WTN, bool DUAL>
__device__ inline void store_tile(const f32x16 (&acc)[FM][FN], void* __restrict__ c, int m, int n, int ldc, int epi,
                                  int m0, int n0, int wm, int wn, int lane) {
  constexpr int FN_OUT = DUAL ? FN / 2 : FN;
  constexpr int WTN_OUT = DUAL ? WTN / 2 : WTN;
  const int khalf = lane >> 5;
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

// Order in which output tiles are handed to workgroups.  The tile rows are cut into `bands` bands of (almost)
// equal height; inside a band tiles run row-first (M fastest), bands follow each other.  The 32 workgroups
// that an XCD runs at a time then cover a block of about 5 x 6 tiles instead of a whole tile column, so
// fewer distinct A and W slices have to come into that XCD's L2 per K step.
struct TileOrder { int tiles_m, tiles_n, bands; };

__device__ __host__ inline void tile_of(TileOrder o, int logical, int* tile_m, int* tile_n) {
  const int base = o.tiles_m / o.bands, rem = o.tiles_m % o.bands;
  const int cut = rem * (base + 1) * o.tiles_n;   // tiles in the taller bands
  int h, m_start, r;
  if (logical < cut) {
    h = base + 1;
    const int per = h * o.tiles_n;
    m_start = (logical / per) * h;
    r = logical % per;
  } else {
    h = base;
    const int per = h * o.tiles_n;
    const int l2 = logical - cut;
    m_start = rem * (base + 1) + (l2 / per) * h;
    r = l2 % per;
  }
  *tile_m = m_start + r % h;
  *tile_n = r / h;
}

__device__ __host__ inline TileOrder make_tile_order(int tiles_m, int tiles_n) {
  TileOrder o = {tiles_m, tiles_n, (tiles_m + 5) / 6};
  if (o.bands < 1) o.bands = 1;
  return o;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool DUAL, int OCC>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64, OCC)
gemm_mfma_kernel(const bf16* __restrict__ a, const bf16* __restrict__ w, const bf16* __restrict__ w2,
                 const bf16* __restrict__ w3, int ns1, int ns2, void* __restrict__ c, int m, int n, int k, int ldc,
                 int epi, TileOrder order, int total_tiles, int per_xcd, const int* __restrict__ m_live) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int A_PER = BM * 8 / NT, B_PER = BN * 8 / NT;
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  static_assert(A_PER * NT == BM * 8 && B_PER * NT == BN * 8, "tile/threads mismatch");
  static_assert(!DUAL || (FN % 2 == 0), "dual tiles need an even number of column fragments");

  __shared__ uint4 lds_a[BM * 8];
  __shared__ uint4 lds_b[BN * 8];

  const int logical = per_xcd > 0 ? (int)(blockIdx.x % XCDS) * per_xcd + (int)(blockIdx.x / XCDS) : (int)blockIdx.x;
  if (logical >= total_tiles) return;
  int tile_m, tile_n;
  tile_of(order, logical, &tile_m, &tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN_OUT;
  m = live_count(m, m_live);
  if (m0 >= m) return;   // uniform: the grid may be sized for an upper bound of the row count

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

  store_tile<FM, FN, WTM, WTN, DUAL>(acc, c, m, n, ldc, epi, m0, n0, wm, wn, lane);
}

// ------------------------------------------------------------------ direct-to-LDS, double-buffered kernel
// Tiles are fetched with 16-byte global->LDS loads (no staging registers, no LDS store instructions) into two
// alternating LDS buffers, so one barrier per K step suffices: wait for my loads, barrier, start the loads
// of the step after next into the buffer just freed, multiply the current one.
//
// A direct load writes lane l's 16 bytes to (wave-uniform LDS base) + 16 l, i.e. one instruction fills
// 1 KB = 8 rows of 128 bytes.  The XOR placement (chunk c of row r at slot c ^ ((r >> 1) & 7)) is
// therefore applied on the global side: lane l of a row block fetches chunk (l & 7) ^ swz(row).
// Rows past M (or N) re-read the last valid row; their products are never stored.  K must be a
// multiple of 64.
//
// The wavefront sub-tile is built from 16x16x32 MFMA blocks (measured: with the same LDS and load traffic
// this shape sustains about 9 % more matrix throughput than 32x32x16 under the chip's power limit).  A K
// step of 64 is two sub-steps of 32; each sub-step is multiplied in two halves of the weight-column blocks,
// so a pipeline unit is FM x FN/2 MFMAs with the LDS reads of the next unit in flight.  16 lanes reading the
// same chunk of 16 consecutive rows (one operand fetch) touch all 64 LDS banks once, as in the kernel above.
//
// The weight fragment is passed as the first MFMA operand, so that accumulator (i, j) of a lane holds
//   row    i*16 + lane%16                 of the wavefront's activation rows,
//   column j*16 + 4*(lane/16) + e         of its output columns, e = 0..3:
// four consecutive output columns per lane, stored with one 16-byte (f32) or 8-byte (bf16) access.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

template <int FM, int FN, int WTM, int WTN, bool DUAL>
__device__ inline void store_tile16(const f32x4 (&acc)[FM][FN], void* __restrict__ c, int m, int n, int ldc, int epi,
                                    int m0, int n0, int wm, int wn, int lane) {
  constexpr int FN_OUT = DUAL ? FN / 2 : FN;
  constexpr int WTN_OUT = DUAL ? WTN / 2 : WTN;
  const bool f32_out = !DUAL && (epi == EPI_STORE_F32 || epi == EPI_ADD_F32);
  const bool vec_ok = (ldc & 3) == 0 && (reinterpret_cast<size_t>(c) & (f32_out ? 15 : 7)) == 0;
  if constexpr (!DUAL) {
    // residual add with the wavefront's columns all inside C: the old values of a block row are requested together and
    // added afterwards, so the wavefront waits for memory once per block row instead of once per 16 x 16 block
    if (epi == EPI_ADD_F32 && vec_ok && n0 + wn * WTN + WTN <= n) {   // wave-uniform
      float* const cf = reinterpret_cast<float*>(c);
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = m0 + wm * WTM + i * 16 + (lane & 15);
        if (row >= m) continue;
        float4* const dst = reinterpret_cast<float4*>(cf + (size_t)row * ldc + n0 + wn * WTN + 4 * (lane >> 4));
        float4 old[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) old[j] = dst[j * 4];
#pragma unroll
        for (int j = 0; j < FN; ++j)
          dst[j * 4] = make_float4(old[j].x + acc[i][j][0], old[j].y + acc[i][j][1], old[j].z + acc[i][j][2],
                                   old[j].w + acc[i][j][3]);
      }
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int row = m0 + wm * WTM + i * 16 + (lane & 15);
    if (row >= m) continue;
#pragma unroll
    for (int j = 0; j < FN_OUT; ++j) {
      const int col = n0 + wn * WTN_OUT + j * 16 + 4 * (lane >> 4);
      if (col >= n) continue;
      const size_t o = (size_t)row * ldc + col;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = DUAL ? silu_mf(acc[i][j][e]) * acc[i][j + FN_OUT][e] : acc[i][j][e];
      if (vec_ok && col + 3 < n) {
        if (f32_out) {
          float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(c) + o);
          float4 t = make_float4(v[0], v[1], v[2], v[3]);
          if (epi == EPI_ADD_F32) { const float4 old = *dst; t.x += old.x; t.y += old.y; t.z += old.z; t.w += old.w; }
          *dst = t;
        } else {
          union { bf16 h[4]; uint2 u; } pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk.h[e] = f32_to_bf16(v[e]);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16*>(c) + o) = pk.u;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (col + e >= n) continue;
          if (!f32_out) reinterpret_cast<bf16*>(c)[o + e] = f32_to_bf16(v[e]);
          else if (epi == EPI_ADD_F32) reinterpret_cast<float*>(c)[o + e] += v[e];
          else reinterpret_cast<float*>(c)[o + e] = v[e];
        }
      }
    }
  }
}

// One output tile (or one K part of it): the work of a workgroup once it knows its tile.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool DUAL>
__device__ __forceinline__ void gemm_tile_body(const bf16* __restrict__ a, const bf16* __restrict__ w,
                                               const bf16* __restrict__ w2, const bf16* __restrict__ w3, int ns1, int ns2,
                                               void* __restrict__ c, int m, int n, int k, int ldc, int epi, int m0, int n0,
                                               int k_begin, int k_end, int part_slot, float* __restrict__ partial) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int FM = WTM / 16, FN = WTN / 16, FH = FN / 2;
  constexpr int A_BLK = BM / 8, B_BLK = BN / 8;
  constexpr int A_PER = A_BLK / NW, B_PER = B_BLK / NW;
  static_assert(A_PER * NW == A_BLK && B_PER * NW == B_BLK, "tile/waves mismatch");
  static_assert(FN % 2 == 0 && BK == 64, "two sub-steps of 32, two halves of the column blocks");
  constexpr int TILE_BYTES = (BM + BN) * 128;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];   // 2 x [A tile | B tile]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const int lrow = lane >> 3, lslot = lane & 7;
  const bf16* pa[A_PER];
  const bf16* pb[B_PER];
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int row = (wave + i * NW) * 8 + lrow;
    const int chunk = lslot ^ ((row >> 1) & 7);
    pa[i] = a + (size_t)min(m0 + row, m - 1) * k + chunk * 8;
  }
#pragma unroll
  for (int i = 0; i < B_PER; ++i) {
    const int row = (wave + i * NW) * 8 + lrow;
    const int chunk = lslot ^ ((row >> 1) & 7);
    const bf16* src;
    if (DUAL) {
      const int half = row >= BN / 2;
      const int col = min(n0 + row - half * (BN / 2), n - 1);
      src = (half ? w2 : w) + (size_t)col * k;
    } else {
      const int col = min(n0 + row, n - 1);
      src = col < ns1 ? w + (size_t)col * k : (col < ns2 ? w2 + (size_t)(col - ns1) * k : w3 + (size_t)(col - ns2) * k);
    }
    pb[i] = src + chunk * 8;
  }
  auto issue = [&](int k0, int buf) {
    unsigned char* base = lds + buf * TILE_BYTES;
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(pa[i] + k0),
                                       (__attribute__((address_space(3))) void*)(base + (wave + i * NW) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(pb[i] + k0),
                                       (__attribute__((address_space(3))) void*)(base + BM * 128 + (wave + i * NW) * 1024), 16, 0, 0);
  };

  f32x4 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // LDS rows this lane reads its operands from: lane%16 selects the row of a 16-row block, lane/16 the 8-k chunk
  int arow[FM], brow[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) arow[i] = wm * WTM + i * 16 + (lane & 15);
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    if (DUAL) brow[j] = (j < FH ? wn * (WTN / 2) + j * 16 : BN / 2 + wn * (WTN / 2) + (j - FH) * 16) + (lane & 15);
    else brow[j] = wn * WTN + j * 16 + (lane & 15);
  }
  const int kq = lane >> 4;

  bf16x8 fa[2][FM], fb[2][FH];
  auto load_a = [&](int b, int s) {
    const uint4* la = reinterpret_cast<const uint4*>(lds + b * TILE_BYTES);
    const int chunk = 4 * s + kq;
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[s][i] = __builtin_bit_cast(bf16x8, la[arow[i] * 8 + (chunk ^ ((arow[i] >> 1) & 7))]);
  };
  auto load_b = [&](int b, int s, int h) {
    const uint4* lb = reinterpret_cast<const uint4*>(lds + b * TILE_BYTES + BM * 128);
    const int chunk = 4 * s + kq;
#pragma unroll
    for (int j = 0; j < FH; ++j) {
      const int r = brow[h * FH + j];
      fb[h][j] = __builtin_bit_cast(bf16x8, lb[r * 8 + (chunk ^ ((r >> 1) & 7))]);
    }
  };
  auto multiply = [&](int s, int h) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FH; ++j)
        acc[i][h * FH + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[h][j], fa[s][i], acc[i][h * FH + j], 0, 0, 0);
  };

  if (k_begin < k_end) {
    issue(k_begin, 0);
    if (k_begin + BK < k_end) issue(k_begin + BK, 1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    load_a(0, 0);
    load_b(0, 0, 0);
  }
  int buf = 0;
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    load_b(buf, 0, 1);
    __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads of the next unit ahead of this unit's MFMAs
    multiply(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    load_a(buf, 1);
    load_b(buf, 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(0, 1);
    __builtin_amdgcn_sched_barrier(0);
    load_b(buf, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(1, 0);
    __builtin_amdgcn_sched_barrier(0);
    // the last unit's operands are being read; once they are in registers nobody needs buffer `buf` any more
    __builtin_amdgcn_s_waitcnt(0);   // my LDS reads and my direct loads of the next step are complete
    __syncthreads();
    if (k0 + 2 * BK < k_end) issue(k0 + 2 * BK, buf);
    if (k0 + BK < k_end) { load_a(buf ^ 1, 0); load_b(buf ^ 1, 0, 0); }
    __builtin_amdgcn_sched_barrier(0);
    multiply(1, 1);
    __builtin_amdgcn_sched_barrier(0);
    buf ^= 1;
  }

  if (part_slot >= 0) {
    // raw accumulators, register-major so that consecutive lanes write consecutive floats
    constexpr int NT = NW * 64;
    float* dst = partial + (size_t)part_slot * (FM * FN * 4) * NT + tid;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[(size_t)((i * FN + j) * 4 + e) * NT] = acc[i][j][e];
    return;
  }
  store_tile16<FM, FN, WTM, WTN, DUAL>(acc, c, m, n, ldc, epi, m0, n0, wm, wn, lane);
}

// What the launch's grid does.  Workgroups [0, n_full_wgs) each own one of the first full_tiles output tiles
// (whole K range).  The remaining tiles, too few to fill the chip, are each cut along K into `split` parts:
// workgroup n_full_wgs + j takes part j % split of the tile after the whole ones + j / split and leaves its raw
// accumulators in `partial`; gemm_fixup_kernel adds the parts in a fixed order and applies the epilogue.
//
// Thin tiles: when the last tile row has at most 64 live rows (a prompt whose live rows are a multiple of the tile
// height plus a few: the last reused token, a short suffix), its n_thin tiles are multiplied by a 64-row body whose
// eight wavefronts sit side by side, which costs about a third of a full tile; `order` then describes the tile rows
// above it only.  The thin tiles are always whole-K tiles and are dealt out evenly over the XCDs' queues, at
// the tail of each, where they fill the last round.  (A 128-row body for up to 128 live rows was measured
// as well: no gain.)
struct GridPlan {
  TileOrder order;      // the normal tiles (all tile rows, or all but the ragged last one)
  int full_tiles;       // whole-K tiles: normal ones first, then the n_thin thin ones
  int per_xcd;          // > 0: workgroup ids are regrouped per XCD, this many queue slots each
  int n_full_wgs;       // workgroups reserved for whole-K tiles (some may stay empty)
  int split, kpp;       // K parts per remaining tile, K steps per part
  int n_thin;
};
struct BlockWork { int kind /* 0: nothing, 1: normal tile, 2: thin tile */, tile_m, tile_n, k_begin, k_end, part_slot; };

__device__ __host__ inline BlockWork block_work(const GridPlan& g, int bid, int k) {
  BlockWork bw = {0, 0, 0, 0, k, -1};
  const int n_normal_full = g.full_tiles - g.n_thin;
  int u = 0, thin_tile = -1;   // u: index among the normal tiles
  if (bid < g.n_full_wgs) {
    if (g.per_xcd > 0) {
      const int x = bid % XCDS, j = bid / XCDS;
      const int cnt = g.n_thin / XCDS + (x < g.n_thin % XCDS ? 1 : 0);                          // thin tiles of this XCD
      const int before = x * (g.n_thin / XCDS) + (x < g.n_thin % XCDS ? x : g.n_thin % XCDS);   // ... of the XCDs before it
      if (j >= g.per_xcd - cnt) thin_tile = (j - (g.per_xcd - cnt)) * XCDS + x;
      else u = x * g.per_xcd - before + j;
    } else if (bid >= n_normal_full) {
      thin_tile = bid - n_normal_full;
      if (thin_tile >= g.n_thin) return bw;
    } else {
      u = bid;
    }
    if (thin_tile < 0 && u >= n_normal_full) return bw;
  } else {
    const int j = bid - g.n_full_wgs;
    u = n_normal_full + j / g.split;
    bw.part_slot = j;
    bw.k_begin = (j % g.split) * g.kpp * BK;
    bw.k_end = bw.k_begin + g.kpp * BK < k ? bw.k_begin + g.kpp * BK : k;
  }
  if (thin_tile >= 0) {
    bw.kind = 2;
    bw.tile_m = g.order.tiles_m;   // the row below the normal ones
    bw.tile_n = thin_tile;
  } else {
    bw.kind = 1;
    tile_of(g.order, u, &bw.tile_m, &bw.tile_n);
  }
  return bw;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool DUAL, int OCC, bool THIN>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64, OCC)
gemm_mfma_dl_kernel(const bf16* __restrict__ a, const bf16* __restrict__ w, const bf16* __restrict__ w2,
                    const bf16* __restrict__ w3, int ns1, int ns2, void* __restrict__ c, int m, int n, int k, int ldc,
                    int epi, GridPlan plan, float* __restrict__ partial, const int* __restrict__ m_live) {
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  if (m_live) {
    // The row count lives on the device (rows selected by a threshold) and the host's m only sized the grid.  The
    // schedule is rebuilt here for the live count, in its plain form: every tile whole, by one workgroup, ids
    // regrouped per XCD over the live tiles (so that all XCDs share them), no K-split tail, no thin tiles.
    m = min(m, *m_live);
    if (m <= 0) return;
    const int tiles_m = (m + BM - 1) / BM, tiles_n = plan.order.tiles_n;
    const int total = tiles_m * tiles_n, per_xcd = (total + XCDS - 1) / XCDS;
    const int x = (int)blockIdx.x % XCDS, j = (int)blockIdx.x / XCDS;
    const int logical = plan.per_xcd > 0 ? x * per_xcd + j : (int)blockIdx.x;
    if ((plan.per_xcd > 0 && j >= per_xcd) || logical >= total) return;
    int tile_m, tile_n;
    tile_of(make_tile_order(tiles_m, tiles_n), logical, &tile_m, &tile_n);
    gemm_tile_body<BM, BN, WAVES_M, WAVES_N, DUAL>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, tile_m * BM, tile_n * BN_OUT,
                                                   0, k, -1, partial);
    return;
  }
  const BlockWork bw = block_work(plan, (int)blockIdx.x, k);
  if (bw.kind == 0) return;
  if constexpr (THIN) {
    if (bw.kind == 2) {
      gemm_tile_body<64, BN, 1, WAVES_M * WAVES_N, DUAL>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, bw.tile_m * BM,
                                                         bw.tile_n * BN_OUT, 0, k, -1, partial);
      return;
    }
  }
  gemm_tile_body<BM, BN, WAVES_M, WAVES_N, DUAL>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, bw.tile_m * BM,
                                                 bw.tile_n * BN_OUT, bw.k_begin, bw.k_end, bw.part_slot, partial);
}

// Sum of the K-split parts of the tail tiles (fixed order: part 0, 1, ...) followed by the epilogue.  One
// workgroup per (tile, accumulator (i, j)); thread t owns the same (wavefront, lane) as thread t of the GEMM
// kernel, so all reads of a part are coalesced.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool DUAL>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64)
gemm_fixup_kernel(void* __restrict__ c, int m, int n, int ldc, int epi, TileOrder order, int full_tiles /* of `order` */,
                  int split, const float* __restrict__ partial) {
  constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int FM = WTM / 16, FN = WTN / 16;
  constexpr int FN_OUT = DUAL ? FN / 2 : FN;
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  constexpr int PER_TILE = FM * FN_OUT;
  const int t = (int)blockIdx.x / PER_TILE;
  const int rest = (int)blockIdx.x % PER_TILE;
  const int j = rest % FN_OUT, i = rest / FN_OUT;
  int tile_m, tile_n;
  tile_of(order, full_tiles + t, &tile_m, &tile_n);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  // the sums land in a one-accumulator "tile" so that the epilogue code is the GEMM kernel's own
  f32x4 one[1][DUAL ? 2 : 1];
#pragma unroll
  for (int e = 0; e < 4; ++e) { one[0][0][e] = 0.f; if (DUAL) one[0][DUAL ? 1 : 0][e] = 0.f; }
  for (int p = 0; p < split; ++p) {
    const float* src = partial + (size_t)(t * split + p) * (FM * FN * 4) * NT + tid;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      one[0][0][e] += src[(size_t)((i * FN + j) * 4 + e) * NT];
      if (DUAL) one[0][DUAL ? 1 : 0][e] += src[(size_t)((i * FN + j + FN_OUT) * 4 + e) * NT];
    }
  }
  // row/column origin of accumulator (i, j) of this wavefront
  const int m_org = tile_m * BM + wm * WTM + i * 16;
  const int n_org = tile_n * BN_OUT + wn * (DUAL ? WTN / 2 : WTN) + j * 16;
  store_tile16<1, DUAL ? 2 : 1, 16, DUAL ? 32 : 16, DUAL>(one, c, m, n, ldc, epi, m_org, n_org, 0, 0, lane);
}

// Rough time model (microseconds, measured on MI355X) used to choose the tile and the K-split of the tail:
// one K step of a full round costs kStep256 with 256x256 tiles, kStep192 with 256x192 tiles (one workgroup per
// CU each) and kStep128 with 128x128 tiles (two per CU); summing one tile part in the fix-up costs kFixPart.
static constexpr float kStep256 = 1.9f, kStep192 = 1.55f, kStep128 = 1.2f, kFixPart = 0.1f, kFixLaunch = 6.f;

struct SplitPlan { int rem, split; float cost; };
// total tiles over `slots` workgroup slots: full rounds, then `rem` tiles cut into `split` K parts each
static SplitPlan plan_tail_split(int total, int slots, int ksteps, float step = kStep256) {
  SplitPlan best;
  best.rem = total % slots;
  best.split = 1;
  const int full_rounds = total / slots;
  best.cost = (full_rounds + (best.rem > 0 ? 1 : 0)) * ksteps * step;
  if (best.rem == 0) return best;
  const int gmax = std::min(std::min(slots / best.rem, 16), ksteps);
  for (int g = 2; g <= gmax; ++g) {
    if (best.rem * g > 256) break;
    const float c = full_rounds * ksteps * step + ((ksteps + g - 1) / g) * step + best.rem * g * kFixPart + kFixLaunch;
    if (c < best.cost) { best.cost = c; best.split = g; }
  }
  return best;
}

// compute units of the current device (asked once per device)
static int num_cus() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  std::atomic<int>& slot = cached[dev & 63];
  int n = slot.load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    slot.store(n, std::memory_order_relaxed);
  }
  return n;
}

size_t gemm_partial_bytes() { return (size_t)256 * 256 * 256 * sizeof(float) + 4096; }   // 256 tile parts

// Schedule of a launch of 256-row tiles: which tiles run whole, which are cut along K, and whether the ragged
// last tile row goes to the thin body.  A thin tile is priced at kThinCost of a full one.
static constexpr float kThinCost = 0.4f;
static constexpr int kThinRows = 64;
static int g_thin_tiles = 1;
void set_gemm_thin_tiles(int on) { g_thin_tiles = on; }

struct LaunchPlan {
  int n_thin;                 // tiles of the ragged last tile row handled by the thin body (0: none)
  int n_normal;               // tiles of the other rows
  int rem, split, kpp;        // the last `rem` normal tiles are cut into `split` parts of `kpp` K steps
  float cost;
};

// thin: price and schedule the launch with the ragged last tile row on the thin body; cost < 0 if that is not possible
static LaunchPlan plan_one(int m, int tiles_n, int bm, int ksteps, int slots, float step, bool may_split, bool thin) {
  const int tiles_m = (m + bm - 1) / bm;
  LaunchPlan p = {};
  p.cost = -1.f;
  if (thin) {
    const int ragged = m - (tiles_m - 1) * bm;   // live rows of the last tile row
    if (tiles_m < 2 || ragged > kThinRows) return p;
    p.n_thin = tiles_n;
  }
  p.n_normal = tiles_m * tiles_n - p.n_thin;
  const int equiv = p.n_normal + (int)(p.n_thin * kThinCost + 0.999f);
  p.split = 1;
  p.kpp = ksteps;
  float cost;
  if (may_split) {
    const SplitPlan sp = plan_tail_split(equiv, slots, ksteps, step);
    cost = sp.cost;
    if (sp.split > 1) {
      p.rem = sp.rem;
      p.kpp = (ksteps + sp.split - 1) / sp.split;
      p.split = (ksteps + p.kpp - 1) / p.kpp;
    }
  } else {
    cost = ((equiv + slots - 1) / slots) * ksteps * step;
  }
  // thin tiles only among the whole tiles of a launch that has at least one full round
  if (thin && (equiv < slots || p.rem > p.n_normal)) return p;
  p.cost = cost;
  return p;
}

static LaunchPlan plan_launch(int m, int tiles_n, int bm, int ksteps, int slots, float step, bool may_split, bool may_thin) {
  const LaunchPlan plain = plan_one(m, tiles_n, bm, ksteps, slots, step, may_split, false);
  if (may_thin && g_thin_tiles) {
    const LaunchPlan thin = plan_one(m, tiles_n, bm, ksteps, slots, step, may_split, true);
    if (thin.cost >= 0.f && thin.cost < plain.cost) return thin;
  }
  return plain;
}

// the grid of a direct-to-LDS launch: tiles of bm rows, tiles_n tile columns
static GridPlan make_grid_plan(int m, int tiles_n, int bm, int ksteps, int slots, float step, bool may_split, bool may_thin,
                               int* n_blocks, int* rem_tiles) {
  const int tiles_m = (m + bm - 1) / bm;
  const LaunchPlan lp = plan_launch(m, tiles_n, bm, ksteps, slots, step, may_split, may_thin);
  GridPlan g;
  g.order = make_tile_order(lp.n_thin > 0 ? tiles_m - 1 : tiles_m, tiles_n);
  g.full_tiles = lp.n_thin + lp.n_normal - lp.rem;
  g.per_xcd = (g.full_tiles + XCDS - 1) / XCDS;
  g.n_full_wgs = g.per_xcd * XCDS;
  g.split = lp.split;
  g.kpp = lp.kpp;
  g.n_thin = lp.n_thin;
  *n_blocks = g.n_full_wgs + lp.rem * lp.split;
  *rem_tiles = lp.rem;
  if (!g_xcd_remap) g.per_xcd = 0;
  return g;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int OCC>
static hipError_t launch_dl(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2, void* c,
                            int m, int n, int k, int ldc, GemmEpilogue epi, float* partial, hipStream_t st,
                            const int* m_live) {
  if (m_live) partial = nullptr;   // the kernel rebuilds the plain schedule for the live row count
  const bool dual = epi == EPI_SWIGLU_T;
  const int bn_out = dual ? BN / 2 : BN;
  const int tiles_n = (n + bn_out - 1) / bn_out;
  // Full rounds of one tile per workgroup slot; the remainder (less than one round) is cut along K so
  // that it also fills the chip.  Only with a partial buffer, and only for the one-workgroup-per-CU tiles.
  constexpr bool THIN = BM == 256 && BN == 256 && OCC == 1;
  int n_blocks = 0, rem_tiles = 0;
  const GridPlan plan = make_grid_plan(m, tiles_n, BM, k / BK, num_cus() * OCC, BN == 192 ? kStep192 : kStep256,
                                       partial != nullptr && OCC == 1, THIN && m_live == nullptr, &n_blocks, &rem_tiles);
  const int normal_full = plan.full_tiles - plan.n_thin;
  const dim3 grid((unsigned)n_blocks);
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * 128;
  hipError_t e = hipSuccess;
  if (dual) {
    auto kern = gemm_mfma_dl_kernel<BM, BN, WAVES_M, WAVES_N, true, OCC, THIN>;
    static std::atomic<unsigned long long> told{0};
    e = allow_dynamic_lds((const void*)kern, (int)lds_bytes, told);
    if (e != hipSuccess) return e;
    kern<<<grid, NT, lds_bytes, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, (int)epi, plan, partial, m_live);
    if (rem_tiles > 0)
      gemm_fixup_kernel<BM, BN, WAVES_M, WAVES_N, true><<<rem_tiles * (BM / WAVES_M / 16) * (BN / WAVES_N / 32), NT, 0, st>>>(
          c, m, n, ldc, (int)epi, plan.order, normal_full, plan.split, partial);
  } else {
    auto kern = gemm_mfma_dl_kernel<BM, BN, WAVES_M, WAVES_N, false, OCC, THIN>;
    static std::atomic<unsigned long long> told{0};
    e = allow_dynamic_lds((const void*)kern, (int)lds_bytes, told);
    if (e != hipSuccess) return e;
    kern<<<grid, NT, lds_bytes, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, (int)epi, plan, partial, m_live);
    if (rem_tiles > 0)
      gemm_fixup_kernel<BM, BN, WAVES_M, WAVES_N, false><<<rem_tiles * (BM / WAVES_M / 16) * (BN / WAVES_N / 16), NT, 0, st>>>(
          c, m, n, ldc, (int)epi, plan.order, normal_full, plan.split, partial);
  }
  return hipGetLastError();
}

// Host-side check of a launch's grid: every output tile must be covered exactly once, by one whole-K workgroup or by
// K parts that partition [0, k) in part order; thin tiles only in the last tile row and only for at most 64 live rows.
// Returns the number of violations; *n_blocks_out receives the grid size.  tile: 5, 6 or 7; n_cus: CUs to plan for.
int check_grid_plan(int m, int n, int k, bool dual, int tile, int n_cus, bool with_partial, int* n_blocks_out) {
  const int bm = tile == 6 ? 128 : 256, bn = tile == 6 ? 128 : (tile == 7 ? 192 : 256), occ = tile == 6 ? 2 : 1;
  const int bn_out = dual ? bn / 2 : bn;
  const int tiles_m = (m + bm - 1) / bm, tiles_n = (n + bn_out - 1) / bn_out;
  int n_blocks = 0, rem_tiles = 0;
  const GridPlan g = make_grid_plan(m, tiles_n, bm, k / BK, n_cus * occ, tile == 7 ? kStep192 : kStep256,
                                    with_partial && occ == 1, tile == 5, &n_blocks, &rem_tiles);
  if (n_blocks_out) *n_blocks_out = n_blocks;
  int errors = 0;
  std::vector<int> covered((size_t)tiles_m * tiles_n, 0), next_k((size_t)tiles_m * tiles_n, 0), slots;
  for (int bid = 0; bid < n_blocks; ++bid) {
    const BlockWork bw = block_work(g, bid, k);
    if (bw.kind == 0) continue;
    if (bw.tile_m < 0 || bw.tile_m >= tiles_m || bw.tile_n < 0 || bw.tile_n >= tiles_n) { ++errors; continue; }
    const size_t t = (size_t)bw.tile_m * tiles_n + bw.tile_n;
    if (bw.kind == 2 && (bw.tile_m != tiles_m - 1 || m - (tiles_m - 1) * bm > kThinRows || bw.part_slot >= 0)) ++errors;
    if (bw.part_slot < 0) {
      if (bw.k_begin != 0 || bw.k_end != k || covered[t] != 0) ++errors;
      covered[t] = 1;
      next_k[t] = k;
    } else {
      // parts arrive in block order = part order
      if (covered[t] == 1 || bw.k_begin != next_k[t] || bw.k_end <= bw.k_begin || bw.k_end > k) ++errors;
      covered[t] = 2;
      next_k[t] = bw.k_end;
      slots.push_back(bw.part_slot);
    }
  }
  for (size_t t = 0; t < covered.size(); ++t)
    if (covered[t] == 0 || next_k[t] != k) ++errors;
  // part slots are 0, 1, ... without gaps and fit the partial buffer
  for (size_t i = 0; i < slots.size(); ++i)
    if (slots[i] != (int)i) ++errors;
  if (slots.size() > 256) ++errors;
  return errors;
}

static int g_gemm_tile = 0;   // 0: by shape; 1-3: register-staged 128x256 / 256x256 / 128x128; 5-7: direct-to-LDS 256x256 / 128x128 / 256x192
void set_gemm_tile(int t) { g_gemm_tile = t; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int OCC>
static hipError_t launch_cfg(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2, void* c,
                             int m, int n, int k, int ldc, GemmEpilogue epi, hipStream_t st, const int* m_live) {
  const bool dual = epi == EPI_SWIGLU_T;
  const int bn_out = dual ? BN / 2 : BN;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + bn_out - 1) / bn_out;
  const int total = tiles_m * tiles_n;
  int per_xcd = (total + XCDS - 1) / XCDS;
  const dim3 grid((unsigned)(per_xcd * XCDS));
  if (!g_xcd_remap) per_xcd = 0;
  constexpr int NT = WAVES_M * WAVES_N * 64;
  if (dual)
    gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, true, OCC><<<grid, NT, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc,
                                                                              (int)epi, make_tile_order(tiles_m, tiles_n), total, per_xcd, m_live);
  else
    gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, false, OCC><<<grid, NT, 0, st>>>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc,
                                                                               (int)epi, make_tile_order(tiles_m, tiles_n), total, per_xcd, m_live);
  return hipGetLastError();
}

static hipError_t dispatch(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2, void* c,
                           int m, int n, int k, int ldc, GemmEpilogue epi, float* partial, hipStream_t st,
                           const int* m_live) {
  if (m <= 0 || n <= 0) return hipSuccess;
  int tile = g_gemm_tile;
  if (tile == 0 && gemm_skinny_applies(m, n, k, ns1, ns2))
    return launch_gemm_skinny_bf16(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st, m_live);
  if (m_live) partial = nullptr;   // live row count on the device: plain schedule, priced as such
  if (tile == 0) {
    if (k % BK != 0) {
      tile = 3;
    } else {
      // 256x256 tiles (one workgroup per CU, K-split tail) against 128x128 tiles (two per CU), by the time model
      const bool dual = epi == EPI_SWIGLU_T;
      const int ksteps = k / BK;
      const long t6 = (long)((m + 127) / 128) * ((n + (dual ? 63 : 127)) / (dual ? 64 : 128));
      const int slots6 = 2 * num_cus();
      const float cost5 = plan_launch(m, (n + (dual ? 127 : 255)) / (dual ? 128 : 256), 256, ksteps, num_cus(), kStep256,
                                      partial != nullptr, true).cost;
      const long last6 = t6 % slots6;
      const float cost6 = (t6 / slots6) * ksteps * kStep128 +
                          (last6 == 0 ? 0.f : (last6 * 2 <= slots6 ? 0.65f : 1.f) * ksteps * kStep128);
      tile = cost5 <= cost6 ? 5 : 6;
      // 256x192 tiles where they cover N exactly (the fused q|k|v projection: 6144 = 32 x 192): a launch of a
      // few hundred rows then has a third more tiles to spread over the CUs
      if (!dual && n % 192 == 0) {
        const float cost7 = plan_launch(m, n / 192, 256, ksteps, num_cus(), kStep192, partial != nullptr, false).cost;
        if (cost7 < std::min(cost5, cost6)) tile = 7;
      }
    }
  }
  if (tile >= 5 && (k % BK) != 0) tile = 3;   // the direct-load kernels need whole K steps
  switch (tile) {
    case 5: return launch_dl<256, 256, 4, 2, 1>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, partial, st, m_live);
    case 6: return launch_dl<128, 128, 2, 2, 2>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, nullptr, st, m_live);
    case 7: return launch_dl<256, 192, 4, 2, 1>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, partial, st, m_live);
    case 2: return launch_cfg<256, 256, 4, 2, 1>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st, m_live);
    case 3: return launch_cfg<128, 128, 2, 2, 2>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st, m_live);
    default: return launch_cfg<128, 256, 2, 2, 2>(a, w, w2, w3, ns1, ns2, c, m, n, k, ldc, epi, st, m_live);
  }
}

template <>
hipError_t launch_gemm<bf16>(const bf16* a, const bf16* w, const bf16* w2, void* c, int m, int n, int k, int ldc,
                             GemmEpilogue epi, hipStream_t st, const int* m_live) {
  return dispatch(a, w, w2, nullptr, n, n, c, m, n, k, ldc, epi, nullptr, st, m_live);
}

hipError_t launch_gemm_bf16(const bf16* a, const bf16* w, const bf16* w2, void* c, int m, int n, int k, int ldc,
                            GemmEpilogue epi, float* partial, hipStream_t st, const int* m_live) {
  return dispatch(a, w, w2, nullptr, n, n, c, m, n, k, ldc, epi, partial, st, m_live);
}

hipError_t launch_gemm_qkv_bf16(const bf16* a, const bf16* wq, int nq, const bf16* wk, const bf16* wv, int nkv, float* c,
                                int m, int k, float* partial, hipStream_t st, const int* m_live) {
  const int n = nq + 2 * nkv;
  return dispatch(a, wq, wk, wv, nq, nq + nkv, c, m, n, k, n, EPI_STORE_F32, partial, st, m_live);
}

// q | k | v projections of the same rows as one GEMM over the concatenated output columns
template <>
hipError_t launch_gemm_qkv<bf16>(const bf16* a, const bf16* wq, int nq, const bf16* wk, const bf16* wv, int nkv,
                                 float* c, int m, int k, hipStream_t st, const int* m_live) {
  const int n = nq + 2 * nkv;
  return dispatch(a, wq, wk, wv, nq, nq + nkv, c, m, n, k, n, EPI_STORE_F32, nullptr, st, m_live);
}

}  // namespace rc
