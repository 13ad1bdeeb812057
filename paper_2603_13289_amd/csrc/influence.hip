// Influence accumulation of the decode-side cache manager (Eq. 6): for the one query row that a
// decoding step adds per request, the attention weight it puts on every cached position, summed over
// the query heads, is added to that request's s_inf vector; the caller adds up layers and steps by
// calling once per layer and step.
//
// Three small memory-bound kernels per layer (K is read once; no float atomics, fixed summation order):
//   scores   s[row][h][j] = q[row][h] . k[j][h / G] / sqrt(dh)          for j <= pos(row)
//   norm     m[row][h] = log2(e) max_j s,  l[row][h] = sum_j exp2(log2(e) s - m)     (skipped when the attention
//            kernel, which computes the same pair for its own softmax, has written it)
//   add      s_inf[req][j] += sum_h exp2(log2(e) s[row][h][j] - m[row][h]) / l[row][h]   (h ascending)
// m is only a reference exponent: any value gives the same weights as long as l was summed against it.
#include "common.h"

namespace rc {

static constexpr int kInfThreads = 256;

// grid: (key chunks of kInfKeys, kv heads, rows).  dh / VEC consecutive lanes share one key row (each a
// 16-byte piece, so a row is read with one coalesced access), keep the matching pieces of the G query heads
// in registers, and add their partial dot products up with shuffles.  Key rows are requested kInfAhead
// passes at a time before the first of them is used.
static constexpr int kInfKeys = 512;
static constexpr int kInfAhead = 8;

template <typename T>
__global__ void __launch_bounds__(kInfThreads)
influence_scores_kernel(const T* __restrict__ q, const int* __restrict__ row_pos, const int* __restrict__ row_req,
                        const ReqTable* __restrict__ table, const T* __restrict__ k_pool, KvGeom g, int n_q_heads,
                        int max_len, float* __restrict__ scores) {
  constexpr int VEC = Vec16<T>::N;
  const int row = blockIdx.z, hk = blockIdx.y;
  const int G = n_q_heads / g.n_kv_heads, dh = g.head_dim;
  const int pos = row_pos[row];
  const int j0 = blockIdx.x * kInfKeys;
  if (j0 > pos) return;
  const int lpr = dh / VEC;                  // lanes per key row: 16 or 32
  const int sub = threadIdx.x % lpr;         // my 16-byte piece of the row
  const int keys_per_pass = kInfThreads / lpr;
  const float scale = rsqrtf((float)dh);
  const int seq = table->r[row_req[row] & kRowReqMask].dst_seq;
  const int j_end = min(j0 + kInfKeys, pos + 1);
  const bool contig = g.max_blocks == 1;     // one block per sequence: rows are a linear function of the position
  const T* kbase = contig ? k_pool + kv_row_offset(g, seq, 0, hk) + sub * VEC : nullptr;
  float qv[8][VEC];
#pragma unroll
  for (int gq = 0; gq < 8; ++gq) {
    if (gq < G) {
      Vec16<T>::load(q + ((size_t)row * n_q_heads + (size_t)hk * G + gq) * dh + sub * VEC, qv[gq]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) qv[gq][e] *= scale;
    }
  }
  float* srow = scores + ((size_t)row * n_q_heads + (size_t)hk * G) * max_len;
  for (int jb = j0 + threadIdx.x / lpr; jb < j_end + keys_per_pass; jb += kInfAhead * keys_per_pass) {
    if (jb - (int)(threadIdx.x / lpr) >= j_end) break;       // uniform: the whole pass group is past the end
    float kv[kInfAhead][VEC];
#pragma unroll
    for (int p = 0; p < kInfAhead; ++p) {
      const int j = jb + p * keys_per_pass;
      if (j < j_end) Vec16<T>::load(contig ? kbase + (size_t)j * dh : k_pool + kv_row_offset(g, seq, j, hk) + sub * VEC, kv[p]);
      else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) kv[p][e] = 0.f;
      }
    }
#pragma unroll
    for (int p = 0; p < kInfAhead; ++p) {
      const int j = jb + p * keys_per_pass;
#pragma unroll
      for (int gq = 0; gq < 8; ++gq) {
        if (gq < G) {
          float acc = 0.f;
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc = fmaf(qv[gq][e], kv[p][e], acc);
          for (int o = lpr >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
          if (j < j_end && sub == 0) srow[(size_t)gq * max_len + j] = acc;
        }
      }
    }
  }
}

// grid: (query heads, rows)
__global__ void __launch_bounds__(kInfThreads)
influence_norm_kernel(const float* __restrict__ scores, const int* __restrict__ row_pos, int n_q_heads, int max_len,
                      float2* __restrict__ ml) {
  __shared__ float red[kInfThreads / 64];
  const int h = blockIdx.x, row = blockIdx.y;
  const int n = row_pos[row] + 1;
  const float* s = scores + ((size_t)row * n_q_heads + h) * max_len;
  constexpr float kLog2e = 1.4426950408889634f;
  float m = -INFINITY;
  for (int j = threadIdx.x; j < n; j += kInfThreads) m = fmaxf(m, s[j] * kLog2e);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float l = 0.f;
  for (int j = threadIdx.x; j < n; j += kInfThreads) l += __builtin_amdgcn_exp2f(s[j] * kLog2e - m);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = l;
  __syncthreads();
  if (threadIdx.x == 0) ml[(size_t)row * n_q_heads + h] = make_float2(m, ((red[0] + red[1]) + red[2]) + red[3]);
}

// grid: (key chunks of 256, rows)
__global__ void __launch_bounds__(kInfThreads)
influence_add_kernel(const float* __restrict__ scores, const float2* __restrict__ ml, const int* __restrict__ row_pos,
                     const int* __restrict__ row_req, InfluencePtrs out, int n_q_heads, int max_len) {
  const int row = blockIdx.y;
  const int j = blockIdx.x * kInfThreads + threadIdx.x;
  if (j > row_pos[row]) return;
  float* dst = out.s_inf[row_req[row] & kRowReqMask];
  if (dst == nullptr) return;
  float acc = 0.f;
  for (int h = 0; h < n_q_heads; ++h) {
    const float2 t = ml[(size_t)row * n_q_heads + h];
    acc += __builtin_amdgcn_exp2f(scores[((size_t)row * n_q_heads + h) * max_len + j] * 1.4426950408889634f - t.x) / t.y;
  }
  dst[j] += acc;
}

size_t influence_scratch_floats(int n_rows, int n_q_heads, int max_len) {
  // scores [rows][Hq][max_len] followed by (m, l) pairs [rows][Hq]
  return (size_t)n_rows * n_q_heads * max_len + 2 * (size_t)n_rows * n_q_heads + 64;
}

template <typename T>
hipError_t launch_influence_scores(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                   int n_rows, const T* k_pool, KvGeom g, int n_q_heads, int max_len, float* scratch,
                                   hipStream_t st) {
  if (n_rows <= 0 || max_len <= 0) return hipSuccess;
  if (n_q_heads / g.n_kv_heads > 8) return hipErrorInvalidValue;
  const unsigned key_chunks = (unsigned)((max_len + kInfKeys - 1) / kInfKeys);
  influence_scores_kernel<T><<<dim3(key_chunks, (unsigned)g.n_kv_heads, (unsigned)n_rows), kInfThreads, 0, st>>>(
      q, row_pos, row_req, table, k_pool, g, n_q_heads, max_len, scratch);
  return hipGetLastError();
}
template hipError_t launch_influence_scores<float>(const float*, const int*, const int*, const ReqTable*, int,
                                                   const float*, KvGeom, int, int, float*, hipStream_t);
template hipError_t launch_influence_scores<bf16>(const bf16*, const int*, const int*, const ReqTable*, int,
                                                  const bf16*, KvGeom, int, int, float*, hipStream_t);

hipError_t launch_influence_finish(const int* row_pos, const int* row_req, int n_rows, int n_q_heads, int max_len,
                                   const InfluencePtrs& out, float* scratch, bool have_pairs, hipStream_t st) {
  if (n_rows <= 0 || max_len <= 0) return hipSuccess;
  float2* ml = influence_pairs(scratch, n_rows, n_q_heads, max_len);
  const unsigned chunks = (unsigned)((max_len + kInfThreads - 1) / kInfThreads);
  if (!have_pairs)
    influence_norm_kernel<<<dim3((unsigned)n_q_heads, (unsigned)n_rows), kInfThreads, 0, st>>>(scratch, row_pos, n_q_heads,
                                                                                             max_len, ml);
  influence_add_kernel<<<dim3(chunks, (unsigned)n_rows), kInfThreads, 0, st>>>(scratch, ml, row_pos, row_req, out,
                                                                               n_q_heads, max_len);
  return hipGetLastError();
}

}  // namespace rc
