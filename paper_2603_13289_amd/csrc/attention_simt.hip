// K6 for the float configuration: causal grouped-query attention of arbitrary query rows over a paged
// cache on the vector ALUs.  One wavefront (= one workgroup) per (query row, query head); keys are
// consumed 64 at a time with a running softmax.  bf16 models use the MFMA kernel instead.
#include "common.h"

namespace rc {

template <typename T>
__global__ void __launch_bounds__(64)
attn_simt_kernel(const T* __restrict__ q, const int* __restrict__ row_pos, const int* __restrict__ row_req,
                 const ReqTable* __restrict__ table, int fixed_seq, const T* __restrict__ k_pool,
                 const T* __restrict__ v_pool, KvGeom g, int n_q_heads, T* __restrict__ out) {
  constexpr int VEC = Vec16<T>::N;
  __shared__ float q_s[128];
  __shared__ float p_s[64];
  const int lane = threadIdx.x;
  const int r = blockIdx.x / n_q_heads, hq = blockIdx.x - r * n_q_heads;
  if (table && r >= table->total_rows) return;   // the grid may be sized for an upper bound of the row count
  const int kvh = hq / (n_q_heads / g.n_kv_heads);
  const int dh = g.head_dim;
  const int pos = row_pos[r];
  const int seq = table ? table->r[row_req[r] & kRowReqMask].dst_seq : fixed_seq;
  const T* qrow = q + ((size_t)r * n_q_heads + hq) * dh;
  for (int c = lane; c < dh; c += 64) q_s[c] = to_f32(qrow[c]);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)dh);
  float m = -INFINITY, l = 0.f, acc[2] = {0.f, 0.f};
  for (int t0 = 0; t0 <= pos; t0 += 64) {
    const int t = t0 + lane;
    float s = -INFINITY;
    if (t <= pos) {
      const T* krow = k_pool + kv_row_offset(g, seq, t, kvh);
      float d = 0.f;
      for (int c = 0; c < dh; c += VEC) {
        float kv[VEC];
        Vec16<T>::load(krow + c, kv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) d = fmaf(q_s[c + e], kv[e], d);
      }
      s = d * scale;
    }
    float mx = s;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float m_new = fmaxf(m, mx);
    const float p = (t <= pos) ? expf(s - m_new) : 0.f;
    const float corr = expf(m - m_new);
    float ps = p;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
    l = l * corr + ps;
    m = m_new;
    p_s[lane] = p;
    __syncthreads();
    acc[0] *= corr;
    acc[1] *= corr;
    const int nt = min(64, pos - t0 + 1);
    for (int tt = 0; tt < nt; ++tt) {
      const T* vrow = v_pool + kv_row_offset(g, seq, t0 + tt, kvh);
      const float pw = p_s[tt];
      if (lane < dh) acc[0] = fmaf(pw, to_f32(vrow[lane]), acc[0]);
      if (lane + 64 < dh) acc[1] = fmaf(pw, to_f32(vrow[lane + 64]), acc[1]);
    }
    __syncthreads();
  }
  T* orow = out + ((size_t)r * n_q_heads + hq) * dh;
  if (lane < dh) orow[lane] = from_f32<T>(acc[0] / l);
  if (lane + 64 < dh) orow[lane + 64] = from_f32<T>(acc[1] / l);
}

template <typename T>
hipError_t launch_attention_simt(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                 int fixed_seq, int total_rows, const T* k_pool, const T* v_pool, KvGeom g,
                                 int n_q_heads, T* out, hipStream_t st) {
  if (total_rows <= 0) return hipSuccess;
  attn_simt_kernel<T><<<(unsigned)(total_rows * n_q_heads), 64, 0, st>>>(q, row_pos, row_req, table, fixed_seq,
                                                                        k_pool, v_pool, g, n_q_heads, out);
  return hipGetLastError();
}
template hipError_t launch_attention_simt<float>(const float*, const int*, const int*, const ReqTable*, int, int,
                                                 const float*, const float*, KvGeom, int, float*, hipStream_t);
template hipError_t launch_attention_simt<bf16>(const bf16*, const int*, const int*, const ReqTable*, int, int,
                                                const bf16*, const bf16*, KvGeom, int, bf16*, hipStream_t);


template <>
hipError_t launch_attention<float>(const float* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                   int fixed_seq, int total_rows, int total_tiles, const float* k_pool,
                                   const float* v_pool, KvGeom g, int n_q_heads, float* out, hipStream_t st) {
  (void)total_tiles;
  return launch_attention_simt<float>(q, row_pos, row_req, table, fixed_seq, total_rows, k_pool, v_pool, g,
                                      n_q_heads, out, st);
}

int attention_tile_rows(int dtype, int n_q_heads, int n_kv_heads) {
  (void)dtype; (void)n_q_heads; (void)n_kv_heads;
  return 32;
}

}  // namespace rc
