// Bandwidth-bound stages of the selective-recompute prefill: rotary re-rotation of reused keys,
// active-row bookkeeping, RMSNorm, rotary + paged scatter of fresh K/V, Eq. (1) scoring.
#include "common.h"

namespace rc {

static constexpr int kThreads = 256;

// ------------------------------------------------------------------ request table upload
// The table travels as a kernel argument and is copied to device memory by the kernel itself,
// so no host-to-device copy (and no pinned staging buffer) is needed.
__global__ void upload_table_kernel(ReqTable t, ReqTable* dst) {
  const int* s = reinterpret_cast<const int*>(&t);
  int* d = reinterpret_cast<int*>(dst);
  for (int i = threadIdx.x; i < (int)(sizeof(ReqTable) / sizeof(int)); i += blockDim.x) d[i] = s[i];
}

hipError_t launch_upload_table(const ReqTable& host_table, ReqTable* dev_slot, hipStream_t st) {
  upload_table_kernel<<<1, kThreads, 0, st>>>(host_table, dev_slot);
  return hipGetLastError();
}

// ------------------------------------------------------------------ threshold selector: tables from device counts
// One thread (a few dozen requests at most).  tabs[PH_C] and tabs[PH_D] arrive with their static fields and with
// every token counted as selected; the counts the selector left in sel_cnt replace that, and everything that
// depends on them (row counts, row and tile offsets, links to the phase before, attention slots) is recomputed
// with the same functions the host uses when it knows the counts.
__global__ void finalize_tables_kernel(ReqTable* tabs, const int* __restrict__ sel_cnt, int tile_rows, int kv_tile,
                                       int thr_c, int chunks_c, int cap_c, int thr_d, int chunks_d, int cap_d) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  ReqTable* c = tabs + PH_C;
  ReqTable* dd = tabs + PH_D;
  for (int b = 0; b < c->n_req; ++b) {
    if (c->r[b].k <= 0) continue;            // a request without a segment takes no part in the selection
    const int k = min(max(sel_cnt[b], 0), c->r[b].S);
    c->r[b].k = k;
    dd->r[b].k = k;
  }
  fill_phase_table(c, PH_C, tabs + PH_B, tile_rows);
  assign_split_slots(c, tile_rows, kv_tile, thr_c, chunks_c, cap_c);
  fill_phase_table(dd, PH_D, c, tile_rows);
  assign_split_slots(dd, tile_rows, kv_tile, thr_d, chunks_d, cap_d);
}

hipError_t launch_finalize_tables(ReqTable* tabs, const int* sel_cnt, int tile_rows, int kv_tile, int thr_c,
                                  int chunks_c, int cap_c, int thr_d, int chunks_d, int cap_d, hipStream_t st) {
  finalize_tables_kernel<<<1, 64, 0, st>>>(tabs, sel_cnt, tile_rows, kv_tile, thr_c, chunks_c, cap_c, thr_d, chunks_d, cap_d);
  return hipGetLastError();
}

// ------------------------------------------------------------------ rotary tables
// tab[pos][i] = (cos, sin)(pos * base^(-2i/dh)), evaluated in double so that positions in the tens
// of thousands keep full float accuracy.
__global__ void rope_table_kernel(float2* tab, int n_pos, int half, double base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pos * half) return;
  const int pos = idx / half, i = idx - pos * half;
  const double theta = pow(base, -(double)i / (double)half);   // -2i/dh with dh = 2*half
  double s, c;
  sincos((double)pos * theta, &s, &c);
  tab[idx] = make_float2((float)c, (float)s);
}

hipError_t launch_rope_table(float2* tab, int n_pos, int half, double base, hipStream_t st) {
  const int n = n_pos * half;
  if (n <= 0) return hipSuccess;
  rope_table_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, st>>>(tab, n_pos, half, base);
  return hipGetLastError();
}

// tab[b][i] = (cos, sin)(rot_delta_b * theta_i): rotation that moves already-rotated keys
__global__ void delta_table_kernel(float2* tab, const ReqTable* table, int n_req, int half, double base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_req * half) return;
  const int b = idx / half, i = idx - b * half;
  const double theta = pow(base, -(double)i / (double)half);
  double s, c;
  sincos((double)table->r[b].rot_delta * theta, &s, &c);
  tab[idx] = make_float2((float)c, (float)s);
}

hipError_t launch_delta_table(float2* tab, const ReqTable* table, int n_req, int half, double base,
                              hipStream_t st) {
  const int n = n_req * half;
  if (n <= 0) return hipSuccess;
  delta_table_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, st>>>(tab, table, n_req, half, base);
  return hipGetLastError();
}

// ------------------------------------------------------------------ K1: re-rotate reused keys, copy values
// One thread moves two 16-byte chunks of one (token, head) row: elements [c, c+VEC) and their rotary
// partners [half+c, half+c+VEC).  grid.y = request, grid.z = layer (pool pointers travel in the
// kernel argument), so one launch takes over the segment in up to kRerotateLayers layers.
template <typename T>
__global__ void __launch_bounds__(kThreads)
rerotate_kernel(RerotatePtrs ptrs, KvGeom gs, KvGeom gd, const ReqTable* __restrict__ table,
                const float2* __restrict__ rope_tab, const float2* __restrict__ delta_tab) {
  constexpr int VEC = Vec16<T>::N;
  const T* __restrict__ k_src = reinterpret_cast<const T*>(ptrs.k_src[blockIdx.z]);
  const T* __restrict__ v_src = reinterpret_cast<const T*>(ptrs.v_src[blockIdx.z]);
  T* __restrict__ k_dst = reinterpret_cast<T*>(ptrs.k_dst[blockIdx.z]);
  T* __restrict__ v_dst = reinterpret_cast<T*>(ptrs.v_dst[blockIdx.z]);
  const ReqDev& rq = table->r[blockIdx.y];
  const int half = gs.head_dim / 2;
  const int tpr = half / VEC;  // threads per (token, head) row
  const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
  const int c = (int)(idx % tpr) * VEC;
  const long th = idx / tpr;
  const int head = (int)(th % gs.n_kv_heads);
  const long j = th / gs.n_kv_heads;
  if (j >= rq.S) return;
  const int new_pos = rq.pos0 + rq.P + (int)j;
  const size_t so = kv_row_offset(gs, rq.src_seq, rq.src_offset + (int)j, head);
  const size_t dof = kv_row_offset(gd, rq.dst_seq, new_pos, head);
  float lo[VEC], hi[VEC], olo[VEC], ohi[VEC];
  Vec16<T>::load(k_src + so + c, lo);
  Vec16<T>::load(k_src + so + half + c, hi);
  const float2* cs = rq.k_is_pre_rope ? rope_tab + (size_t)new_pos * half + c
                                      : delta_tab + (size_t)blockIdx.y * half + c;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    const float2 t = cs[e];
    olo[e] = lo[e] * t.x - hi[e] * t.y;
    ohi[e] = hi[e] * t.x + lo[e] * t.y;
  }
  Vec16<T>::store(k_dst + dof + c, olo);
  Vec16<T>::store(k_dst + dof + half + c, ohi);
  *reinterpret_cast<uint4*>(v_dst + dof + c) = *reinterpret_cast<const uint4*>(v_src + so + c);
  *reinterpret_cast<uint4*>(v_dst + dof + half + c) = *reinterpret_cast<const uint4*>(v_src + so + half + c);
}

template <typename T>
hipError_t launch_rerotate(const RerotatePtrs& ptrs, int n_layers, KvGeom gs, KvGeom gd, const ReqTable* table,
                           int n_req, int max_seg, const float2* rope_tab, const float2* delta_tab,
                           hipStream_t st) {
  if (max_seg <= 0 || n_req <= 0 || n_layers <= 0) return hipSuccess;
  const int tpr = (gs.head_dim / 2) / Vec16<T>::N;
  const long work = (long)max_seg * gs.n_kv_heads * tpr;
  dim3 grid((unsigned)((work + kThreads - 1) / kThreads), (unsigned)n_req, (unsigned)n_layers);
  rerotate_kernel<T><<<grid, kThreads, 0, st>>>(ptrs, gs, gd, table, rope_tab, delta_tab);
  return hipGetLastError();
}
template hipError_t launch_rerotate<float>(const RerotatePtrs&, int, KvGeom, KvGeom, const ReqTable*, int, int,
                                           const float2*, const float2*, hipStream_t);
template hipError_t launch_rerotate<bf16>(const RerotatePtrs&, int, KvGeom, KvGeom, const ReqTable*, int, int,
                                          const float2*, const float2*, hipStream_t);

// ------------------------------------------------------------------ active-row bookkeeping
// Builds the compact residual-stream buffer of a new phase: one workgroup per destination row.
// Rows of a request are ordered by position: prefix, active segment rows, suffix.
template <typename T>
__global__ void __launch_bounds__(kThreads)
build_rows_kernel(const ReqTable* __restrict__ table, const float* __restrict__ h_old, float* __restrict__ h_new,
                  int* __restrict__ row_pos, int* __restrict__ row_req, const int* __restrict__ sel_idx, int d) {
  const int r = blockIdx.x;
  if (r >= table->total_rows) return;   // the grid may be sized for an upper bound of the row count
  int b = 0;
  while (b + 1 < table->n_req && r >= table->r[b].row_base + table->r[b].n_rows) ++b;
  const ReqDev& rq = table->r[b];
  const int i = r - rq.row_base;
  int pos, flags = 0;
  const T* src_t = nullptr;      // input tensor row (T)
  const float* src_f = nullptr;  // row of the previous phase's buffer
  if (i < rq.P) {
    pos = rq.pos0 + i;
    if (rq.has_old) src_f = h_old + (size_t)(rq.old_row_base + i) * d;
    else src_t = reinterpret_cast<const T*>(rq.x_prefix) + (size_t)i * d;
  } else if (i < rq.P + rq.n_seg_rows) {
    const int si = i - rq.P;
    int j;
    if (rq.seg_mode == SEG_ALL) j = si;
    else if (rq.seg_mode == SEG_SEL) {
      j = (si < rq.k) ? sel_idx[rq.sel_base + si] : rq.S - 1;
      // the extra row of the last token, when the (ascending) selection ends with that token as well
      if (si >= rq.k && rq.k > 0 && sel_idx[rq.sel_base + rq.k - 1] == rq.S - 1) flags = kRowNoCacheWrite;
    } else j = rq.S - 1;
    j = min(max(j, 0), rq.S - 1);
    pos = rq.pos0 + rq.P + j;
    if (rq.old_seg_mode == SEG_ALL) src_f = h_old + (size_t)(rq.old_row_base + rq.P + j) * d;
    else if (rq.old_seg_mode == SEG_SEL) src_f = h_old + (size_t)(rq.old_row_base + rq.P + rq.old_n_seg_rows - 1) * d;
    else if (rq.old_seg_mode == SEG_LAST) src_f = h_old + (size_t)(rq.old_row_base + rq.P) * d;
    else src_t = reinterpret_cast<const T*>(rq.h_start) + (size_t)j * d;
  } else {
    const int si = i - rq.P - rq.n_seg_rows;
    pos = rq.pos0 + rq.P + rq.S + si;
    if (rq.has_old) src_f = h_old + (size_t)(rq.old_row_base + rq.P + rq.old_n_seg_rows + si) * d;
    else src_t = reinterpret_cast<const T*>(rq.x_suffix) + (size_t)si * d;
  }
  if (threadIdx.x == 0) {
    row_pos[r] = pos;
    row_req[r] = b | flags;
  }
  float* dst = h_new + (size_t)r * d;
  if (src_f) {
    for (int c = threadIdx.x * 4; c < d; c += kThreads * 4)
      *reinterpret_cast<float4*>(dst + c) = *reinterpret_cast<const float4*>(src_f + c);
  } else {
    for (int c = threadIdx.x; c < d; c += kThreads) dst[c] = to_f32(src_t[c]);
  }
}

template <typename T>
hipError_t launch_build_rows(const ReqTable* table, int total_rows, const float* h_old, float* h_new,
                             int* row_pos, int* row_req, const int* sel_idx, int d, hipStream_t st) {
  if (total_rows <= 0) return hipSuccess;
  build_rows_kernel<T><<<total_rows, kThreads, 0, st>>>(table, h_old, h_new, row_pos, row_req, sel_idx, d);
  return hipGetLastError();
}
template hipError_t launch_build_rows<float>(const ReqTable*, int, const float*, float*, int*, int*, const int*,
                                             int, hipStream_t);
template hipError_t launch_build_rows<bf16>(const ReqTable*, int, const float*, float*, int*, int*, const int*,
                                            int, hipStream_t);

// hidden states entering a layer, written out per request in T (what the cache manager keeps)
template <typename T>
__global__ void __launch_bounds__(kThreads)
capture_rows_kernel(const ReqTable* __restrict__ table, const float* __restrict__ h,
                    const int* __restrict__ row_req, int d) {
  const int r = blockIdx.x;
  if (r >= table->total_rows) return;
  const ReqDev& rq = table->r[row_req[r] & kRowReqMask];
  if (rq.h_capture == nullptr) return;
  T* dst = reinterpret_cast<T*>(rq.h_capture) + (size_t)(r - rq.row_base) * d;
  const float* src = h + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += kThreads) dst[c] = from_f32<T>(src[c]);
}

template <typename T>
hipError_t launch_capture_rows(const ReqTable* table, int total_rows, const float* h, const int* row_req,
                               int d, hipStream_t st) {
  if (total_rows <= 0) return hipSuccess;
  capture_rows_kernel<T><<<total_rows, kThreads, 0, st>>>(table, h, row_req, d);
  return hipGetLastError();
}
template hipError_t launch_capture_rows<float>(const ReqTable*, int, const float*, const int*, int, hipStream_t);
template hipError_t launch_capture_rows<bf16>(const ReqTable*, int, const float*, const int*, int, hipStream_t);

// ------------------------------------------------------------------ block reduction helper
__device__ inline float block_sum(float v, float* lds /* >= 4 floats */) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds[w] = v;
  __syncthreads();
  float s = 0.f;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) s += lds[i];
  return s;
}

// four consecutive elements of T from / to four floats
__device__ inline void store4(float* p, const float* v) { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
__device__ inline void store4(bf16* p, const float* v) {
  uint2 pk;
  pk.x = (uint32_t)f32_to_bf16(v[0]).v | ((uint32_t)f32_to_bf16(v[1]).v << 16);
  pk.y = (uint32_t)f32_to_bf16(v[2]).v | ((uint32_t)f32_to_bf16(v[3]).v << 16);
  *reinterpret_cast<uint2*>(p) = pk;
}
__device__ inline void load4(const float* p, float* v) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ inline void load4(const bf16* p, float* v) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}

// ------------------------------------------------------------------ K2: RMSNorm on the active rows
// One workgroup per row; the row stays in registers between the sum of squares and the scaling when it is
// at most kNormKeep floats per thread (d <= 8192), else it is read again.
constexpr int kNormKeep = 8;
template <typename T>
__global__ void __launch_bounds__(kThreads)
rmsnorm_kernel(const float* __restrict__ h, const T* __restrict__ gain, T* __restrict__ out, int d, float eps,
               const int* __restrict__ m_live) {
  __shared__ float red[kThreads / 64];
  if (m_live && (int)blockIdx.x >= *m_live) return;
  const float* x = h + (size_t)blockIdx.x * d;
  float4 keep[kNormKeep];
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < kNormKeep; ++u) {
    const int c = (threadIdx.x + u * kThreads) * 4;
    if (c < d) {
      keep[u] = *reinterpret_cast<const float4*>(x + c);
      ss += keep[u].x * keep[u].x + keep[u].y * keep[u].y + keep[u].z * keep[u].z + keep[u].w * keep[u].w;
    }
  }
  for (int c = (threadIdx.x + kNormKeep * kThreads) * 4; c < d; c += kThreads * 4) {
    const float4 v = *reinterpret_cast<const float4*>(x + c);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  T* o = out + (size_t)blockIdx.x * d;
#pragma unroll
  for (int u = 0; u < kNormKeep; ++u) {
    const int c = (threadIdx.x + u * kThreads) * 4;
    if (c < d) {
      float gv[4];
      load4(gain + c, gv);
      const float y[4] = {keep[u].x * r * gv[0], keep[u].y * r * gv[1], keep[u].z * r * gv[2], keep[u].w * r * gv[3]};
      store4(o + c, y);
    }
  }
  for (int c = (threadIdx.x + kNormKeep * kThreads) * 4; c < d; c += kThreads * 4) {
    const float4 v = *reinterpret_cast<const float4*>(x + c);
    float gv[4];
    load4(gain + c, gv);
    const float y[4] = {v.x * r * gv[0], v.y * r * gv[1], v.z * r * gv[2], v.w * r * gv[3]};
    store4(o + c, y);
  }
}

template <typename T>
hipError_t launch_rmsnorm(const float* h, const T* gain, T* out, int rows, int d, float eps, hipStream_t st,
                          const int* m_live) {
  if (rows <= 0) return hipSuccess;
  rmsnorm_kernel<T><<<rows, kThreads, 0, st>>>(h, gain, out, d, eps, m_live);
  return hipGetLastError();
}
template hipError_t launch_rmsnorm<float>(const float*, const float*, float*, int, int, float, hipStream_t, const int*);
template hipError_t launch_rmsnorm<bf16>(const float*, const bf16*, bf16*, int, int, float, hipStream_t, const int*);

// ------------------------------------------------------------------ rotary on fresh q/k + K7: paged scatter
// One workgroup per live row.  qkv is the float output of the three projections laid out
// [row][Hq*dh | Hkv*dh | Hkv*dh].  A work item is four consecutive rotary pairs of one head (q or k) or four
// consecutive value elements, so every access is 16 bytes of float or 8 bytes of bf16.
template <typename T>
__global__ void __launch_bounds__(kThreads)
rope_scatter_kernel(const float* __restrict__ qkv, const int* __restrict__ row_pos, const int* __restrict__ row_req,
                    const ReqTable* __restrict__ table, const float2* __restrict__ rope_tab, T* __restrict__ q_out,
                    T* __restrict__ k_pool, T* __restrict__ v_pool, T* __restrict__ k_pre_pool, KvGeom g,
                    int n_q_heads) {
  const int r = blockIdx.x;
  if (r >= table->total_rows) return;
  const int pos = row_pos[r];
  const int rr = row_req ? row_req[r] : 0;     // no per-row request array: all rows belong to request 0
  const int seq = table->r[rr & kRowReqMask].dst_seq;
  const bool write_cache = (rr & kRowNoCacheWrite) == 0;
  const int dh = g.head_dim, half = dh / 2, quads = half / 4;
  const int nq = n_q_heads * dh, nkv = g.n_kv_heads * dh;
  const float* row = qkv + (size_t)r * (nq + 2 * nkv);
  const float2* cs = rope_tab + (size_t)pos * half;
  const int n_rot = (n_q_heads + g.n_kv_heads) * quads;    // query heads first, then key heads
  const int n_val = g.n_kv_heads * (dh / 4);
  for (int item = threadIdx.x; item < n_rot + n_val; item += kThreads) {
    if (item < n_rot) {
      const int head = item / quads, i = (item - head * quads) * 4;
      const bool is_q = head < n_q_heads;
      const float* src = row + (is_q ? head * dh : nq + (head - n_q_heads) * dh);
      const float4 a4 = *reinterpret_cast<const float4*>(src + i);
      const float4 b4 = *reinterpret_cast<const float4*>(src + half + i);
      const float4 t01 = *reinterpret_cast<const float4*>(cs + i);        // (cos, sin) of pairs i, i+1
      const float4 t23 = *reinterpret_cast<const float4*>(cs + i + 2);    // pairs i+2, i+3
      const float a[4] = {a4.x, a4.y, a4.z, a4.w}, b[4] = {b4.x, b4.y, b4.z, b4.w};
      const float c[4] = {t01.x, t01.z, t23.x, t23.z}, sn[4] = {t01.y, t01.w, t23.y, t23.w};
      float lo[4], hi[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lo[e] = a[e] * c[e] - b[e] * sn[e];
        hi[e] = b[e] * c[e] + a[e] * sn[e];
      }
      if (is_q) {
        T* o = q_out + (size_t)r * nq + head * dh;
        store4(o + i, lo);
        store4(o + half + i, hi);
      } else if (write_cache) {
        // rotated into the cache (and optionally un-rotated into the pre-RoPE pool)
        const size_t off = kv_row_offset(g, seq, pos, head - n_q_heads);
        store4(k_pool + off + i, lo);
        store4(k_pool + off + half + i, hi);
        if (k_pre_pool) {
          store4(k_pre_pool + off + i, a);
          store4(k_pre_pool + off + half + i, b);
        }
      }
    } else if (write_cache) {
      const int vi = item - n_rot;
      const int head = vi / (dh / 4), i = (vi - head * (dh / 4)) * 4;
      const float4 v4 = *reinterpret_cast<const float4*>(row + nq + nkv + head * dh + i);
      const float v[4] = {v4.x, v4.y, v4.z, v4.w};
      store4(v_pool + kv_row_offset(g, seq, pos, head) + i, v);
    }
  }
}

template <typename T>
hipError_t launch_rope_scatter(const float* qkv, int n_rows, const int* row_pos, const int* row_req,
                               const ReqTable* table, const float2* rope_tab, T* q_out, T* k_pool, T* v_pool,
                               T* k_pre_pool, KvGeom g, int n_q_heads, hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  rope_scatter_kernel<T><<<n_rows, kThreads, 0, st>>>(qkv, row_pos, row_req, table, rope_tab, q_out, k_pool,
                                                      v_pool, k_pre_pool, g, n_q_heads);
  return hipGetLastError();
}
template hipError_t launch_rope_scatter<float>(const float*, int, const int*, const int*, const ReqTable*,
                                               const float2*, float*, float*, float*, float*, KvGeom, int,
                                               hipStream_t);
template hipError_t launch_rope_scatter<bf16>(const float*, int, const int*, const int*, const ReqTable*,
                                              const float2*, bf16*, bf16*, bf16*, bf16*, KvGeom, int, hipStream_t);

// K7 as a stand-alone stage: rows already in T, keys already rotated
template <typename T>
__global__ void __launch_bounds__(kThreads)
scatter_rows_kernel(const T* __restrict__ k_rows, const T* __restrict__ v_rows, const int* __restrict__ pos, int n,
                    T* __restrict__ k_pool, T* __restrict__ v_pool, KvGeom g, int seq) {
  constexpr int VEC = Vec16<T>::N;
  const int cpr = g.head_dim / VEC;  // 16-byte chunks per (row, head)
  const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
  const int c = (int)(idx % cpr) * VEC;
  const long rh = idx / cpr;
  const int head = (int)(rh % g.n_kv_heads);
  const long i = rh / g.n_kv_heads;
  if (i >= n) return;
  const size_t so = ((size_t)i * g.n_kv_heads + head) * g.head_dim + c;
  const size_t dof = kv_row_offset(g, seq, pos[i], head) + c;
  *reinterpret_cast<uint4*>(k_pool + dof) = *reinterpret_cast<const uint4*>(k_rows + so);
  *reinterpret_cast<uint4*>(v_pool + dof) = *reinterpret_cast<const uint4*>(v_rows + so);
}

template <typename T>
hipError_t launch_scatter_rows(const T* k_rows, const T* v_rows, const int* pos, int n, T* k_pool, T* v_pool,
                               KvGeom g, int seq, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const long work = (long)n * g.n_kv_heads * (g.head_dim / Vec16<T>::N);
  scatter_rows_kernel<T><<<(unsigned)((work + kThreads - 1) / kThreads), kThreads, 0, st>>>(k_rows, v_rows, pos, n,
                                                                                          k_pool, v_pool, g, seq);
  return hipGetLastError();
}
template hipError_t launch_scatter_rows<float>(const float*, const float*, const int*, int, float*, float*, KvGeom,
                                               int, hipStream_t);
template hipError_t launch_scatter_rows<bf16>(const bf16*, const bf16*, const int*, int, bf16*, bf16*, KvGeom, int,
                                              hipStream_t);

// ------------------------------------------------------------------ K4: Eq. (1) deviation score
// One wavefront per segment token.  A lane owns 16-byte chunks of the token's [Hkv][dh] values;
// dh/VEC consecutive lanes cover one head, so a head's sums are reduced with shuffles inside that
// lane group, and the per-head deviations are then summed across groups.
//
// 1 - cos(a, b) is evaluated as 0.5 * |a/|a| - b/|b||^2, which is the same quantity without the
// cancellation of "1 - (number close to 1)": deviations of 1e-5 keep ~6 significant digits in float,
// which the ranking of tokens needs.  When |a||b| is below the 1e-12 floor the literal form
// 1 - a.b / 1e-12 is used, so a zero vector scores exactly 1.
template <typename T>
__global__ void __launch_bounds__(kThreads)
vdev_score_kernel(const T* __restrict__ v_fresh, int fresh_row_stride, const T* __restrict__ v_pool, KvGeom g,
                  const ReqTable* __restrict__ table, float* __restrict__ scores) {
  constexpr int VEC = Vec16<T>::N;
  const ReqDev& rq = table->r[blockIdx.y];
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (j >= rq.S || rq.seg_mode != SEG_ALL) return;   // only requests whose whole segment is live
  const int lph = g.head_dim / VEC;          // lanes per head (16 or 32)
  const int hpp = 64 / lph;                  // heads per pass
  const int sub = lane % lph, hslot = lane / lph;
  const T* fresh = v_fresh + (size_t)(rq.row_base + rq.P + j) * fresh_row_stride;
  float dev_sum = 0.f;
  // two passes of heads at a time, so that four 16-byte loads per lane are in flight before the first reduction
  for (int h0 = 0; h0 < g.n_kv_heads; h0 += 2 * hpp) {
    float a[2][VEC], b[2][VEC];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int head = h0 + u * hpp + hslot;
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[u][e] = b[u][e] = 0.f;
      if (head < g.n_kv_heads) {
        Vec16<T>::load(v_pool + kv_row_offset(g, rq.dst_seq, rq.pos0 + rq.P + j, head) + sub * VEC, a[u]);
        Vec16<T>::load(fresh + head * g.head_dim + sub * VEC, b[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int head = h0 + u * hpp + hslot;
      float dot = 0.f, na = 0.f, nb = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        dot += a[u][e] * b[u][e];
        na += a[u][e] * a[u][e];
        nb += b[u][e] * b[u][e];
      }
      for (int o = lph >> 1; o > 0; o >>= 1) {
        dot += __shfl_xor(dot, o, 64);
        na += __shfl_xor(na, o, 64);
        nb += __shfl_xor(nb, o, 64);
      }
      const float la = sqrtf(na), lb = sqrtf(nb);
      const bool floored = la * lb < 1e-12f;
      const float ra = floored ? 0.f : 1.0f / la, rb = floored ? 0.f : 1.0f / lb;
      float dd = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float t = a[u][e] * ra - b[u][e] * rb;
        dd += t * t;
      }
      for (int o = lph >> 1; o > 0; o >>= 1) dd += __shfl_xor(dd, o, 64);
      if (sub == 0 && head < g.n_kv_heads) dev_sum += floored ? 1.0f - dot / 1e-12f : 0.5f * dd;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) dev_sum += __shfl_xor(dev_sum, o, 64);
  if (lane == 0) scores[rq.score_base + j] = dev_sum / (float)g.n_kv_heads;
}

template <typename T>
hipError_t launch_vdev_score(const T* v_fresh, int fresh_row_stride, const T* v_pool, KvGeom g,
                             const ReqTable* table, int n_req, int max_seg, float* scores, hipStream_t st) {
  if (max_seg <= 0 || n_req <= 0) return hipSuccess;
  constexpr int tokens_per_block = kThreads / 64;
  dim3 grid((unsigned)((max_seg + tokens_per_block - 1) / tokens_per_block), (unsigned)n_req);
  vdev_score_kernel<T><<<grid, kThreads, 0, st>>>(v_fresh, fresh_row_stride, v_pool, g, table, scores);
  return hipGetLastError();
}
template hipError_t launch_vdev_score<float>(const float*, int, const float*, KvGeom, const ReqTable*, int, int,
                                             float*, hipStream_t);
template hipError_t launch_vdev_score<bf16>(const bf16*, int, const bf16*, KvGeom, const ReqTable*, int, int, float*,
                                            hipStream_t);

// ------------------------------------------------------------------ misc
__global__ void copy_i32_kernel(const int* __restrict__ src, int* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
hipError_t launch_copy_i32(const int* src, int* dst, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  copy_i32_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, st>>>(src, dst, n);
  return hipGetLastError();
}

// residual-stream row of each request's last position -> out[b][d]
__global__ void __launch_bounds__(kThreads)
gather_last_kernel(const ReqTable* __restrict__ table, const float* __restrict__ h, float* __restrict__ out, int d) {
  const ReqDev& rq = table->r[blockIdx.x];
  if (rq.n_rows <= 0) {   // a request without live rows in the last phase has no logits: defined zeros
    for (int c = threadIdx.x; c < d; c += kThreads) out[(size_t)blockIdx.x * d + c] = 0.f;
    return;
  }
  const float* src = h + (size_t)(rq.row_base + rq.n_rows - 1) * d;
  for (int c = threadIdx.x; c < d; c += kThreads) out[(size_t)blockIdx.x * d + c] = src[c];
}
hipError_t launch_gather_last(const ReqTable* table, int n_req, const float* h, float* out, int d, hipStream_t st) {
  if (n_req <= 0) return hipSuccess;
  gather_last_kernel<<<n_req, kThreads, 0, st>>>(table, h, out, d);
  return hipGetLastError();
}

}  // namespace rc
