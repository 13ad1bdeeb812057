// Shared device/host declarations of the selective-recompute prefill library (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/relaycache.h"

namespace rc {

// ------------------------------------------------------------------ element types
struct bf16 {
  uint16_t v;
};

__host__ __device__ inline float bf16_to_f32(bf16 x) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)x.v << 16;
  return c.f;
}
// round to nearest, ties to even; NaN stays NaN
__host__ __device__ inline bf16 f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  bf16 h;
  h.v = __builtin_bit_cast(uint16_t, (__bf16)f);   // hardware convert, same rounding
  return h;
#endif
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  bf16 r;
  if ((u & 0x7fffffffu) > 0x7f800000u) {
    r.v = (uint16_t)((u >> 16) | 0x0040u);
  } else {
    r.v = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
  return r;
}

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16 x) { return bf16_to_f32(x); }
template <typename T> __device__ inline T from_f32(float x);
template <> __device__ inline float from_f32<float>(float x) { return x; }
template <> __device__ inline bf16 from_f32<bf16>(float x) { return f32_to_bf16(x); }

// 16-byte vector access: VEC elements of T
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ inline void load(const float* p, float* out) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
  static __device__ inline void store(float* p, const float* in) {
    *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
  }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  static __device__ inline void load(const bf16* p, float* out) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ inline void store(bf16* p, const float* in) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[i] = (uint32_t)f32_to_bf16(in[2 * i]).v | ((uint32_t)f32_to_bf16(in[2 * i + 1]).v << 16);
    }
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// ------------------------------------------------------------------ paged cache geometry
struct KvGeom {
  int n_blocks, block_size;
  const int32_t* block_table;  // device [n_seq][max_blocks]
  int max_blocks;
  int n_kv_heads, head_dim;
  int bs_shift;  // log2(block_size) when it is a power of two, else -1
};

inline int log2_if_pow2(int x) {
  if (x <= 0 || (x & (x - 1))) return -1;
  int s = 0;
  while ((1 << s) < x) ++s;
  return s;
}

// element offset of (seq, pos, head, 0) inside one layer's pool; positions, table slots and block ids
// are clamped to the geometry, so bad indices read or write a wrong row but never leave the pool
__device__ inline size_t kv_row_offset(const KvGeom& g, int seq, int pos, int head) {
  pos = max(pos, 0);
  int bi, slot;
  if (g.max_blocks == 1) {            // contiguous cache: one block per sequence
    bi = 0;
    slot = min(pos, g.block_size - 1);
  } else if (g.bs_shift >= 0) {       // power-of-two pages: no integer division
    bi = min(pos >> g.bs_shift, g.max_blocks - 1);
    slot = min(pos - (bi << g.bs_shift), g.block_size - 1);
  } else {
    bi = min(pos / g.block_size, g.max_blocks - 1);
    slot = min(pos - bi * g.block_size, g.block_size - 1);
  }
  int blk = g.block_table[(size_t)seq * g.max_blocks + bi];
  blk = min(max(blk, 0), g.n_blocks - 1);
  return (((size_t)blk * g.n_kv_heads + head) * g.block_size + slot) * (size_t)g.head_dim;
}

// ------------------------------------------------------------------ per-request phase table
enum SegMode : int { SEG_NONE = 0, SEG_ALL = 1, SEG_SEL = 2, SEG_LAST = 3 };

struct ReqDev {
  int P, S, nsuf, k;
  int pos0;             // position of the request's first row (rows 0..pos0-1 of the sequence are already final)
  int carries_logits;   // 1: no suffix, so the last segment token stays live to the end and yields the logits
  int row_base, n_seg_rows, n_rows, seg_mode;           // current phase
  int old_row_base, old_n_seg_rows, old_seg_mode, has_old;  // phase being left (has_old = 0: inputs)
  int dst_seq, src_seq, src_offset, rot_delta;           // rot_delta valid when keys are rotated
  int sel_base, score_base, tile_base, k_is_pre_rope;
  int long_tile_start, part_base;   // attention KV split: first local tile that may be split, its slot base
  int item_base;                    // attention grid: first work item of this request (requests are served last to first)
  int merge_base;                   // merge grid: rows of the tiles that may be split, counted over the requests before this one
  const void* x_prefix;
  const void* h_start;
  const void* x_suffix;
  void* h_capture;
};

// row_req[r] holds the row's request index in its low bits and, for the one live row per request that is a second
// copy of a selected token (the logits-carrying last segment token when the selection already contains it), the
// flag below: such a row runs through the layers like any other but leaves the cache writes to its twin, so that
// the cache row has exactly one writer and the result does not depend on which of two bit-different sums lands last.
constexpr int kRowReqMask = 0xff;
constexpr int kRowNoCacheWrite = 0x100;
static_assert(RC_MAX_REQ <= kRowReqMask + 1, "request index must fit the mask");

struct ReqTable {
  int n_req, total_rows, total_tiles;
  int total_items;   // attention grid: work items = whole query tiles + (query tile, KV chunk) pairs of the tiles that may be split
  int total_merge_rows;   // rows of the tiles that may be split (the merge pass visits only those)
  int pad_[3];
  ReqDev r[RC_MAX_REQ];
};

// ------------------------------------------------------------------ phases of a call
// A: layers before l_start (new tokens only); B: dense detect layers [l_start, l_det) (all segment rows);
// C: sparse rectification [l_det, l_end] (selected rows); D: layers after l_end.
enum Phase : int { PH_A = 0, PH_B = 1, PH_C = 2, PH_D = 3, PH_COUNT = 4 };

// which segment rows of a request are live in a phase, and how many
__host__ __device__ inline void phase_seg_rows(const ReqDev& r, int ph, int* mode, int* n) {
  const int last = (r.carries_logits && r.S > 0) ? 1 : 0;
  if (ph == PH_B && r.k > 0) { *mode = SEG_ALL; *n = r.S; }
  else if (ph == PH_C && r.k > 0) { *mode = SEG_SEL; *n = r.k + last; }
  else if (ph == PH_A) { *mode = SEG_NONE; *n = 0; }
  else { *mode = last ? SEG_LAST : SEG_NONE; *n = last; }
}

// Fills the phase-dependent fields of a table whose static fields (P, S, nsuf, k, ...) are in place; `prev` is
// the table of the phase being left (nullptr at the start of a call).  Runs on the host when the row counts are
// known there, and on the device when they depend on a selection made on the device.
__host__ __device__ inline void fill_phase_table(ReqTable* t, int ph, const ReqTable* prev, int tile_rows) {
  int row = 0, tile = 0;
  for (int b = 0; b < t->n_req; ++b) {
    ReqDev& r = t->r[b];
    int mode, n;
    phase_seg_rows(r, ph, &mode, &n);
    r.seg_mode = mode;
    r.n_seg_rows = n;
    r.n_rows = r.P + n + r.nsuf;
    r.row_base = row;
    r.tile_base = tile;
    row += r.n_rows;
    tile += (r.n_rows + tile_rows - 1) / tile_rows;
    if (prev) {
      r.has_old = 1;
      r.old_row_base = prev->r[b].row_base;
      r.old_n_seg_rows = prev->r[b].n_seg_rows;
      r.old_seg_mode = prev->r[b].seg_mode;
    } else {
      r.has_old = 0;
      r.old_row_base = 0;
      r.old_n_seg_rows = 0;
      r.old_seg_mode = SEG_NONE;
    }
  }
  t->total_rows = row;
  t->total_tiles = tile;
}

// Attention KV split of one phase, per-request part: the first query tile of each request that may be split
// (a tile of new-prefix rows only has exactly known, short ranges and stays whole) and the request's base in the
// array of partial-result slots.  Returns the slots the phase needs; with more than `capacity` slots the split
// is switched off for the phase (every tile is then done by one workgroup) and 0 is returned.
__host__ __device__ inline int assign_split_slots(ReqTable* t, int tile_rows, int kv_tile, int long_thr, int n_chunks,
                                                  int capacity) {
  int base = 0;
  for (int b = 0; b < t->n_req; ++b) {
    ReqDev& r = t->r[b];
    const int tiles = (r.n_rows + tile_rows - 1) / tile_rows;
    int start = tiles;
    for (int j = 0; j < tiles; ++j) {
      const int i_last = ((j + 1) * tile_rows < r.n_rows ? (j + 1) * tile_rows : r.n_rows) - 1;
      if (i_last >= r.P || (r.pos0 + i_last) / kv_tile + 1 > long_thr) { start = j; break; }
    }
    r.long_tile_start = start;
    r.part_base = base;
    base += (tiles - start) * n_chunks;
  }
  const bool off = n_chunks <= 1 || base == 0 || base > capacity;
  if (off) {
    base = 0;
    for (int b = 0; b < t->n_req; ++b) {
      t->r[b].long_tile_start = 1 << 30;
      t->r[b].part_base = 0;
    }
  }
  // the attention grid: requests last to first, inside a request the tiles that may be split (the late, long ones:
  // one item per KV chunk) before the whole ones
  int items = 0;
  for (int b = t->n_req - 1; b >= 0; --b) {
    ReqDev& r = t->r[b];
    const int tiles = (r.n_rows + tile_rows - 1) / tile_rows;
    const int start = r.long_tile_start < tiles ? r.long_tile_start : tiles;
    r.item_base = items;
    items += (tiles - start) * (off ? 1 : n_chunks) + start;
  }
  t->total_items = items;
  int mrows = 0;
  for (int b = 0; b < t->n_req; ++b) {
    ReqDev& r = t->r[b];
    r.merge_base = mrows;
    const long first = (long)r.long_tile_start * tile_rows;
    if (first < r.n_rows) mrows += r.n_rows - (int)first;
  }
  t->total_merge_rows = mrows;
  return base;
}

// Row count of a launch: the host's figure, or, when the count is only known on the device (rows selected by a
// threshold), the device value, of which the host's figure is an upper bound that sized the grid.
__device__ inline int live_count(int bound, const int* live) { return live ? min(bound, *live) : bound; }

// ------------------------------------------------------------------ launchers (host)
// Every launcher enqueues on `st` and returns hipGetLastError().
hipError_t launch_upload_table(const ReqTable& host_table, ReqTable* dev_slot, hipStream_t st);
hipError_t launch_rope_table(float2* tab, int n_pos, int half, double base, hipStream_t st);
hipError_t launch_delta_table(float2* tab, const ReqTable* table, int n_req, int half, double base,
                              hipStream_t st);

// pool pointers of up to kRerotateLayers layers, passed to the re-rotation kernel by value
constexpr int kRerotateLayers = 32;
struct RerotatePtrs {
  const void* k_src[kRerotateLayers];
  const void* v_src[kRerotateLayers];
  void* k_dst[kRerotateLayers];
  void* v_dst[kRerotateLayers];
};
template <typename T>
hipError_t launch_rerotate(const RerotatePtrs& ptrs, int n_layers, KvGeom gs, KvGeom gd, const ReqTable* table,
                           int n_req, int max_seg, const float2* rope_tab, const float2* delta_tab, hipStream_t st);

template <typename T>
hipError_t launch_build_rows(const ReqTable* table, int total_rows, const float* h_old, float* h_new,
                             int* row_pos, int* row_req, const int* sel_idx, int d, hipStream_t st);
template <typename T>
hipError_t launch_capture_rows(const ReqTable* table, int total_rows, const float* h, const int* row_req,
                               int d, hipStream_t st);

// m_live (optional, device): the live row count when `rows` is only an upper bound
template <typename T>
hipError_t launch_rmsnorm(const float* h, const T* gain, T* out, int rows, int d, float eps, hipStream_t st,
                          const int* m_live = nullptr);

enum GemmEpilogue : int { EPI_STORE_F32 = 0, EPI_STORE_T = 1, EPI_ADD_F32 = 2, EPI_SWIGLU_T = 3 };
// C[M][ldc] (op)= A[M][K] * W[N][K]^T ; W2 only for EPI_SWIGLU_T (gate = W, up = W2)
// m_live (optional, device): the live row count when m is only an upper bound (rows selected on the device);
// the launch then covers m rows' worth of tiles and workgroups past the live rows leave at once
template <typename T>
hipError_t launch_gemm(const T* a, const T* w, const T* w2, void* c, int m, int n, int k, int ldc,
                       GemmEpilogue epi, hipStream_t st, const int* m_live = nullptr);

// few-row variant (M <= 32, weights streamed once); columns < ns1 come from w, < ns2 from w2, the rest from w3
bool gemm_skinny_applies(int m, int n, int k, int ns1, int ns2);
hipError_t launch_gemm_skinny_bf16(const bf16* a, const bf16* w, const bf16* w2, const bf16* w3, int ns1, int ns2,
                                   void* c, int m, int n, int k, int ldc, GemmEpilogue epi, hipStream_t st,
                                   const int* m_live = nullptr);

// C[M][nq + 2 nkv] (float) = A * [wq; wk; wv]^T
template <typename T>
hipError_t launch_gemm_qkv(const T* a, const T* wq, int nq, const T* wk, const T* wv, int nkv, float* c, int m,
                           int k, hipStream_t st, const int* m_live = nullptr);

// bf16 GEMMs with a scratch buffer (gemm_partial_bytes()) for the K-split tail of the tile schedule;
// partial == nullptr: every tile is done by one workgroup.
size_t gemm_partial_bytes();
hipError_t launch_gemm_bf16(const bf16* a, const bf16* w, const bf16* w2, void* c, int m, int n, int k, int ldc,
                            GemmEpilogue epi, float* partial, hipStream_t st, const int* m_live = nullptr);
hipError_t launch_gemm_qkv_bf16(const bf16* a, const bf16* wq, int nq, const bf16* wk, const bf16* wv, int nkv, float* c,
                                int m, int k, float* partial, hipStream_t st, const int* m_live = nullptr);
void set_gemm_xcd_remap(int on);
int check_grid_plan(int m, int n, int k, bool dual, int tile, int n_cus, bool with_partial, int* n_blocks_out);
void set_gemm_thin_tiles(int on);   // 1: a ragged last tile row of at most 64 rows goes to the thin tile body
void set_gemm_tile(int t);  // 0: by shape; 1-3 register-staged tiles; 5-7 direct-to-LDS tiles (bf16 MFMA GEMM)

template <typename T>
hipError_t launch_rope_scatter(const float* qkv, int n_rows, const int* row_pos, const int* row_req,
                               const ReqTable* table, const float2* rope_tab, T* q_out, T* k_pool, T* v_pool,
                               T* k_pre_pool, KvGeom g, int n_q_heads, hipStream_t st);

// Attention of the active rows over one layer of the cache.  With a table, row r belongs to request
// row_req[r] (sequence table->r[..].dst_seq) and tiles never straddle requests; with table == nullptr
// all rows belong to sequence `fixed_seq`.
template <typename T>
hipError_t launch_attention(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                            int fixed_seq, int total_rows, int total_tiles, const T* k_pool, const T* v_pool,
                            KvGeom g, int n_q_heads, T* out, hipStream_t st);
template <typename T>
hipError_t launch_attention_simt(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                 int fixed_seq, int total_rows, const T* k_pool, const T* v_pool, KvGeom g,
                                 int n_q_heads, T* out, hipStream_t st);
int attention_tile_rows(int dtype, int n_q_heads, int n_kv_heads);  // query rows per attention tile

// bf16 attention with an optional split of every query tile's KV range into chunks (partial results
// in `part`, merged by a second kernel).  part == nullptr: no split.
// With a table, total_tiles is the number of work items of the launch (ReqTable::total_items as assign_split_slots
// left it, or an upper bound when the table is finalized on the device).
// A query tile whose KV range spans more than long_thr tiles is cut into chunks of chunk_tiles tiles;
// n_chunks is the grid's chunk dimension (1: no split at all), total_slots the (tile, chunk) slots of
// partial results the plan may touch.
struct AttnSplit { int n_chunks, chunk_tiles, long_thr, total_slots; };
inline AttnSplit attention_no_split() { AttnSplit sp = {1, 1 << 24, 1 << 24, 0}; return sp; }
int attention_forced_chunk_tiles();
void set_attention_chunk_tiles(int t);  // 0: by shape; > 0: forced KV tiles per chunk
size_t attention_partial_floats(int total_slots, int n_q_heads);
hipError_t launch_attention_bf16(const bf16* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                 int fixed_seq, int total_rows, int total_tiles, const bf16* k_pool,
                                 const bf16* v_pool, KvGeom g, int n_q_heads, bf16* out, AttnSplit sp, float* part,
                                 hipStream_t st, float* scores = nullptr, int scores_len = 0, int merge_rows = 0);

template <typename T>
hipError_t launch_vdev_score(const T* v_fresh, int fresh_row_stride, const T* v_pool, KvGeom g,
                             const ReqTable* table, int n_req, int max_seg, float* scores, hipStream_t st);

hipError_t launch_topk(const float* score, int n, int k, int* idx_out, hipStream_t st);
// All requests of a call in one launch (one workgroup per request, read from the table: scores at score_base,
// S of them, output at sel_base).  Budget: the r.k largest.  Threshold: Eq. (5)-(10) with the requests' influence
// vectors (nullptr: none), counts to sel_cnt[b].  Requests with k <= 0 are skipped.
struct InfluenceIn { const float* s_inf[RC_MAX_REQ]; };
hipError_t launch_topk_batch(const float* scores, const ReqTable* table, int n_req, int* sel_idx, hipStream_t st);
hipError_t launch_final_select_batch(const float* scores, const InfluenceIn& inf, const ReqTable* table, int n_req,
                                     float tau_dev, float tau_inf, int k_suf, int* sel_idx, int* sel_cnt,
                                     hipStream_t st);
hipError_t launch_copy_sel_batch(const int* forced, const ReqTable* table, int n_req, int* sel_idx, hipStream_t st);
// Threshold selector: turns the device-side counts into the tables of the sparse phase and the phase after it
// (tabs[PH_C], tabs[PH_D], uploaded with their static fields and k = S), so that no count has to travel to the host.
struct AttnSplit;
hipError_t launch_finalize_tables(ReqTable* tabs, const int* sel_cnt, int tile_rows, int kv_tile, int thr_c,
                                  int chunks_c, int cap_c, int thr_d, int chunks_d, int cap_d, hipStream_t st);
hipError_t launch_threshold_select(const float* score, int n, float tau, int* idx_out, int* count_out,
                                   hipStream_t st);
// per-request influence vectors (Eq. 6), passed to the accumulation kernel by value; nullptr: not tracked
struct InfluencePtrs { float* s_inf[RC_MAX_REQ]; };
size_t influence_scratch_floats(int n_rows, int n_q_heads, int max_len);
// scratch holds the scores [rows][Hq][max_len] (q.k / sqrt(dh)) followed by one (reference exponent in log2 units,
// sum of exp2(score * log2(e) - reference)) pair per (row, head).  The scores are written by launch_influence_scores
// or by the bf16 attention kernel, which also writes the pairs (have_pairs); launch_influence_finish computes the
// pairs if they are missing, turns the scores into weights and adds them to the requests' vectors.
inline float2* influence_pairs(float* scratch, int n_rows, int n_q_heads, int max_len) {
  size_t off = (size_t)n_rows * n_q_heads * max_len;
  off = (off + 1) & ~(size_t)1;   // 8-byte aligned
  return reinterpret_cast<float2*>(scratch + off);
}
template <typename T>
hipError_t launch_influence_scores(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                   int n_rows, const T* k_pool, KvGeom g, int n_q_heads, int max_len, float* scratch,
                                   hipStream_t st);
hipError_t launch_influence_finish(const int* row_pos, const int* row_req, int n_rows, int n_q_heads, int max_len,
                                   const InfluencePtrs& out, float* scratch, bool have_pairs, hipStream_t st);
hipError_t launch_final_select(const float* s_dev, const float* s_inf, int n, float tau_dev, float tau_inf, int k_suf,
                               int* idx_out, int* count_out, hipStream_t st);
hipError_t launch_copy_i32(const int* src, int* dst, int n, hipStream_t st);

// Kernels that use more dynamic LDS than a kernel gets without asking must say so once per device.  `done` is a
// per-kernel bit mask of the devices that have been told (one static per call site).
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// machine ceilings (ceilings.hip)
hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
size_t mfma_loop_out_floats(int n_workgroups);
double mfma_loop_flops(int n_workgroups, int iters);
hipError_t launch_mfma_loop(float* out, int n_workgroups, int iters, hipStream_t st);

template <typename T>
hipError_t launch_scatter_rows(const T* k_rows, const T* v_rows, const int* pos, int n, T* k_pool,
                               T* v_pool, KvGeom g, int seq, hipStream_t st);

hipError_t launch_gather_last(const ReqTable* table, int n_req, const float* h, float* out, int d,
                              hipStream_t st);

}  // namespace rc
