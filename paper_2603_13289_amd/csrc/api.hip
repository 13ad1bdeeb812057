// C ABI of the selective-recompute prefill: argument checking, workspace carving and the per-layer
// launch sequence.  All device work is done by the kernels in the sibling files; this file only
// decides which rows are active in which layer and enqueues launches.
#include <algorithm>
#include <new>
#include <vector>

#include "common.h"

using namespace rc;

struct rc_model {
  rc_model_desc d;
  std::vector<rc_layer_w> layers;
  const void* g_final;
  const void* w_lm;
};

namespace {

#define RC_HIP(expr)                         \
  do {                                       \
    if ((expr) != hipSuccess) return RC_E_HIP; \
  } while (0)
#define RC_TRY(expr)               \
  do {                             \
    rc_status _s = (expr);         \
    if (_s != RC_OK) return _s;    \
  } while (0)

// ---------------------------------------------------------------- optional per-class GPU timing
enum ProfClass : int {
  PC_REROTATE = 0, PC_ROWS, PC_RMSNORM, PC_GEMM_QKV, PC_GEMM_O, PC_GEMM_GATE_UP, PC_GEMM_DOWN, PC_GEMM_VFRESH,
  PC_GEMM_LM_HEAD, PC_ROPE_SCATTER, PC_ATTENTION, PC_SCORE, PC_SELECT, PC_TABLES, PC_INFLUENCE, PC_COUNT
};
const char* const kProfNames[PC_COUNT] = {"rope_rerotate", "row_bookkeeping", "rmsnorm", "gemm_qkv", "gemm_o",
                                          "gemm_gate_up", "gemm_down", "gemm_vfresh", "gemm_lm_head",
                                          "rope_scatter", "attention", "vdev_score", "select", "tables", "influence"};
struct ProfRec { int cls; hipEvent_t a, b; };
struct Profiler {
  bool on = false;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
} g_prof;

struct ProfScope {
  hipStream_t st;
  hipEvent_t b = nullptr;
  ProfScope(int cls, hipStream_t s) : st(s) {
    if (!g_prof.on) return;
    hipEvent_t a = g_prof.get();
    b = g_prof.get();
    if (!a || !b) { b = nullptr; return; }
    (void)hipEventRecord(a, st);
    g_prof.recs.push_back({cls, a, b});
  }
  ~ProfScope() { if (b) (void)hipEventRecord(b, st); }
};
#define RC_LAUNCH(cls, expr)          \
  do {                                \
    ProfScope _ps((cls), st);         \
    if ((expr) != hipSuccess) return RC_E_HIP; \
  } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
inline size_t elem_size(int dtype) { return dtype == RC_BF16 ? 2 : 4; }

rc_status check_desc(const rc_model_desc& d) {
  if (d.n_layers < 1 || d.d_model < 1 || d.n_q_heads < 1 || d.n_kv_heads < 1 || d.head_dim < 1 ||
      d.d_ffn < 1 || d.vocab < 1 || !(d.rope_base > 0.f) || !(d.rms_eps >= 0.f))
    return RC_E_INVALID_ARG;
  if (d.dtype != RC_F32 && d.dtype != RC_BF16) return RC_E_INVALID_ARG;
  if (d.n_q_heads % d.n_kv_heads != 0) return RC_E_INVALID_ARG;
  if (d.n_layers > RC_MAX_LAYERS) return RC_E_CAPACITY;
  if (d.dtype == RC_BF16 && d.head_dim != 128) return RC_E_UNSUPPORTED;
  if (d.dtype == RC_F32 && d.head_dim != 64 && d.head_dim != 128) return RC_E_UNSUPPORTED;
  if (d.d_model % 8 || d.d_ffn % 8) return RC_E_UNSUPPORTED;
  return RC_OK;
}

KvGeom geom_of(const rc_paged_kv& kv, const rc_model_desc& d) {
  KvGeom g;
  g.n_blocks = kv.n_blocks;
  g.block_size = kv.block_size;
  g.block_table = kv.block_table;
  g.max_blocks = kv.max_blocks_per_seq;
  g.n_kv_heads = d.n_kv_heads;
  g.head_dim = d.head_dim;
  g.bs_shift = log2_if_pow2(kv.block_size);
  return g;
}

KvGeom geom_of(const rc_kv_layer& kv) {
  KvGeom g;
  g.n_blocks = kv.n_blocks;
  g.block_size = kv.block_size;
  g.block_table = kv.block_table;
  g.max_blocks = kv.max_blocks_per_seq;
  g.n_kv_heads = kv.n_kv_heads;
  g.head_dim = kv.head_dim;
  g.bs_shift = log2_if_pow2(kv.block_size);
  return g;
}

rc_status check_paged(const rc_paged_kv* kv, int n_layers) {
  if (!kv || !kv->k_pool || !kv->v_pool || !kv->block_table) return RC_E_INVALID_ARG;
  if (kv->n_blocks < 1 || kv->block_size < 1 || kv->n_seq < 1 || kv->max_blocks_per_seq < 1)
    return RC_E_INVALID_ARG;
  for (int l = 0; l < n_layers; ++l)
    if (!kv->k_pool[l] || !kv->v_pool[l]) return RC_E_INVALID_ARG;
  return RC_OK;
}

rc_status check_kv_layer(const rc_kv_layer* kv) {
  if (!kv || !kv->k || !kv->v || !kv->block_table) return RC_E_INVALID_ARG;
  if (kv->n_blocks < 1 || kv->block_size < 1 || kv->n_seq < 1 || kv->max_blocks_per_seq < 1 ||
      kv->n_kv_heads < 1)
    return RC_E_INVALID_ARG;
  if (kv->dtype != RC_F32 && kv->dtype != RC_BF16) return RC_E_INVALID_ARG;
  if (kv->dtype == RC_BF16 && kv->head_dim != 128) return RC_E_UNSUPPORTED;
  if (kv->dtype == RC_F32 && kv->head_dim != 64 && kv->head_dim != 128) return RC_E_UNSUPPORTED;
  return RC_OK;
}

// ---------------------------------------------------------------- phases
Phase phase_of_layer(int l, int l_start, int l_det, int l_end) {
  if (l < l_start) return PH_A;
  if (l < l_det) return PH_B;
  if (l <= l_end) return PH_C;
  return PH_D;
}

// rows of a phase for the given static fields (a scratch copy of the table is filled)
int total_rows_in(const ReqTable& base, Phase ph) {
  long t = 0;
  for (int b = 0; b < base.n_req; ++b) {
    int mode, n;
    phase_seg_rows(base.r[b], ph, &mode, &n);
    t += base.r[b].P + n + base.r[b].nsuf;
  }
  return (int)t;
}

// ---------------------------------------------------------------- attention KV-split plan of one phase
// Query tiles whose KV range is long are cut into chunks when the phase has too few tiles to keep the
// chip busy otherwise (sparse rectification: few rows, long context).  Row positions are known on the
// host except for the selected rows, which are taken as evenly spread over the segment.
constexpr int kLongKvTiles = 24;   // a query tile with more KV tiles (of 64 keys) than this may be split
constexpr int kKvTile = 64;

int est_row_pos(const ReqDev& r, int i) {
  if (i < r.P) return r.pos0 + i;
  if (i < r.P + r.n_seg_rows) {
    const int si = i - r.P;
    if (r.seg_mode == SEG_ALL) return r.pos0 + r.P + si;
    if (r.seg_mode == SEG_SEL)
      return r.pos0 + r.P + (int)std::min<long>((long)(si + 1) * r.S / std::max(r.n_seg_rows, 1), r.S) - 1;
    return r.pos0 + r.P + r.S - 1;
  }
  return r.pos0 + r.P + r.S + (i - r.P - r.n_seg_rows);
}

// Chooses chunk length and split threshold for a phase from the (estimated) row positions of table t; the
// per-request slot assignment is left to assign_split_slots.  n_chunks == 1: no split.
//
// A workgroup serves one (query tile, KV head[, KV chunk]) and costs its KV tiles plus a fixed part (prologue, first
// tile's latency); two workgroups share a compute unit.  Candidates (no split, chunks of 4 ... 128 KV tiles; a tile is
// split when its range is longer than one chunk) are priced by a list-scheduling estimate: the busier of "the longest
// workgroup" and "all work spread over the slots", plus half a longest workgroup for the ragged end of a launch with
// more workgroups than slots,
// plus the merge pass over the partial results of the split rows.  Units: one KV tile step of one slot (~2.2 us).
// Measured on the 2048 + 16384-token workload: its sparse layers (1639 selected rows, up to 288 KV tiles each) take
// 520 us unsplit and 182 + 33 us with chunks of 32; the dense layer and the short prefix-only layers are best left whole.
// A decoding step (one row per sequence, 8 KV heads, 80 KV tiles) gets chunks of 4: 160 workgroups instead of 40.
constexpr float kWgFixedSteps = 4.f;       // fixed cost of a workgroup
constexpr float kMergeFixedSteps = 3.5f;   // launch of the merge kernel
constexpr float kMergeBytesPerStep = 8.8e6f;

float price_split(const ReqTable* t, int n_kv_heads, int n_q_heads, int tile_rows, int chunk /* 0: none */, int slots) {
  double work = 0.0, merge_bytes = 0.0;
  long wgs = 0;
  int longest = 0;
  for (int b = 0; b < t->n_req; ++b) {
    const ReqDev& r = t->r[b];
    for (int i0 = 0; i0 < r.n_rows; i0 += tile_rows) {
      const int rows = std::min(tile_rows, r.n_rows - i0);
      const int n = est_row_pos(r, i0 + rows - 1) / kKvTile + 1;
      if (chunk > 0 && n > chunk) {
        const int parts = (n + chunk - 1) / chunk;
        work += (double)(n + kWgFixedSteps * parts) * n_kv_heads;
        wgs += (long)parts * n_kv_heads;
        longest = std::max(longest, chunk);
        merge_bytes += (double)rows * n_q_heads * parts * (128 + 2) * 4;
      } else {
        work += (double)(n + kWgFixedSteps) * n_kv_heads;
        wgs += n_kv_heads;
        longest = std::max(longest, n);
      }
    }
  }
  const float l = longest + kWgFixedSteps;
  float cost = std::max(l, (float)(work / slots));
  if (wgs > slots) cost += 0.5f * l;     // later rounds of workgroups end raggedly; a launch that fits the slots does not
  if (merge_bytes > 0.0) cost += kMergeFixedSteps + (float)(merge_bytes / kMergeBytesPerStep);
  return cost;
}

AttnSplit choose_phase_split(const ReqTable* t, int n_kv_heads, int n_q_heads, int tile_rows, int max_pos) {
  int chunk_tiles = 0;
  const int forced = attention_forced_chunk_tiles();
  if (forced > 0) {
    chunk_tiles = forced;
  } else {
    // query-head groups of up to four wavefronts run two workgroups per compute unit, wider ones one
    const int slots = (n_q_heads / n_kv_heads <= 4 ? 2 : 1) * 256;
    float best = price_split(t, n_kv_heads, n_q_heads, tile_rows, 0, slots);
    // chunks shorter than 16 tiles only for phases of a handful of query tiles (decoding steps): with a few hundred
    // workgroups already there, the model's fixed costs are too coarse to tell a gain of a few tile steps from the
    // price of the merge pass (prefix-only layers of 1024 rows: 36 us whole, 30 + 13 us in chunks of 8)
    long whole_wgs = 0;
    for (int b = 0; b < t->n_req; ++b) whole_wgs += (long)((t->r[b].n_rows + tile_rows - 1) / tile_rows) * n_kv_heads;
    const int min_chunk = whole_wgs * 8 <= slots ? 4 : 16;
    for (int c : {4, 8, 12, 16, 24, 32, 48, 64, 96, 128}) {
      if (c < min_chunk) continue;
      const float p = price_split(t, n_kv_heads, n_q_heads, tile_rows, c, slots);
      if (p < 0.97f * best) { best = p; chunk_tiles = c; }     // a split has to pay for itself
    }
    if (chunk_tiles == 0) return attention_no_split();
  }
  const int max_tiles = (max_pos + kKvTile - 1) / kKvTile;
  const int n_chunks = (max_tiles + chunk_tiles - 1) / chunk_tiles;
  if (n_chunks <= 1) return attention_no_split();
  AttnSplit sp = {n_chunks, chunk_tiles, chunk_tiles, 0};
  return sp;
}

// the whole plan of a phase whose row counts the host knows: decision, then slots (no capacity limit)
AttnSplit plan_phase_split(ReqTable* t, int n_kv_heads, int n_q_heads, int tile_rows, int max_pos) {
  AttnSplit sp = choose_phase_split(t, n_kv_heads, n_q_heads, tile_rows, max_pos);
  sp.total_slots = assign_split_slots(t, tile_rows, kKvTile, sp.long_thr, sp.n_chunks, 1 << 30);
  if (sp.total_slots == 0) return attention_no_split();
  return sp;
}

// ---------------------------------------------------------------- workspace
struct Workspace {
  ReqTable* tables;  // PH_COUNT slots
  float2* rope_tab;
  float2* delta_tab;
  int* row_pos;
  int* row_req;
  float* h[2];
  void* a;       // normalised activations [R][d] of T
  float* qkv;    // [R][Hq*dh + 2*Hkv*dh]
  void* q;       // rotated queries [R][Hq*dh] of T
  void* o;       // attention output [R][Hq*dh] of T
  void* act;     // SwiGLU output [R][F] of T
  void* vfresh;  // [R][Hkv*dh] of T
  float* scores;
  float* h_last;
  void* a_last;
  float* attn_part;   // partial attention results when a layer's KV range is split into chunks
  float* gemm_part;   // accumulators of K-split tail tiles of the bf16 GEMMs
  float* inf_scratch; // attention scores of the decoding rows (influence accumulation)
  size_t attn_part_floats;
  size_t bytes;
};

Workspace carve(void* base, const rc_model_desc& d, int max_rows, int max_pos, int n_req, int sum_seg,
                size_t attn_part_floats, size_t inf_floats = 0) {
  Workspace w;
  size_t off = 0;
  char* p = reinterpret_cast<char*>(base);
  auto take = [&](size_t bytes) {
    void* r = p ? p + off : nullptr;
    off += align_up(bytes);
    return r;
  };
  const size_t es = elem_size(d.dtype);
  const size_t R = (size_t)(max_rows > 0 ? max_rows : 1);
  const size_t nq = (size_t)d.n_q_heads * d.head_dim, nkv = (size_t)d.n_kv_heads * d.head_dim;
  w.tables = (ReqTable*)take(sizeof(ReqTable) * PH_COUNT);
  w.rope_tab = (float2*)take(sizeof(float2) * (size_t)(max_pos > 0 ? max_pos : 1) * (d.head_dim / 2));
  w.delta_tab = (float2*)take(sizeof(float2) * (size_t)n_req * (d.head_dim / 2));
  w.row_pos = (int*)take(sizeof(int) * R);
  w.row_req = (int*)take(sizeof(int) * R);
  w.h[0] = (float*)take(sizeof(float) * R * d.d_model);
  w.h[1] = (float*)take(sizeof(float) * R * d.d_model);
  w.a = take(es * R * d.d_model);
  w.qkv = (float*)take(sizeof(float) * R * (nq + 2 * nkv));
  w.q = take(es * R * nq);
  w.o = take(es * R * nq);
  w.act = take(es * R * d.d_ffn);
  w.vfresh = take(es * R * nkv);
  w.scores = (float*)take(sizeof(float) * (size_t)(sum_seg > 0 ? sum_seg : 1));
  w.h_last = (float*)take(sizeof(float) * (size_t)n_req * d.d_model);
  w.a_last = take(es * (size_t)n_req * d.d_model);
  w.attn_part = (float*)take(sizeof(float) * (attn_part_floats > 0 ? attn_part_floats : 1));
  w.attn_part_floats = attn_part_floats;
  w.gemm_part = (float*)take(d.dtype == RC_BF16 ? gemm_partial_bytes() : 256);
  w.inf_scratch = (float*)take(sizeof(float) * (inf_floats > 0 ? inf_floats : 1));
  w.bytes = off;
  return w;
}

// ---------------------------------------------------------------- the layer engine
struct Job {
  const rc_model* m;
  ReqTable base;                  // static per-request fields (P, S, nsuf, k, positions, pointers)
  int l_start, l_det, l_end;      // l_start >= n_layers: plain prefill
  const rc_paged_kv* src;
  const rc_paged_kv* dst;
  void* const* k_pre_pool;
  int capture_layer;              // -1: none
  const int32_t* forced_idx;
  int selector;                   // rc_selector
  float tau_dev, tau_inf;
  int k_suf;
  const float* s_inf[RC_MAX_REQ];
  float* logits;
  int32_t* sel_idx;
  int32_t* sel_cnt;
  float* scores_out;
  int max_pos, sum_seg, max_seg;
  bool takeover = true;           // false: the segment rows already sit in dst (a decoding step)
  bool any_inf = false;
  InfluencePtrs inf;
};

template <typename T>
hipError_t attention_dispatch(const T* q, const int* row_pos, const int* row_req, const ReqTable* table,
                              int total_rows, int total_tiles, const T* k_pool, const T* v_pool, KvGeom g,
                              int n_q_heads, T* out, AttnSplit sp, float* part, hipStream_t st, float* scores,
                              int scores_len, int merge_rows);
template <>
hipError_t attention_dispatch<float>(const float* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                     int total_rows, int total_tiles, const float* k_pool, const float* v_pool,
                                     KvGeom g, int n_q_heads, float* out, AttnSplit, float*, hipStream_t st, float*, int, int) {
  return launch_attention<float>(q, row_pos, row_req, table, 0, total_rows, total_tiles, k_pool, v_pool, g,
                                 n_q_heads, out, st);
}
template <>
hipError_t attention_dispatch<bf16>(const bf16* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                    int total_rows, int total_tiles, const bf16* k_pool, const bf16* v_pool,
                                    KvGeom g, int n_q_heads, bf16* out, AttnSplit sp, float* part, hipStream_t st,
                                    float* scores, int scores_len, int merge_rows) {
  return launch_attention_bf16(q, row_pos, row_req, table, 0, total_rows, total_tiles, k_pool, v_pool, g, n_q_heads,
                               out, sp, part, st, scores, scores_len, merge_rows);
}

template <typename T>
hipError_t gemm_any(const T* a, const T* wt, const T* wt2, void* c, int m, int n, int k, int ldc, GemmEpilogue epi,
                    float* partial, hipStream_t st, const int* m_live = nullptr);
template <>
hipError_t gemm_any<float>(const float* a, const float* wt, const float* wt2, void* c, int m, int n, int k, int ldc,
                           GemmEpilogue epi, float*, hipStream_t st, const int* m_live) {
  return launch_gemm<float>(a, wt, wt2, c, m, n, k, ldc, epi, st, m_live);
}
template <>
hipError_t gemm_any<bf16>(const bf16* a, const bf16* wt, const bf16* wt2, void* c, int m, int n, int k, int ldc,
                          GemmEpilogue epi, float* partial, hipStream_t st, const int* m_live) {
  return launch_gemm_bf16(a, wt, wt2, c, m, n, k, ldc, epi, partial, st, m_live);
}
template <typename T>
hipError_t gemm_qkv_any(const T* a, const T* wq, int nq, const T* wk, const T* wv, int nkv, float* c, int m, int k,
                        float* partial, hipStream_t st, const int* m_live);
template <>
hipError_t gemm_qkv_any<float>(const float* a, const float* wq, int nq, const float* wk, const float* wv, int nkv,
                               float* c, int m, int k, float*, hipStream_t st, const int* m_live) {
  return launch_gemm_qkv<float>(a, wq, nq, wk, wv, nkv, c, m, k, st, m_live);
}
template <>
hipError_t gemm_qkv_any<bf16>(const bf16* a, const bf16* wq, int nq, const bf16* wk, const bf16* wv, int nkv, float* c,
                              int m, int k, float* partial, hipStream_t st, const int* m_live) {
  return launch_gemm_qkv_bf16(a, wq, nq, wk, wv, nkv, c, m, k, partial, st, m_live);
}

// Partial-attention slots the sparse phase (and the phase after it) may use when the threshold selector decides the
// row counts on the device: planned for a nominal selection of a fifth of every segment, with room for twice that;
// a selection that needs more attends unsplit.
struct ThresholdSplit { AttnSplit sp[PH_COUNT]; int cap[PH_COUNT]; };
ThresholdSplit plan_threshold_split(const ReqTable& base, int n_kv_heads, int n_q_heads, int tile_rows, int max_pos, bool bf16_model) {
  ThresholdSplit ts;
  for (int p = 0; p < PH_COUNT; ++p) { ts.sp[p] = attention_no_split(); ts.cap[p] = 0; }
  if (!bf16_model) return ts;
  for (int p = PH_C; p <= PH_D; ++p) {
    ReqTable t = base;
    for (int b = 0; b < t.n_req; ++b)
      if (t.r[b].k > 0) t.r[b].k = std::max(1, t.r[b].S / 5);
    fill_phase_table(&t, p, nullptr, tile_rows);
    AttnSplit sp = choose_phase_split(&t, n_kv_heads, n_q_heads, tile_rows, max_pos);
    if (sp.n_chunks <= 1) continue;
    for (int b = 0; b < t.n_req; ++b)
      if (t.r[b].k > 0) t.r[b].k = std::min(t.r[b].S, 2 * t.r[b].k);
    fill_phase_table(&t, p, nullptr, tile_rows);
    const int cap = assign_split_slots(&t, tile_rows, kKvTile, sp.long_thr, sp.n_chunks, 1 << 30);
    if (cap <= 0) continue;
    sp.total_slots = cap;
    ts.sp[p] = sp;
    ts.cap[p] = cap;
  }
  return ts;
}

template <typename T>
rc_status run_job(Job& job, Workspace& w, hipStream_t st) {
  const rc_model_desc& d = job.m->d;
  const int n_req = job.base.n_req;
  const int D = d.d_model, nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, F = d.d_ffn;
  const int tile_rows = attention_tile_rows(d.dtype, d.n_q_heads, d.n_kv_heads);
  const KvGeom gd = geom_of(*job.dst, d);
  const bool has_seg = job.max_seg > 0;
  const bool by_threshold = job.selector == RC_SELECT_THRESHOLD;

  ReqTable tabs[PH_COUNT];
  AttnSplit splits[PH_COUNT];
  bool on_device[PH_COUNT] = {false, false, false, false};   // table already written (and finalized) on the device
  for (int p = 0; p < PH_COUNT; ++p) tabs[p] = job.base;

  RC_LAUNCH(PC_TABLES, launch_rope_table(w.rope_tab, job.max_pos, d.head_dim / 2, (double)d.rope_base, st));

  int cur = -1;   // phase whose rows are live in w.h[hbuf]
  int hbuf = 0;
  // Row counts of the phase: exact on the host, or (threshold selector, from the sparse phase on) an upper bound
  // that sizes the grids while the kernels read the live counts from the device table.
  auto live = [&](int ph) -> const int* { return on_device[ph] ? &(w.tables + ph)->total_rows : nullptr; };
  auto enter_phase = [&](Phase ph) -> rc_status {
    if (!on_device[ph]) {
      fill_phase_table(&tabs[ph], ph, cur >= 0 ? &tabs[cur] : nullptr, tile_rows);
      splits[ph] = d.dtype == RC_BF16 ? plan_phase_split(&tabs[ph], d.n_kv_heads, d.n_q_heads, tile_rows, job.max_pos)
                                      : attention_no_split();
      if (attention_partial_floats(splits[ph].total_slots, d.n_q_heads) > w.attn_part_floats) {
        // the plan was made for other row counts than the workspace was sized for: attend unsplit
        splits[ph] = attention_no_split();
      }
      if (splits[ph].n_chunks <= 1) assign_split_slots(&tabs[ph], tile_rows, kKvTile, 1 << 24, 1, 0);   // items = tiles
      RC_LAUNCH(PC_TABLES, launch_upload_table(tabs[ph], w.tables + ph, st));
    }
    const int nb = cur >= 0 ? 1 - hbuf : hbuf;
    RC_LAUNCH(PC_ROWS, launch_build_rows<T>(w.tables + ph, tabs[ph].total_rows, w.h[hbuf], w.h[nb], w.row_pos, w.row_req,
                                job.sel_idx, D, st));
    hbuf = nb;
    cur = ph;
    return RC_OK;
  };

  for (int l = 0; l < d.n_layers; ++l) {
    const rc_layer_w& lw = job.m->layers[l];
    const Phase ph = phase_of_layer(l, job.l_start, job.l_det, job.l_end);
    if (cur < 0 || (ph != cur && ph != PH_C)) RC_TRY(enter_phase(ph));

    // K1, once: take over the reused rows of every layer (keys to their new positions, values copied).
    // Layers that recompute rows later simply overwrite them.
    if (l == 0 && has_seg && job.takeover) {
      const KvGeom gs = geom_of(*job.src, d);
      RC_LAUNCH(PC_TABLES, launch_delta_table(w.delta_tab, w.tables + cur, n_req, d.head_dim / 2, (double)d.rope_base, st));
      for (int l0 = 0; l0 < d.n_layers; l0 += kRerotateLayers) {
        const int nl = std::min(kRerotateLayers, d.n_layers - l0);
        RerotatePtrs ptrs;
        for (int i = 0; i < nl; ++i) {
          ptrs.k_src[i] = job.src->k_pool[l0 + i];
          ptrs.v_src[i] = job.src->v_pool[l0 + i];
          ptrs.k_dst[i] = job.dst->k_pool[l0 + i];
          ptrs.v_dst[i] = job.dst->v_pool[l0 + i];
        }
        RC_LAUNCH(PC_REROTATE, launch_rerotate<T>(ptrs, nl, gs, gd, w.tables + cur, n_req, job.max_seg, w.rope_tab,
                                                  w.delta_tab, st));
      }
    }

    // detection layer: fresh values of every segment token -> Eq. (1) -> selection
    if (ph == PH_C && cur != PH_C) {
      bool any = false;
      for (int b = 0; b < n_req; ++b) any = any || job.base.r[b].k > 0;
      if (any) {
        const int rows_b = tabs[cur].total_rows;
        RC_LAUNCH(PC_RMSNORM, launch_rmsnorm<T>(w.h[hbuf], (const T*)lw.g_attn, (T*)w.a, rows_b, D, d.rms_eps, st));
        RC_LAUNCH(PC_GEMM_VFRESH, gemm_any<T>((const T*)w.a, (const T*)lw.wv, nullptr, w.vfresh, rows_b, nkv, D, nkv, EPI_STORE_T, w.gemm_part, st));
        float* sc = job.scores_out ? job.scores_out : w.scores;
        RC_LAUNCH(PC_SCORE, launch_vdev_score<T>((const T*)w.vfresh, nkv, (const T*)job.dst->v_pool[l], gd, w.tables + cur,
                                    n_req, job.max_seg, sc, st));
        // one launch for all requests (the table of the dense phase carries score_base, S, k and sel_base)
        if (by_threshold) {
          InfluenceIn inf;
          for (int b = 0; b < RC_MAX_REQ; ++b) inf.s_inf[b] = b < n_req ? job.s_inf[b] : nullptr;
          RC_LAUNCH(PC_SELECT, launch_final_select_batch(sc, inf, w.tables + cur, n_req, job.tau_dev, job.tau_inf, job.k_suf,
                                                         job.sel_idx, job.sel_cnt, st));
          // The rows of the sparse layers depend on the scores.  The tables of the two remaining phases go to the
          // device with every token counted as selected (the bound that sizes all grids from here on) and a
          // one-thread kernel rewrites their counts, row offsets and attention slots from sel_cnt: nothing comes
          // back to the host, the call stays asynchronous.
          const ThresholdSplit ts = plan_threshold_split(job.base, d.n_kv_heads, d.n_q_heads, tile_rows, job.max_pos, d.dtype == RC_BF16);
          int phase_before = cur;
          for (int p = PH_C; p <= PH_D; ++p) {
            fill_phase_table(&tabs[p], p, &tabs[phase_before], tile_rows);
            splits[p] = ts.sp[p];
            if (attention_partial_floats(splits[p].total_slots, d.n_q_heads) > w.attn_part_floats) splits[p] = attention_no_split();
            // work items of the attention grid, as an upper bound over every possible selection: all tiles whole, or
            // the tiles that stay whole plus as many (tile, chunk) pairs as there are slots
            assign_split_slots(&tabs[p], tile_rows, kKvTile, splits[p].long_thr, splits[p].n_chunks, 1 << 30);
            int whole = 0;
            for (int b = 0; b < n_req; ++b)
              whole += std::min(tabs[p].r[b].long_tile_start, (tabs[p].r[b].n_rows + tile_rows - 1) / tile_rows);
            tabs[p].total_items = std::max(tabs[p].total_tiles, whole + splits[p].total_slots);
            RC_LAUNCH(PC_TABLES, launch_upload_table(tabs[p], w.tables + p, st));
            on_device[p] = true;
            phase_before = p;
          }
          RC_LAUNCH(PC_TABLES, launch_finalize_tables(w.tables, job.sel_cnt, tile_rows, kKvTile, splits[PH_C].long_thr,
                                                      splits[PH_C].n_chunks, splits[PH_C].total_slots, splits[PH_D].long_thr,
                                                      splits[PH_D].n_chunks, splits[PH_D].total_slots, st));
        } else if (job.forced_idx) {
          RC_LAUNCH(PC_SELECT, launch_copy_sel_batch(job.forced_idx, w.tables + cur, n_req, job.sel_idx, st));
        } else {
          RC_LAUNCH(PC_SELECT, launch_topk_batch(sc, w.tables + cur, n_req, job.sel_idx, st));
        }
      }
      RC_TRY(enter_phase(PH_C));
    }

    const int rows = tabs[cur].total_rows;
    if (rows == 0) continue;
    const int* m_live = live(cur);
    if (l == job.capture_layer) RC_LAUNCH(PC_ROWS, launch_capture_rows<T>(w.tables + cur, rows, w.h[hbuf], w.row_req, D, st));

    float* h = w.h[hbuf];
    RC_LAUNCH(PC_RMSNORM, launch_rmsnorm<T>(h, (const T*)lw.g_attn, (T*)w.a, rows, D, d.rms_eps, st, m_live));
    RC_LAUNCH(PC_GEMM_QKV, gemm_qkv_any<T>((const T*)w.a, (const T*)lw.wq, nq, (const T*)lw.wk, (const T*)lw.wv, nkv,
                                              w.qkv, rows, D, w.gemm_part, st, m_live));
    // rotary on q/k at the rows' absolute positions; fresh K/V written into the cache before anyone attends
    RC_LAUNCH(PC_ROPE_SCATTER, launch_rope_scatter<T>(w.qkv, rows, w.row_pos, w.row_req, w.tables + cur, w.rope_tab, (T*)w.q,
                                  (T*)job.dst->k_pool[l], (T*)job.dst->v_pool[l],
                                  job.k_pre_pool ? (T*)job.k_pre_pool[l] : nullptr, gd, d.n_q_heads, st));
    // influence accumulation (decoding): the bf16 matrix-core attention kernel hands out its scores; the other
    // paths compute them in a pass of their own
    const bool scores_from_attention = job.any_inf && d.dtype == RC_BF16 && d.n_q_heads / d.n_kv_heads <= 8;
    if (job.any_inf && !scores_from_attention)
      RC_LAUNCH(PC_INFLUENCE, launch_influence_scores<T>((const T*)w.q, w.row_pos, w.row_req, w.tables + cur, rows,
                                                         (const T*)job.dst->k_pool[l], gd, d.n_q_heads, job.max_pos,
                                                         w.inf_scratch, st));
    RC_LAUNCH(PC_ATTENTION, attention_dispatch<T>((const T*)w.q, w.row_pos, w.row_req, w.tables + cur, rows,
                                 tabs[cur].total_items, (const T*)job.dst->k_pool[l],
                                 (const T*)job.dst->v_pool[l], gd, d.n_q_heads, (T*)w.o, splits[cur], w.attn_part, st,
                                 scores_from_attention ? w.inf_scratch : nullptr, job.max_pos, tabs[cur].total_merge_rows));
    if (job.any_inf)
      RC_LAUNCH(PC_INFLUENCE, launch_influence_finish(w.row_pos, w.row_req, rows, d.n_q_heads, job.max_pos, job.inf,
                                                      w.inf_scratch, scores_from_attention, st));
    RC_LAUNCH(PC_GEMM_O, gemm_any<T>((const T*)w.o, (const T*)lw.wo, nullptr, h, rows, D, nq, D, EPI_ADD_F32, w.gemm_part, st, m_live));
    RC_LAUNCH(PC_RMSNORM, launch_rmsnorm<T>(h, (const T*)lw.g_ffn, (T*)w.a, rows, D, d.rms_eps, st, m_live));
    RC_LAUNCH(PC_GEMM_GATE_UP, gemm_any<T>((const T*)w.a, (const T*)lw.w_gate, (const T*)lw.w_up, w.act, rows, F, D, F, EPI_SWIGLU_T, w.gemm_part, st, m_live));
    RC_LAUNCH(PC_GEMM_DOWN, gemm_any<T>((const T*)w.act, (const T*)lw.w_down, nullptr, h, rows, D, F, D, EPI_ADD_F32, w.gemm_part, st, m_live));
  }

  // first-token logits from the last position of each request
  RC_LAUNCH(PC_ROWS, launch_gather_last(w.tables + cur, n_req, w.h[hbuf], w.h_last, D, st));
  RC_LAUNCH(PC_RMSNORM, launch_rmsnorm<T>(w.h_last, (const T*)job.m->g_final, (T*)w.a_last, n_req, D, d.rms_eps, st));
  RC_LAUNCH(PC_GEMM_LM_HEAD, gemm_any<T>((const T*)w.a_last, (const T*)job.m->w_lm, nullptr, job.logits, n_req, d.vocab, D, d.vocab,
                        EPI_STORE_F32, w.gemm_part, st));
  return RC_OK;
}

rc_status check_seq_fits(const rc_paged_kv* kv, int seq, int len) {
  if (seq < 0 || seq >= kv->n_seq) return RC_E_CAPACITY;
  if ((long)len > (long)kv->max_blocks_per_seq * kv->block_size) return RC_E_CAPACITY;
  return RC_OK;
}

// shared validation of rc_reuse / rc_reuse_workspace_bytes; fills the job's host-side tables
rc_status prepare_reuse(const rc_model* m, const rc_request* reqs, int32_t n_req, const rc_plan* plan, Job* job) {
  if (!m || !reqs || !plan) return RC_E_INVALID_ARG;
  if (n_req < 1) return RC_E_INVALID_ARG;
  if (n_req > RC_MAX_REQ) return RC_E_CAPACITY;
  const rc_model_desc& d = m->d;
  if (!(0 <= plan->l_start && plan->l_start < plan->l_det && plan->l_det <= plan->l_end &&
        plan->l_end < d.n_layers))
    return RC_E_INVALID_ARG;
  const bool by_threshold = plan->selector == RC_SELECT_THRESHOLD;
  if (plan->selector != RC_SELECT_BUDGET && !by_threshold) return RC_E_INVALID_ARG;
  if (!by_threshold && !plan->k_per_req) return RC_E_INVALID_ARG;
  if (by_threshold && (plan->forced_idx || plan->k_suf < 0 || !(plan->tau_dev >= 0.f) || !(plan->tau_inf >= 0.f)))
    return RC_E_INVALID_ARG;
  job->m = m;
  job->selector = plan->selector;
  job->tau_dev = plan->tau_dev;
  job->tau_inf = plan->tau_inf;
  job->k_suf = plan->k_suf;
  job->l_start = plan->l_start;
  job->l_det = plan->l_det;
  job->l_end = plan->l_end;
  job->forced_idx = plan->forced_idx;
  job->k_pre_pool = nullptr;
  job->capture_layer = -1;
  job->base = ReqTable();
  job->base.n_req = n_req;
  int sel = 0, seg = 0, max_pos = 0, max_seg = 0;
  for (int b = 0; b < n_req; ++b) {
    const rc_request& q = reqs[b];
    // threshold selector: sized for the worst case (every token selected) until the counts are known
    const int k = by_threshold ? q.n_seg : plan->k_per_req[b];
    if (q.n_prefix < 0 || q.n_seg < 0 || q.n_suffix < 0) return RC_E_INVALID_ARG;
    if (q.n_prefix + q.n_seg + q.n_suffix < 1) return RC_E_INVALID_ARG;
    if (q.n_prefix > 0 && !q.x_prefix) return RC_E_INVALID_ARG;
    if (q.n_seg > 0 && !q.h_start) return RC_E_INVALID_ARG;
    if (q.n_suffix > 0 && !q.x_suffix) return RC_E_INVALID_ARG;
    if (k < 0 || k > q.n_seg) return RC_E_INVALID_ARG;
    job->s_inf[b] = by_threshold ? q.s_inf : nullptr;
    if (q.src_offset < 0 || q.seg_old_start_pos < 0 || q.n_cached < 0) return RC_E_INVALID_ARG;
    ReqDev& r = job->base.r[b];
    r.P = q.n_prefix; r.S = q.n_seg; r.nsuf = q.n_suffix; r.k = k;
    r.carries_logits = (q.n_suffix == 0 && !q.no_logits) ? 1 : 0;
    r.pos0 = q.n_cached;
    r.dst_seq = q.dst_seq; r.src_seq = q.src_seq; r.src_offset = q.src_offset;
    r.k_is_pre_rope = q.k_is_pre_rope ? 1 : 0;
    r.rot_delta = q.n_cached + q.n_prefix - q.seg_old_start_pos;
    r.sel_base = by_threshold ? seg : sel; r.score_base = seg;
    r.x_prefix = q.x_prefix; r.h_start = q.h_start; r.x_suffix = q.x_suffix; r.h_capture = nullptr;
    sel += k; seg += q.n_seg;
    max_pos = std::max(max_pos, q.n_cached + q.n_prefix + q.n_seg + q.n_suffix);
    max_seg = std::max(max_seg, q.n_seg);
  }
  job->max_pos = max_pos;
  job->sum_seg = seg;
  job->max_seg = max_seg;
  return RC_OK;
}

// floats of partial-attention scratch the largest phase needs (bf16 path only)
size_t attn_part_need(const Job& job) {
  const rc_model_desc& d = job.m->d;
  if (d.dtype != RC_BF16) return 0;
  const int tile_rows = attention_tile_rows(d.dtype, d.n_q_heads, d.n_kv_heads);
  size_t need = 0;
  const bool by_threshold = job.selector == RC_SELECT_THRESHOLD;
  // threshold selector: the row counts of the sparse phase and the one after it are decided on the device
  ThresholdSplit ts{};
  if (by_threshold) ts = plan_threshold_split(job.base, d.n_kv_heads, d.n_q_heads, tile_rows, job.max_pos, true);
  for (int p = 0; p < PH_COUNT; ++p) {
    if (by_threshold && p >= PH_C) {
      need = std::max(need, attention_partial_floats(ts.cap[p], d.n_q_heads));
      continue;
    }
    ReqTable t = job.base;
    fill_phase_table(&t, p, nullptr, tile_rows);
    const AttnSplit sp = plan_phase_split(&t, d.n_kv_heads, d.n_q_heads, tile_rows, job.max_pos);
    need = std::max(need, attention_partial_floats(sp.total_slots, d.n_q_heads));
  }
  return need;
}

int max_rows_of(const Job& job) {
  int r = 0;
  for (int p = 0; p < PH_COUNT; ++p) r = std::max(r, total_rows_in(job.base, (Phase)p));
  return r;
}

}  // namespace

// =================================================================== exported functions
extern "C" {

const char* rc_status_str(rc_status s) {
  switch (s) {
    case RC_OK: return "ok";
    case RC_E_INVALID_ARG: return "invalid argument";
    case RC_E_UNSUPPORTED: return "unsupported configuration";
    case RC_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case RC_E_HIP: return "HIP runtime error";
    case RC_E_CAPACITY: return "capacity exceeded";
    default: return "unknown status";
  }
}

const char* rc_build_info(void) { return "relaycache 0.1 (gfx950, wave64)"; }

rc_status rc_model_create(const rc_model_desc* desc, const rc_layer_w* layers, const void* g_final,
                          const void* w_lm_head, rc_model** out) {
  if (!desc || !layers || !g_final || !w_lm_head || !out) return RC_E_INVALID_ARG;
  RC_TRY(check_desc(*desc));
  for (int l = 0; l < desc->n_layers; ++l) {
    const rc_layer_w& w = layers[l];
    if (!w.wq || !w.wk || !w.wv || !w.wo || !w.w_gate || !w.w_up || !w.w_down || !w.g_attn || !w.g_ffn)
      return RC_E_INVALID_ARG;
  }
  rc_model* m = new (std::nothrow) rc_model();
  if (!m) return RC_E_CAPACITY;
  m->d = *desc;
  m->layers.assign(layers, layers + desc->n_layers);
  m->g_final = g_final;
  m->w_lm = w_lm_head;
  *out = m;
  return RC_OK;
}

rc_status rc_tune_set(int32_t key, int32_t value) {
  if (key == RC_TUNE_GEMM_TILE && (value == 0 || value == 1 || value == 2 || value == 3 || value == 5 || value == 6 || value == 7)) {
    set_gemm_tile(value);
    return RC_OK;
  }
  if (key == RC_TUNE_GEMM_XCD_REMAP && (value == 0 || value == 1)) {
    set_gemm_xcd_remap(value);
    return RC_OK;
  }
  if (key == RC_TUNE_GEMM_THIN_TILES && (value == 0 || value == 1)) {
    set_gemm_thin_tiles(value);
    return RC_OK;
  }
  if (key == RC_TUNE_ATTN_CHUNK_TILES && value >= 0) {
    set_attention_chunk_tiles(value);
    return RC_OK;
  }
  return RC_E_INVALID_ARG;
}

rc_status rc_profile_enable(int32_t on) {
  g_prof.on = on != 0;
  return RC_OK;
}

int32_t rc_profile_class_count(void) { return PC_COUNT; }

const char* rc_profile_class_name(int32_t cls) {
  return (cls >= 0 && cls < PC_COUNT) ? kProfNames[cls] : "";
}

rc_status rc_profile_read(float* ms, int32_t* launches) {
  if (!ms || !launches) return RC_E_INVALID_ARG;
  for (int i = 0; i < PC_COUNT; ++i) { ms[i] = 0.f; launches[i] = 0; }
  rc_status rs = RC_OK;
  for (ProfRec& r : g_prof.recs) {
    float t = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) rs = RC_E_HIP;
    ms[r.cls] += t;
    launches[r.cls] += 1;
    g_prof.pool.push_back(r.a);
    g_prof.pool.push_back(r.b);
  }
  g_prof.recs.clear();
  return rs;
}

rc_status rc_model_destroy(rc_model* m) {
  delete m;
  return RC_OK;
}

size_t rc_reuse_workspace_bytes(const rc_model* m, const rc_request* reqs, int32_t n_req, const rc_plan* plan) {
  Job job;
  if (prepare_reuse(m, reqs, n_req, plan, &job) != RC_OK) return 0;
  return carve(nullptr, m->d, max_rows_of(job), job.max_pos, n_req, job.sum_seg, attn_part_need(job)).bytes;
}

rc_status rc_reuse(const rc_model* m, const rc_request* reqs, int32_t n_req, const rc_plan* plan,
                   const rc_paged_kv* src, const rc_paged_kv* dst, float* logits, int32_t* sel_idx, int32_t* sel_cnt,
                   float* scores, void* workspace, size_t workspace_bytes, void* stream) {
  Job job;
  RC_TRY(prepare_reuse(m, reqs, n_req, plan, &job));
  RC_TRY(check_paged(dst, m->d.n_layers));
  if (!logits) return RC_E_INVALID_ARG;
  int sum_k = 0;
  for (int b = 0; b < n_req; ++b) sum_k += job.base.r[b].k;
  if (sum_k > 0 && !sel_idx) return RC_E_INVALID_ARG;
  if (sum_k > 0 && job.selector == RC_SELECT_THRESHOLD && !sel_cnt) return RC_E_INVALID_ARG;
  if (job.max_seg > 0) RC_TRY(check_paged(src, m->d.n_layers));
  for (int b = 0; b < n_req; ++b) {
    RC_TRY(check_seq_fits(dst, reqs[b].dst_seq, reqs[b].n_cached + reqs[b].n_prefix + reqs[b].n_seg + reqs[b].n_suffix));
    if (reqs[b].n_seg > 0) RC_TRY(check_seq_fits(src, reqs[b].src_seq, reqs[b].src_offset + reqs[b].n_seg));
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RC_E_WORKSPACE;
  Workspace w = carve(workspace, m->d, max_rows_of(job), job.max_pos, n_req, job.sum_seg, attn_part_need(job));
  if (w.bytes > workspace_bytes) return RC_E_WORKSPACE;
  // Source and destination in the same pools: the take-over reads a segment row and writes it at its new position.
  // That is only safe when every row lands on the slot it came from (same block size, segment moved by a whole
  // number of blocks; whether the blocks themselves coincide is the caller's block tables' business).
  if (job.max_seg > 0) {
    bool shared = false;
    for (int l = 0; l < m->d.n_layers; ++l)
      shared = shared || src->k_pool[l] == dst->k_pool[l] || src->v_pool[l] == dst->v_pool[l] ||
               src->k_pool[l] == dst->v_pool[l] || src->v_pool[l] == dst->k_pool[l];
    if (shared) {
      if (src->block_size != dst->block_size) return RC_E_UNSUPPORTED;
      for (int b = 0; b < n_req; ++b)
        if (reqs[b].n_seg > 0 && (reqs[b].n_cached + reqs[b].n_prefix - reqs[b].src_offset) % dst->block_size != 0)
          return RC_E_UNSUPPORTED;
    }
  }
  job.src = src;
  job.dst = dst;
  job.logits = logits;
  job.sel_idx = sel_idx;
  job.sel_cnt = sel_cnt;
  job.scores_out = scores;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return m->d.dtype == RC_BF16 ? run_job<bf16>(job, w, st) : run_job<float>(job, w, st);
}

static rc_status prepare_prefill(const rc_model* m, const void* const* x, const int32_t* n_tokens,
                                 const int32_t* dst_seq, int32_t n_req, void* const* h_capture, Job* job) {
  if (!m || !n_tokens) return RC_E_INVALID_ARG;
  if (n_req < 1) return RC_E_INVALID_ARG;
  if (n_req > RC_MAX_REQ) return RC_E_CAPACITY;
  job->m = m;
  job->l_start = job->l_det = job->l_end = m->d.n_layers;   // every layer is a "before l_start" layer
  job->forced_idx = nullptr;
  job->selector = RC_SELECT_BUDGET;
  job->base = ReqTable();
  job->base.n_req = n_req;
  int max_pos = 0;
  for (int b = 0; b < n_req; ++b) {
    if (n_tokens[b] < 1) return RC_E_INVALID_ARG;
    if (x && !x[b]) return RC_E_INVALID_ARG;
    ReqDev& r = job->base.r[b];
    r.P = n_tokens[b];
    r.dst_seq = dst_seq ? dst_seq[b] : 0;
    r.x_prefix = x ? x[b] : nullptr;
    r.h_capture = h_capture ? h_capture[b] : nullptr;
    max_pos = std::max(max_pos, r.P);
  }
  job->max_pos = max_pos;
  job->sum_seg = 0;
  job->max_seg = 0;
  return RC_OK;
}

size_t rc_prefill_workspace_bytes(const rc_model* m, const int32_t* n_tokens, int32_t n_req) {
  Job job;
  if (prepare_prefill(m, nullptr, n_tokens, nullptr, n_req, nullptr, &job) != RC_OK) return 0;
  return carve(nullptr, m->d, max_rows_of(job), job.max_pos, n_req, 0, attn_part_need(job)).bytes;
}

rc_status rc_prefill(const rc_model* m, const void* const* x, const int32_t* n_tokens, const int32_t* dst_seq,
                     int32_t n_req, const rc_paged_kv* dst, void* const* k_pre_pool, int32_t capture_layer,
                     void* const* h_capture, float* logits, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !dst_seq || !logits) return RC_E_INVALID_ARG;
  Job job;
  RC_TRY(prepare_prefill(m, x, n_tokens, dst_seq, n_req, h_capture, &job));
  RC_TRY(check_paged(dst, m->d.n_layers));
  if (h_capture && (capture_layer < 0 || capture_layer >= m->d.n_layers)) return RC_E_INVALID_ARG;
  if (k_pre_pool)
    for (int l = 0; l < m->d.n_layers; ++l)
      if (!k_pre_pool[l]) return RC_E_INVALID_ARG;
  for (int b = 0; b < n_req; ++b) RC_TRY(check_seq_fits(dst, dst_seq[b], n_tokens[b]));
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RC_E_WORKSPACE;
  Workspace w = carve(workspace, m->d, max_rows_of(job), job.max_pos, n_req, 0, attn_part_need(job));
  if (w.bytes > workspace_bytes) return RC_E_WORKSPACE;
  job.src = nullptr;
  job.dst = dst;
  job.k_pre_pool = k_pre_pool;
  job.capture_layer = h_capture ? capture_layer : -1;
  job.logits = logits;
  job.sel_idx = nullptr;
  job.scores_out = nullptr;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return m->d.dtype == RC_BF16 ? run_job<bf16>(job, w, st) : run_job<float>(job, w, st);
}

// ------------------------------------------------------------------ decoding with the cache manager
static rc_status prepare_decode(const rc_model* m, const rc_decode_req* reqs, int32_t n_req, Job* job) {
  if (!m || !reqs) return RC_E_INVALID_ARG;
  if (n_req < 1) return RC_E_INVALID_ARG;
  if (n_req > RC_MAX_REQ) return RC_E_CAPACITY;
  job->m = m;
  job->l_start = job->l_det = job->l_end = m->d.n_layers;   // every layer only runs the new token
  job->forced_idx = nullptr;
  job->selector = RC_SELECT_BUDGET;
  job->takeover = false;
  job->any_inf = false;
  job->base = ReqTable();
  job->base.n_req = n_req;
  int max_pos = 0, max_seg = 0;
  for (int b = 0; b < n_req; ++b) {
    const rc_decode_req& q = reqs[b];
    if (!q.x || q.pos < 0) return RC_E_INVALID_ARG;
    // the cached rows 0..pos-1 play the part of a reused segment that is already in place; the new token
    // is the one-row suffix behind it
    ReqDev& r = job->base.r[b];
    r.P = 0; r.S = q.pos; r.nsuf = 1; r.k = 0;
    r.dst_seq = q.seq; r.src_seq = q.seq;
    r.x_suffix = q.x;
    r.h_capture = q.h_capture;
    job->inf.s_inf[b] = q.s_inf;
    job->any_inf = job->any_inf || q.s_inf != nullptr;
    max_pos = std::max(max_pos, q.pos + 1);
    max_seg = std::max(max_seg, q.pos);
  }
  for (int b = n_req; b < RC_MAX_REQ; ++b) job->inf.s_inf[b] = nullptr;
  job->max_pos = max_pos;
  job->sum_seg = 0;
  job->max_seg = max_seg;
  return RC_OK;
}

static size_t decode_inf_floats(const Job& job) {
  return job.any_inf ? influence_scratch_floats(job.base.n_req, job.m->d.n_q_heads, job.max_pos) : 0;
}

size_t rc_decode_workspace_bytes(const rc_model* m, const rc_decode_req* reqs, int32_t n_req) {
  Job job;
  if (prepare_decode(m, reqs, n_req, &job) != RC_OK) return 0;
  return carve(nullptr, m->d, max_rows_of(job), job.max_pos, n_req, 0, attn_part_need(job), decode_inf_floats(job)).bytes;
}

rc_status rc_decode_step(const rc_model* m, const rc_decode_req* reqs, int32_t n_req, const rc_paged_kv* cache,
                         void* const* k_pre_pool, int32_t capture_layer, float* logits, void* workspace,
                         size_t workspace_bytes, void* stream) {
  Job job;
  RC_TRY(prepare_decode(m, reqs, n_req, &job));
  RC_TRY(check_paged(cache, m->d.n_layers));
  if (!logits) return RC_E_INVALID_ARG;
  bool any_capture = false;
  for (int b = 0; b < n_req; ++b) {
    RC_TRY(check_seq_fits(cache, reqs[b].seq, reqs[b].pos + 1));
    any_capture = any_capture || reqs[b].h_capture != nullptr;
  }
  if (any_capture && (capture_layer < 0 || capture_layer >= m->d.n_layers)) return RC_E_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RC_E_WORKSPACE;
  Workspace w = carve(workspace, m->d, max_rows_of(job), job.max_pos, n_req, 0, attn_part_need(job), decode_inf_floats(job));
  if (w.bytes > workspace_bytes) return RC_E_WORKSPACE;
  job.src = nullptr;
  job.dst = cache;
  job.k_pre_pool = k_pre_pool;
  job.capture_layer = any_capture ? capture_layer : -1;
  job.logits = logits;
  job.sel_idx = nullptr;
  job.sel_cnt = nullptr;
  job.scores_out = nullptr;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return m->d.dtype == RC_BF16 ? run_job<bf16>(job, w, st) : run_job<float>(job, w, st);
}

// ------------------------------------------------------------------ stage calls
size_t rc_stage_workspace_bytes(int32_t n_positions, int32_t head_dim) {
  if (n_positions < 0 || head_dim < 2) return 0;
  return align_up(sizeof(ReqTable)) + align_up(sizeof(float2) * (size_t)(n_positions + 1) * (head_dim / 2)) +
         align_up(sizeof(float2) * (size_t)(head_dim / 2));
}

// Argument checks shared by rc_rope_rerotate and its allocation-free twin (everything but the scratch).
static rc_status check_rerotate(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset, const rc_kv_layer* dst,
                                int32_t dst_seq, int32_t dst_offset, int32_t n_tokens, int32_t old_start_pos,
                                float rope_base) {
  RC_TRY(check_kv_layer(src));
  RC_TRY(check_kv_layer(dst));
  if (src->n_kv_heads != dst->n_kv_heads || src->head_dim != dst->head_dim || src->dtype != dst->dtype)
    return RC_E_INVALID_ARG;
  if (n_tokens < 0 || src_offset < 0 || dst_offset < 0 || old_start_pos < 0 || !(rope_base > 0.f))
    return RC_E_INVALID_ARG;
  if (src_seq < 0 || src_seq >= src->n_seq || dst_seq < 0 || dst_seq >= dst->n_seq) return RC_E_CAPACITY;
  if ((long)src_offset + n_tokens > (long)src->max_blocks_per_seq * src->block_size ||
      (long)dst_offset + n_tokens > (long)dst->max_blocks_per_seq * dst->block_size)
    return RC_E_CAPACITY;
  return RC_OK;
}

// The launches of the re-rotation stage; `scratch` holds rc_stage_workspace_bytes(dst_offset + n_tokens, head_dim)
// bytes of device memory: the request table, then the rotary table, then the delta table.
static rc_status enqueue_rerotate(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset, const rc_kv_layer* dst,
                                  int32_t dst_seq, int32_t dst_offset, int32_t n_tokens, int32_t k_is_pre_rope,
                                  int32_t old_start_pos, float rope_base, void* scratch, hipStream_t st) {
  const int n_pos = dst_offset + n_tokens;
  char* p = reinterpret_cast<char*>(scratch);
  ReqTable* dt = reinterpret_cast<ReqTable*>(p);
  float2* rope_tab = reinterpret_cast<float2*>(p + align_up(sizeof(ReqTable)));
  float2* delta_tab = reinterpret_cast<float2*>(p + align_up(sizeof(ReqTable)) +
                                                align_up(sizeof(float2) * (size_t)(n_pos + 1) * (src->head_dim / 2)));
  ReqTable t = ReqTable();
  t.n_req = 1;
  ReqDev& r = t.r[0];
  r.P = dst_offset; r.S = n_tokens; r.src_seq = src_seq; r.src_offset = src_offset; r.dst_seq = dst_seq;
  r.k_is_pre_rope = k_is_pre_rope ? 1 : 0;
  r.rot_delta = dst_offset - old_start_pos;
  RC_HIP(launch_upload_table(t, dt, st));
  const int half = src->head_dim / 2;
  if (k_is_pre_rope) RC_HIP(launch_rope_table(rope_tab, n_pos, half, (double)rope_base, st));
  else RC_HIP(launch_delta_table(delta_tab, dt, 1, half, (double)rope_base, st));
  RerotatePtrs ptrs;
  ptrs.k_src[0] = src->k; ptrs.v_src[0] = src->v; ptrs.k_dst[0] = dst->k; ptrs.v_dst[0] = dst->v;
  if (src->dtype == RC_BF16)
    RC_HIP(launch_rerotate<bf16>(ptrs, 1, geom_of(*src), geom_of(*dst), dt, 1, n_tokens, rope_tab, delta_tab, st));
  else
    RC_HIP(launch_rerotate<float>(ptrs, 1, geom_of(*src), geom_of(*dst), dt, 1, n_tokens, rope_tab, delta_tab, st));
  return RC_OK;
}

rc_status rc_rope_rerotate(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset, const rc_kv_layer* dst,
                           int32_t dst_seq, int32_t dst_offset, int32_t n_tokens, int32_t k_is_pre_rope,
                           int32_t old_start_pos, float rope_base, void* workspace, size_t workspace_bytes,
                           void* stream) {
  RC_TRY(check_rerotate(src, src_seq, src_offset, dst, dst_seq, dst_offset, n_tokens, old_start_pos, rope_base));
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RC_E_WORKSPACE;
  if (rc_stage_workspace_bytes(dst_offset + n_tokens, src->head_dim) > workspace_bytes) return RC_E_WORKSPACE;
  if (n_tokens == 0) return RC_OK;
  return enqueue_rerotate(src, src_seq, src_offset, dst, dst_seq, dst_offset, n_tokens, k_is_pre_rope, old_start_pos,
                          rope_base, workspace, reinterpret_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------ the same stage without any allocation
// The scratch of the re-rotation stage (request table, rotary table, delta table) lives in a device array of the
// library instead of a caller's workspace.  Every GPU holds its own copy of the array at its own address; host code
// never uses the array's name as an address, only what hipGetSymbolAddress returned for the current device.
static constexpr int kStaticMaxPositions = RC_REROTATE_STATIC_MAX_POSITIONS;
static constexpr size_t kStaticScratchBytes =
    ((sizeof(ReqTable) + 255) / 256 * 256) + (size_t)(kStaticMaxPositions + 1) * 64 * sizeof(float2) + 256 +
    64 * sizeof(float2) + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// device address of `scratch` on the current device, looked up once per device
static rc_status static_scratch(void** out) {
  int dev = 0;
  RC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RC_E_CAPACITY;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    RC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return RC_E_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return RC_OK;
}

size_t rc_rope_rerotate_static_scratch_bytes(void) { return kStaticScratchBytes; }

rc_status rc_rope_rerotate_static(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset, const rc_kv_layer* dst,
                                  int32_t dst_seq, int32_t dst_offset, int32_t n_tokens, int32_t k_is_pre_rope,
                                  int32_t old_start_pos, float rope_base, void* stream) {
  RC_TRY(check_rerotate(src, src_seq, src_offset, dst, dst_seq, dst_offset, n_tokens, old_start_pos, rope_base));
  if ((long)dst_offset + n_tokens > kStaticMaxPositions) return RC_E_CAPACITY;
  if (rc_stage_workspace_bytes(dst_offset + n_tokens, src->head_dim) > kStaticScratchBytes) return RC_E_CAPACITY;
  if (n_tokens == 0) return RC_OK;
  void* ptr = nullptr;
  RC_TRY(static_scratch(&ptr));
  // every byte of the scratch that the kernels read is written earlier in the same call (tables), so nothing
  // has to be cleared between calls
  return enqueue_rerotate(src, src_seq, src_offset, dst, dst_seq, dst_offset, n_tokens, k_is_pre_rope, old_start_pos,
                          rope_base, ptr, reinterpret_cast<hipStream_t>(stream));
}

rc_status rc_vdev_score(const void* v_fresh, const rc_kv_layer* cache, int32_t seq, int32_t offset,
                        int32_t n_tokens, float* score, void* workspace, size_t workspace_bytes, void* stream) {
  RC_TRY(check_kv_layer(cache));
  if (!v_fresh || !score || n_tokens < 0 || offset < 0) return RC_E_INVALID_ARG;
  if (seq < 0 || seq >= cache->n_seq) return RC_E_CAPACITY;
  if ((long)offset + n_tokens > (long)cache->max_blocks_per_seq * cache->block_size) return RC_E_CAPACITY;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RC_E_WORKSPACE;
  if (rc_stage_workspace_bytes(0, cache->head_dim) > workspace_bytes) return RC_E_WORKSPACE;
  if (n_tokens == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  ReqTable* dt = reinterpret_cast<ReqTable*>(workspace);
  ReqTable t = ReqTable();
  t.n_req = 1;
  ReqDev& r = t.r[0];
  r.P = offset; r.S = n_tokens; r.dst_seq = seq; r.seg_mode = SEG_ALL;
  r.row_base = -offset;   // fresh row of token j is j
  r.score_base = 0;
  RC_HIP(launch_upload_table(t, dt, st));
  const int stride = cache->n_kv_heads * cache->head_dim;
  if (cache->dtype == RC_BF16)
    RC_HIP(launch_vdev_score<bf16>((const bf16*)v_fresh, stride, (const bf16*)cache->v, geom_of(*cache), dt, 1,
                                   n_tokens, score, st));
  else
    RC_HIP(launch_vdev_score<float>((const float*)v_fresh, stride, (const float*)cache->v, geom_of(*cache), dt, 1,
                                    n_tokens, score, st));
  return RC_OK;
}

rc_status rc_topk(const float* score, int32_t n, int32_t k, int32_t* idx_out, void* stream) {
  if (n < 0 || k < 0 || k > n) return RC_E_INVALID_ARG;
  if (n > (1 << 20)) return RC_E_CAPACITY;
  if (k == 0) return RC_OK;
  if (!score || !idx_out) return RC_E_INVALID_ARG;
  RC_HIP(launch_topk(score, n, k, idx_out, reinterpret_cast<hipStream_t>(stream)));
  return RC_OK;
}

rc_status rc_threshold_select(const float* score, int32_t n, float tau, int32_t* idx_out, int32_t* count_out,
                              void* stream) {
  if (n < 1 || !score || !idx_out || !count_out) return RC_E_INVALID_ARG;
  if (n > (1 << 20)) return RC_E_CAPACITY;
  RC_HIP(launch_threshold_select(score, n, tau, idx_out, count_out, reinterpret_cast<hipStream_t>(stream)));
  return RC_OK;
}

rc_status rc_final_select(const float* s_dev, const float* s_inf, int32_t n, float tau_dev, float tau_inf,
                          int32_t k_suf, int32_t* idx_out, int32_t* count_out, void* stream) {
  if (n < 1 || k_suf < 0 || !s_dev || !idx_out || !count_out) return RC_E_INVALID_ARG;
  if (n > (1 << 20)) return RC_E_CAPACITY;
  RC_HIP(launch_final_select(s_dev, s_inf, n, tau_dev, tau_inf, k_suf, idx_out, count_out,
                             reinterpret_cast<hipStream_t>(stream)));
  return RC_OK;
}

// stage call: positions live on the device, so the plan only looks at the row count and the cache capacity
static AttnSplit plan_stage_split(int tiles, int n_kv_heads, int capacity) {
  int chunk_tiles, thr;
  const int forced = attention_forced_chunk_tiles();
  if (forced > 0) {
    chunk_tiles = thr = forced;
  } else {
    if ((long)tiles * n_kv_heads >= 1024) return attention_no_split();
    thr = kLongKvTiles;
    chunk_tiles = (long)tiles * n_kv_heads >= 128 ? 16 : 4;
  }
  const int n_chunks = ((capacity + kKvTile - 1) / kKvTile + chunk_tiles - 1) / chunk_tiles;
  if (n_chunks <= 1) return attention_no_split();
  AttnSplit sp = {n_chunks, chunk_tiles, thr, tiles * n_chunks};
  return sp;
}

size_t rc_sparse_attention_workspace_bytes(int32_t n, int32_t n_q_heads, const rc_kv_layer* cache) {
  if (!cache || n < 1 || n_q_heads < 1 || cache->dtype != RC_BF16 || cache->n_kv_heads < 1) return 0;
  const int tile_rows = attention_tile_rows(cache->dtype, n_q_heads, cache->n_kv_heads);
  const int tiles = (n + tile_rows - 1) / tile_rows;
  const AttnSplit sp = plan_stage_split(tiles, cache->n_kv_heads, cache->max_blocks_per_seq * cache->block_size);
  return align_up(sizeof(float) * attention_partial_floats(sp.total_slots, n_q_heads));
}

rc_status rc_sparse_attention(const void* q, const int32_t* q_pos, int32_t n, int32_t n_q_heads,
                              const rc_kv_layer* cache, int32_t seq, void* out, void* workspace,
                              size_t workspace_bytes, void* stream) {
  RC_TRY(check_kv_layer(cache));
  if (!q || !q_pos || !out || n < 0 || n_q_heads < 1 || n_q_heads % cache->n_kv_heads) return RC_E_INVALID_ARG;
  if (seq < 0 || seq >= cache->n_seq) return RC_E_CAPACITY;
  if (n == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int tile_rows = attention_tile_rows(cache->dtype, n_q_heads, cache->n_kv_heads);
  const int tiles = (n + tile_rows - 1) / tile_rows;
  if (cache->dtype == RC_BF16) {
    AttnSplit sp = attention_no_split();
    float* part = nullptr;
    if (workspace) {
      if (reinterpret_cast<uintptr_t>(workspace) & 255u) return RC_E_WORKSPACE;
      if (rc_sparse_attention_workspace_bytes(n, n_q_heads, cache) > workspace_bytes) return RC_E_WORKSPACE;
      sp = plan_stage_split(tiles, cache->n_kv_heads, cache->max_blocks_per_seq * cache->block_size);
      part = reinterpret_cast<float*>(workspace);
    }
    RC_HIP(launch_attention_bf16((const bf16*)q, q_pos, nullptr, nullptr, seq, n, tiles, (const bf16*)cache->k,
                                 (const bf16*)cache->v, geom_of(*cache), n_q_heads, (bf16*)out, sp, part, st));
  } else {
    RC_HIP(launch_attention<float>((const float*)q, q_pos, nullptr, nullptr, seq, n, tiles, (const float*)cache->k,
                                   (const float*)cache->v, geom_of(*cache), n_q_heads, (float*)out, st));
  }
  return RC_OK;
}

int32_t rc_gemm_plan_check(int32_t m, int32_t n, int32_t k, int32_t swiglu, int32_t tile, int32_t n_cus,
                           int32_t with_workspace, int32_t* n_blocks) {
  if (m < 1 || n < 1 || k < 64 || (k % 64) != 0 || n_cus < 1 || (tile != 5 && tile != 6 && tile != 7)) return -1;
  return check_grid_plan(m, n, k, swiglu != 0, tile, n_cus, with_workspace != 0, n_blocks);
}

rc_status rc_ceiling_stream_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || (bytes % 16) != 0) return RC_E_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return RC_E_INVALID_ARG;
  RC_HIP(launch_stream_copy(src, dst, bytes, reinterpret_cast<hipStream_t>(stream)));
  return RC_OK;
}

size_t rc_ceiling_mfma_loop_out_bytes(int32_t n_workgroups) {
  return n_workgroups > 0 ? mfma_loop_out_floats(n_workgroups) * sizeof(float) : 0;
}

rc_status rc_ceiling_mfma_loop(float* out, int32_t n_workgroups, int32_t iters, double* flops, void* stream) {
  if (!out || n_workgroups < 1 || n_workgroups > 65536 || iters < 1 || iters > (1 << 24)) return RC_E_INVALID_ARG;
  if (flops) *flops = mfma_loop_flops(n_workgroups, iters);
  RC_HIP(launch_mfma_loop(out, n_workgroups, iters, reinterpret_cast<hipStream_t>(stream)));
  return RC_OK;
}

size_t rc_gemm_workspace_bytes(void) { return align_up(gemm_partial_bytes()); }

rc_status rc_gemm_rows(int32_t dtype, const void* a, const void* w, float* c, int32_t m, int32_t n, int32_t k,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (dtype != RC_F32 && dtype != RC_BF16) return RC_E_INVALID_ARG;
  if (!a || !w || !c || m < 0 || n < 1 || k < 1) return RC_E_INVALID_ARG;
  if (k % 8) return RC_E_UNSUPPORTED;
  if (workspace && ((reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < rc_gemm_workspace_bytes()))
    return RC_E_WORKSPACE;
  if (m == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (dtype == RC_BF16)
    RC_HIP(launch_gemm_bf16((const bf16*)a, (const bf16*)w, nullptr, c, m, n, k, n, EPI_STORE_F32,
                            reinterpret_cast<float*>(workspace), st));
  else
    RC_HIP(launch_gemm<float>((const float*)a, (const float*)w, nullptr, c, m, n, k, n, EPI_STORE_F32, st));
  return RC_OK;
}

rc_status rc_gemm_rows_fused(int32_t dtype, int32_t epilogue, const void* a, const void* w, const void* w2, void* c,
                             int32_t m, int32_t n, int32_t k, void* workspace, size_t workspace_bytes, void* stream) {
  if (dtype != RC_F32 && dtype != RC_BF16) return RC_E_INVALID_ARG;
  if (epilogue < RC_GEMM_STORE || epilogue > RC_GEMM_SWIGLU) return RC_E_INVALID_ARG;
  if (!a || !w || !c || m < 0 || n < 1 || k < 1) return RC_E_INVALID_ARG;
  if ((epilogue == RC_GEMM_SWIGLU) != (w2 != nullptr)) return RC_E_INVALID_ARG;
  if (k % 8) return RC_E_UNSUPPORTED;
  if (workspace && ((reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < rc_gemm_workspace_bytes()))
    return RC_E_WORKSPACE;
  if (m == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  static_assert((int)RC_GEMM_STORE == (int)EPI_STORE_F32 && (int)RC_GEMM_STORE_T == (int)EPI_STORE_T &&
                (int)RC_GEMM_ADD == (int)EPI_ADD_F32 && (int)RC_GEMM_SWIGLU == (int)EPI_SWIGLU_T, "epilogue codes");
  const GemmEpilogue epi = static_cast<GemmEpilogue>(epilogue);
  if (dtype == RC_BF16)
    RC_HIP(gemm_any<bf16>((const bf16*)a, (const bf16*)w, (const bf16*)w2, c, m, n, k, n, epi,
                          reinterpret_cast<float*>(workspace), st));
  else
    RC_HIP(gemm_any<float>((const float*)a, (const float*)w, (const float*)w2, c, m, n, k, n, epi, nullptr, st));
  return RC_OK;
}

size_t rc_rope_scatter_workspace_bytes(int32_t n, const rc_kv_layer* dst) {
  if (!dst || n < 0 || dst->max_blocks_per_seq < 1 || dst->block_size < 1 || dst->head_dim < 2) return 0;
  const long capacity = (long)dst->max_blocks_per_seq * dst->block_size;
  if (capacity > (1 << 24)) return 0;
  return rc_stage_workspace_bytes((int)capacity, dst->head_dim);
}

rc_status rc_rope_scatter(const float* qkv, const int32_t* pos, int32_t n, int32_t n_q_heads, float rope_base,
                          const rc_kv_layer* dst, int32_t seq, void* q_out, void* workspace, size_t workspace_bytes,
                          void* stream) {
  RC_TRY(check_kv_layer(dst));
  if (!qkv || !pos || !q_out || n < 0 || n_q_heads < 1 || n_q_heads % dst->n_kv_heads || !(rope_base > 0.f))
    return RC_E_INVALID_ARG;
  if (seq < 0 || seq >= dst->n_seq) return RC_E_CAPACITY;
  const size_t need = rc_rope_scatter_workspace_bytes(n, dst);
  if (need == 0) return RC_E_CAPACITY;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || need > workspace_bytes) return RC_E_WORKSPACE;
  if (n == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int capacity = dst->max_blocks_per_seq * dst->block_size;
  char* p = reinterpret_cast<char*>(workspace);
  ReqTable* dt = reinterpret_cast<ReqTable*>(p);
  float2* rope_tab = reinterpret_cast<float2*>(p + align_up(sizeof(ReqTable)));
  ReqTable t = ReqTable();
  t.n_req = 1;
  t.total_rows = n;
  t.r[0].dst_seq = seq;
  t.r[0].n_rows = n;
  RC_HIP(launch_upload_table(t, dt, st));
  RC_HIP(launch_rope_table(rope_tab, capacity, dst->head_dim / 2, (double)rope_base, st));
  const int* row_req = nullptr;   // every row belongs to request 0
  if (dst->dtype == RC_BF16)
    RC_HIP(launch_rope_scatter<bf16>(qkv, n, pos, row_req, dt, rope_tab, (bf16*)q_out, (bf16*)dst->k, (bf16*)dst->v, nullptr,
                                     geom_of(*dst), n_q_heads, st));
  else
    RC_HIP(launch_rope_scatter<float>(qkv, n, pos, row_req, dt, rope_tab, (float*)q_out, (float*)dst->k, (float*)dst->v,
                                      nullptr, geom_of(*dst), n_q_heads, st));
  return RC_OK;
}

rc_status rc_scatter_paged(const void* k_rows, const void* v_rows, const int32_t* pos, int32_t n,
                           const rc_kv_layer* dst, int32_t seq, void* stream) {
  RC_TRY(check_kv_layer(dst));
  if (!k_rows || !v_rows || !pos || n < 0) return RC_E_INVALID_ARG;
  if (seq < 0 || seq >= dst->n_seq) return RC_E_CAPACITY;
  if (n == 0) return RC_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (dst->dtype == RC_BF16)
    RC_HIP(launch_scatter_rows<bf16>((const bf16*)k_rows, (const bf16*)v_rows, pos, n, (bf16*)dst->k, (bf16*)dst->v,
                                     geom_of(*dst), seq, st));
  else
    RC_HIP(launch_scatter_rows<float>((const float*)k_rows, (const float*)v_rows, pos, n, (float*)dst->k,
                                      (float*)dst->v, geom_of(*dst), seq, st));
  return RC_OK;
}

}  // extern "C"
