/*
 * relaycache.h -- C ABI of the MI355X (gfx950) selective-recompute prefill.
 *
 * The library implements the prefill side of RelayCaching (Section 4; Figure
 * "Overview of RelayCaching", item 3): a later agent takes over the KV cache
 * that an earlier agent produced for a shared segment, moves the reused keys
 * to their new positions, recomputes the layers [l_start, l_det) for every
 * segment token from cached hidden states, scores each token's value
 * deviation at l_det (Eq. 1), picks a budget of k tokens, recomputes only
 * those tokens through [l_det, l_end], writes their K/V rows back into a paged
 * cache and returns first-token logits.
 *
 * General conventions
 *   - Structs are host memory and are only read during the call.  Every data
 *     pointer inside them is DEVICE memory owned by the caller unless the field
 *     comment says "host".  The library never frees or keeps caller memory.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and is asynchronous: outputs are valid after the
 *     caller synchronises the stream.
 *   - Argument errors are detected on the host before anything is launched and
 *     reported as a negative rc_status; nothing aborts or throws across the ABI.
 *   - Element type `T` is float (RC_F32) or bfloat16 (RC_BF16).  RC_BF16 needs
 *     head_dim == 128; RC_F32 needs head_dim <= 128 and a multiple of 4.
 *   - Weights are row-major [out][in]: y = x W^T.
 *   - One layer's K (or V) pool is [n_blocks][n_kv_heads][block_size][head_dim]
 *     of T.  Position p of sequence s lives in block block_table[s][p / block_size]
 *     at slot p % block_size.  A contiguous cache is the special case of one
 *     block per sequence with block_size >= sequence length.
 *   - Block-table entries outside [0, n_blocks) are clamped by the kernels
 *     (wrong data, never a wild access).
 */
#ifndef RELAYCACHE_H
#define RELAYCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RC_API __attribute__((visibility("default")))

typedef enum {
  RC_OK = 0,
  RC_E_INVALID_ARG = -1, /* null pointer, negative size, inconsistent shape, bad layer triple */
  RC_E_UNSUPPORTED = -2, /* valid request the kernels do not cover (e.g. head_dim) */
  RC_E_WORKSPACE = -3,   /* workspace pointer null/misaligned or too small */
  RC_E_HIP = -4,         /* a HIP runtime call failed */
  RC_E_CAPACITY = -5     /* too many requests in one call, sequence longer than its block table */
} rc_status;

typedef enum { RC_F32 = 0, RC_BF16 = 1 } rc_dtype;

#define RC_MAX_REQ 32      /* requests per rc_reuse / rc_prefill call */
#define RC_MAX_LAYERS 128

RC_API const char* rc_status_str(rc_status s);
/* Library version, and the gfx target the kernels were compiled for ("gfx950"). */
RC_API const char* rc_build_info(void);

/* ------------------------------------------------------------------ model */

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base; /* rotary base; pair i of a head couples elements (i, i+head_dim/2) */
  float rms_eps;
  int32_t dtype;   /* rc_dtype of weights, activations handed in, and KV pools */
} rc_model_desc;

typedef struct {
  const void *wq, *wk, *wv; /* [Hq*dh][d], [Hkv*dh][d], [Hkv*dh][d] of T */
  const void *wo;           /* [d][Hq*dh] */
  const void *w_gate, *w_up;/* [F][d] */
  const void *w_down;       /* [d][F] */
  const void *g_attn, *g_ffn; /* RMSNorm gains [d] of T */
} rc_layer_w;

typedef struct rc_model rc_model;

/* Records shapes and weight pointers (no copy; the buffers must outlive the handle).
 * layers: host array [n_layers].  g_final [d], w_lm_head [vocab][d] of T. */
RC_API rc_status rc_model_create(const rc_model_desc* desc, const rc_layer_w* layers, const void* g_final,
                          const void* w_lm_head, rc_model** out);
RC_API rc_status rc_model_destroy(rc_model* m);

/* --------------------------------------------------------------- KV cache */

typedef struct {
  void* const* k_pool;        /* host array [n_layers] of device pointers */
  void* const* v_pool;        /* host array [n_layers] of device pointers */
  int32_t n_blocks;           /* blocks in every pool */
  int32_t block_size;         /* tokens per block */
  const int32_t* block_table; /* device [n_seq][max_blocks_per_seq] */
  int32_t n_seq;
  int32_t max_blocks_per_seq;
} rc_paged_kv;

/* One layer of a paged cache, for the stage-level calls. */
typedef struct {
  void* k;
  void* v;
  int32_t n_blocks, block_size;
  const int32_t* block_table; /* device [n_seq][max_blocks_per_seq] */
  int32_t n_seq, max_blocks_per_seq;
  int32_t n_kv_heads, head_dim;
  int32_t dtype;
} rc_kv_layer;

/* ---------------------------------------------------------------- request */

/* One later-agent prefill: [new prefix ; reused segment ; optional new suffix].
 * Positions: prefix 0..P-1, segment P..P+S-1, suffix P+S.. */
typedef struct {
  int32_t n_prefix;      /* P >= 0 */
  const void* x_prefix;  /* [P][d] of T: layer-0 inputs of the new prefix */
  int32_t n_seg;         /* S >= 0 */
  const void* h_start;   /* [S][d] of T: segment hidden states entering layer l_start, cached by the
                            earlier agent (Section 4.2, "Start layer") */
  int32_t n_suffix;      /* tokens after the segment, may be 0 */
  const void* x_suffix;  /* [n_suffix][d] of T */
  int32_t src_seq;       /* row of the source block table holding the earlier agent's sequence */
  int32_t src_offset;    /* position of the segment's first token inside that sequence */
  int32_t k_is_pre_rope; /* 1: source keys are stored before rotation (Figure "Overview", item 2);
                            0: they carry the rotation of positions seg_old_start_pos + j */
  int32_t seg_old_start_pos;
  int32_t dst_seq;       /* row of the destination block table */
  const float* s_inf;    /* optional [S] float: influence scores the earlier agent accumulated while decoding
                            (Eq. 6); only read by the threshold selector; NULL: no influence term */
  int32_t n_cached;      /* rows 0..n_cached-1 of dst_seq are already final (an earlier call wrote them): the
                            request's first token sits at position n_cached and attends over them.  A prompt
                            with several reused segments from different agents (a relay chain) is taken over
                            piece by piece, [new text ; segment] per call on the same dst_seq; under causal
                            attention this equals one pass over the whole prompt. */
  int32_t no_logits;     /* 1: not the last piece: with n_suffix == 0 the last segment token is not kept
                            live for the logits (this request's logits row is then undefined) */
} rc_request;

typedef enum {
  RC_SELECT_BUDGET = 0,    /* the k_per_req[b] tokens with the largest deviation (ties to the lower index) */
  RC_SELECT_THRESHOLD = 1  /* the paper's selector, Eq. (5)-(10): deviation >= tau_dev * mean, united with
                              influence >= tau_inf * mean (if s_inf is given) and the last k_suf tokens */
} rc_selector;

typedef struct {
  int32_t l_start, l_det, l_end; /* 0-based; 0 <= l_start < l_det <= l_end < n_layers.
                                    h_start is the input of layer l_start; layers [l_start, l_det)
                                    are recomputed for all S tokens, [l_det, l_end] for selected
                                    tokens only (both ends included). */
  const int32_t* k_per_req;      /* host [n_req]: recompute budget as a token count, 0 <= k <= S
                                    (RC_SELECT_BUDGET; ignored by RC_SELECT_THRESHOLD) */
  const int32_t* forced_idx;     /* device, optional, budget selector only: concatenated per request,
                                    k_per_req[b] ascending segment indices that replace the top-k result
                                    (scores are still computed).  NULL: select by score. */
  int32_t selector;              /* rc_selector */
  float tau_dev, tau_inf;        /* Eq. (5), Eq. (7) scaling factors (paper defaults 1.5, 1.45) */
  int32_t k_suf;                 /* Eq. (8)-(9): trailing segment tokens always selected (paper default 10) */
} rc_plan;

/* Workspace size for rc_reuse with these requests (0 on invalid arguments). */
RC_API size_t rc_reuse_workspace_bytes(const rc_model* m, const rc_request* reqs, int32_t n_req,
                                const rc_plan* plan);

/* The selective-recompute prefill (Section 4.2, paragraph after Eq. 4; Eq. 1; Figure "Overview", item 3).
 *
 *   src      the earlier agent's cache (read only).  It may share pools with dst (a take-over in place) only
 *            if both have the same block size and every segment moves by a whole number of blocks,
 *            (n_cached + n_prefix - src_offset) % block_size == 0, so that each row lands on the slot it came
 *            from; otherwise RC_E_UNSUPPORTED (checked on the host, last of the argument checks).  Whether the
 *            two block tables then name the same blocks (rows rotated in place) or different ones (a copy
 *            inside one pool) is up to the caller; partial overlaps of the two are the caller's error.
 *   dst      in/out: on return rows 0..P+S+n_suffix-1 of every layer of sequence dst_seq hold
 *            the corrected cache: new tokens' K/V, re-rotated reused K/V, recomputed rows.
 *   logits   [n_req][vocab] float: logits of the last position of each request.
 *   sel_idx  budget selector: [sum k_per_req] int32, per request ascending: the k tokens with the
 *            largest deviation at l_det, equal scores resolved to the lower index.
 *            threshold selector: [sum n_seg] int32; request b's selection starts at the sum of the
 *            earlier requests' n_seg, ascending, sel_cnt[b] entries.
 *   sel_cnt  threshold selector: [n_req] int32 (device), number of selected tokens per request
 *            (requests without a segment are left untouched); may be NULL for the budget selector.
 *            The threshold selector's row counts are only known after scoring, and they stay on the
 *            device: from l_det on every launch is sized for the bound "all tokens selected" and the
 *            kernels read the live counts from device memory, so the call enqueues and returns like
 *            the budget path (it can be captured in a HIP graph); the workspace is sized for the bound.
 *   scores   optional [sum n_seg] float: Eq. (1) at l_det for every segment token of every
 *            request with k > 0 (others untouched); NULL to skip.
 *   With n_suffix == 0 the last segment token is recomputed from l_start to the last layer in
 *   addition to the k selected ones (it yields the logits); it is not listed in sel_idx.
 *   k == 0 for a request skips its dense layers too (pure reuse).
 *
 * Errors: RC_E_INVALID_ARG (nulls, triple, k out of range, n_seg == 0 with no new token),
 * RC_E_CAPACITY (n_req > RC_MAX_REQ, sequence longer than max_blocks_per_seq * block_size,
 * seq index out of range), RC_E_UNSUPPORTED (dtype/head_dim; src and dst sharing pools with a segment
 * that does not move by whole blocks), RC_E_WORKSPACE. */
RC_API rc_status rc_reuse(const rc_model* m, const rc_request* reqs, int32_t n_req, const rc_plan* plan,
                   const rc_paged_kv* src, const rc_paged_kv* dst, float* logits, int32_t* sel_idx,
                   int32_t* sel_cnt, float* scores, void* workspace, size_t workspace_bytes, void* stream);

/* FULL baseline (Appendix "Baseline Descriptions") and the earlier agent's side: a plain causal
 * prefill of n_req sequences of new tokens, written into dst.  Optionally records what the cache
 * manager keeps for later reuse (Figure "Overview", item 2): keys before rotation and the hidden
 * states entering layer `capture_layer`.
 *   x[b]        [n_tokens[b]][d] of T (host array of device pointers)
 *   dst_seq     host [n_req] rows of dst's block table
 *   k_pre_pool  optional host array [n_layers] of device pools with dst's geometry receiving
 *               un-rotated keys; NULL to skip
 *   h_capture   optional host array [n_req] of device [n_tokens[b]][d] of T receiving the hidden
 *               states entering capture_layer; NULL to skip
 *   logits      [n_req][vocab] float, last position of each sequence */
RC_API size_t rc_prefill_workspace_bytes(const rc_model* m, const int32_t* n_tokens, int32_t n_req);
RC_API rc_status rc_prefill(const rc_model* m, const void* const* x, const int32_t* n_tokens,
                     const int32_t* dst_seq, int32_t n_req, const rc_paged_kv* dst,
                     void* const* k_pre_pool, int32_t capture_layer, void* const* h_capture,
                     float* logits, void* workspace, size_t workspace_bytes, void* stream);

/* One decoding step of the earlier agent with the cache manager's bookkeeping (Figure "Overview", item 2;
 * Eq. 6): the new token of each of n_req sequences runs through every layer, attending over the rows
 * its sequence already has in `cache` and itself; its K/V row is appended at position `pos`.
 * Optionally the step also records what a later selective-recompute prefill needs:
 *   k_pre_pool  host array [n_layers] of device pools with the cache's geometry that receive the
 *               key before rotation at the same (seq, pos); NULL to skip
 *   h_capture   per request, device [d] of T receiving the hidden state entering capture_layer
 *   s_inf       per request, device float [pos + 1]: s_inf[j] += the attention weight the new token puts
 *               on position j, summed over all layers and query heads (its weight on itself included).
 *               The caller zeroes the vector before the first step and keeps passing it; rows of
 *               the reused segment are a slice of it.
 *   logits      [n_req][vocab] float: next-token logits.
 * Errors as rc_prefill; RC_E_CAPACITY if pos + 1 exceeds the sequence's capacity. */
typedef struct {
  const void* x;     /* device [d] of T: input hidden state of the new token */
  int32_t pos;       /* its position = number of rows the sequence already holds */
  int32_t seq;       /* row of the cache's block table */
  void* h_capture;   /* optional */
  float* s_inf;      /* optional */
} rc_decode_req;
RC_API size_t rc_decode_workspace_bytes(const rc_model* m, const rc_decode_req* reqs, int32_t n_req);
RC_API rc_status rc_decode_step(const rc_model* m, const rc_decode_req* reqs, int32_t n_req, const rc_paged_kv* cache,
                         void* const* k_pre_pool, int32_t capture_layer, float* logits, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Offline layer-range profiler (Section 4.2, Eq. 2-4; Appendix table "Hyperparameters for Critical Layer
 * Selection").  Host function on host memory: d is [n_layers][n_tokens] float, row l = Eq. (1) of every
 * calibration token at layer l (what rc_vdev_score returns for that layer, copied to the host).
 *   s_l (Eq. 2) = mean_j (1 - d[l][j]);  l_min = argmin s.
 *   l_start = deepest l <= l_min with s_l >= tau_st (0 if none).
 *   l_end: b = mean - std (population) of s over the last `tail` layers; scanning l = l_min, l_min+1, ...:
 *          the first l whose next `consecutive` layers all have s >= b and |s_l' - s_{l'-1}| < lambda * std;
 *          the last layer if there is none; never below l_start + 1.
 *   l_det: rho_l = Spearman correlation (average ranks for ties) of rows l-1 and l; alpha_l = rho_l -
 *          2 rho_{l-1} + rho_{l-2} (l >= 3); l* = first l with alpha_{l-1} > 0 > alpha_l and l_start < l*+1 <=
 *          l_end; l_det = l* + 1 (l_start + 1 if there is none).
 * Indices are rows of d.  s_out / rho_out (optional, host, [n_layers] double) receive s_l and rho_l.
 * The "min rise samples" hyper-parameter of the appendix table is not used by the paper's rules. */
typedef struct {
  float tau_st;          /* 0.99 */
  int32_t tail;          /* T = 5 */
  float lambda;          /* 2.0 */
  int32_t consecutive;   /* C = 2 */
} rc_layer_profile_params;
typedef struct { int32_t l_start, l_det, l_end; } rc_layer_triple;
RC_API rc_status rc_layer_profile(const float* d, int32_t n_layers, int32_t n_tokens,
                           const rc_layer_profile_params* params, rc_layer_triple* out, double* s_out,
                           double* rho_out);

/* ---------------------------------------------------------------- timing
 * Optional per-stage GPU timing of rc_reuse / rc_prefill (the per-stage latency split the paper
 * reports in its Table "Per-agent TTFT breakdown").  While enabled, every kernel launch of those two
 * calls is bracketed by a pair of HIP events on the call's stream.  rc_profile_read waits for the
 * recorded events, adds up milliseconds and launch counts per stage class into ms / launches (host
 * arrays of rc_profile_class_count() entries) and forgets them.  Process-global, not thread-safe. */
RC_API rc_status rc_profile_enable(int32_t on);
RC_API int32_t rc_profile_class_count(void);
RC_API const char* rc_profile_class_name(int32_t cls);
RC_API rc_status rc_profile_read(float* ms, int32_t* launches);

/* Tuning knobs (process-global).  RC_TUNE_GEMM_TILE: kernel / workgroup tile of the bf16 projection GEMM,
 * 0 = chosen per shape (default); register-staged tiles 1 = 128x256, 2 = 256x256, 3 = 128x128;
 * direct-to-LDS tiles 5 = 256x256 (with the K-split tail), 6 = 128x128, 7 = 256x192 (K-split tail). */
#define RC_TUNE_GEMM_TILE 1
/* RC_TUNE_ATTN_CHUNK_TILES: KV tiles (of 64 keys) per attention workgroup when a query tile's KV range is
 * split; 0 = chosen per shape (default), a value beyond the context length disables the split. */
#define RC_TUNE_ATTN_CHUNK_TILES 2
/* RC_TUNE_GEMM_XCD_REMAP: 1 (default) = GEMM workgroup ids are regrouped per XCD, 0 = launch order. */
#define RC_TUNE_GEMM_XCD_REMAP 3
/* RC_TUNE_GEMM_THIN_TILES: 1 (default) = a last row of 256-row GEMM tiles with at most 64 live rows is multiplied
 * by a tile body laid out for 64 rows, 0 = by the full tile body. */
#define RC_TUNE_GEMM_THIN_TILES 4
RC_API rc_status rc_tune_set(int32_t key, int32_t value);

/* Host-only self-check of the bf16 GEMM's launch schedule (no GPU needed): builds the grid the library would launch
 * for C[m][n] = A[m][k] W^T with direct-to-LDS tile `tile` (5, 6 or 7, see RC_TUNE_GEMM_TILE) on a device of n_cus
 * compute units, walks every workgroup id and counts violations of "every output tile is covered exactly once, by
 * one workgroup over the whole K range or by K parts that partition it in order".  swiglu != 0: the gate/up
 * epilogue (half as many output columns per tile); with_workspace != 0: the K-split tail is allowed.
 * *n_blocks (optional) receives the grid size.  Returns the number of violations, or -1 for bad arguments. */
RC_API int32_t rc_gemm_plan_check(int32_t m, int32_t n, int32_t k, int32_t swiglu, int32_t tile, int32_t n_cus,
                                  int32_t with_workspace, int32_t* n_blocks);

/* ------------------------------------------------------------ machine ceilings
 * Two micro-benchmarks for the benchmark report (boards differ, and the chip lowers its clock under matrix load);
 * the caller times them with events on `stream`.
 * rc_ceiling_stream_copy: dst[0, bytes) = src[0, bytes) with 16-byte accesses (bytes a multiple of 16; device
 *   buffers, not overlapping): 2 * bytes of HBM traffic.
 * rc_ceiling_mfma_loop: n_workgroups workgroups of 8 wavefronts issue `iters` rounds of 32 back-to-back 16x16x32
 *   bf16 MFMAs on register operands; *flops receives the floating-point operations of the launch (host pointer).
 *   out: device scratch of rc_ceiling_mfma_loop_out_bytes(n_workgroups) bytes (keeps the loop observable). */
RC_API rc_status rc_ceiling_stream_copy(const void* src, void* dst, size_t bytes, void* stream);
RC_API size_t rc_ceiling_mfma_loop_out_bytes(int32_t n_workgroups);
RC_API rc_status rc_ceiling_mfma_loop(float* out, int32_t n_workgroups, int32_t iters, double* flops, void* stream);

/* ------------------------------------------------------------ stage calls
 * One kernel (family) each, for unit tests and for profiling a stage in isolation. */

/* Scratch the two stage calls below need (request table + rotary table), in bytes. */
RC_API size_t rc_stage_workspace_bytes(int32_t n_positions, int32_t head_dim);

/* Move n_tokens reused keys of one layer to their new positions and copy the values
 * (Figure "Overview", item 3, "re-applies RoPE").  Source rows src_offset..; destination rows
 * dst_offset.. (the new positions).  Pre-RoPE keys are rotated by the new position; rotated keys by
 * (dst_offset - old_start_pos).  src and dst must have equal n_kv_heads, head_dim, dtype.
 * workspace: device scratch of rc_stage_workspace_bytes(dst_offset + n_tokens, head_dim). */
RC_API rc_status rc_rope_rerotate(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset,
                           const rc_kv_layer* dst, int32_t dst_seq, int32_t dst_offset,
                           int32_t n_tokens, int32_t k_is_pre_rope, int32_t old_start_pos,
                           float rope_base, void* workspace, size_t workspace_bytes, void* stream);

/* rc_rope_rerotate for callers that cannot allocate or hand over device scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results, but the stage's scratch (request table, rotary table) is a fixed device array
 * inside the library: rc_rope_rerotate_static_scratch_bytes() bytes (about 16 MiB) that every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing.
 *   limit   dst_offset + n_tokens <= RC_REROTATE_STATIC_MAX_POSITIONS, else RC_E_CAPACITY (nothing is
 *           launched).
 *   sharing all calls on one GPU use that GPU's one array: calls that overlap in time on the same GPU
 *           (different streams or threads) race; serialise them.  The array keeps the last call's tables;
 *           nothing in it has to start at zero, every table entry a call reads it has written itself.
 * Other errors as rc_rope_rerotate; RC_E_HIP if the array's address cannot be obtained. */
#define RC_REROTATE_STATIC_MAX_POSITIONS 32768
RC_API size_t rc_rope_rerotate_static_scratch_bytes(void);
RC_API rc_status rc_rope_rerotate_static(const rc_kv_layer* src, int32_t src_seq, int32_t src_offset,
                                  const rc_kv_layer* dst, int32_t dst_seq, int32_t dst_offset,
                                  int32_t n_tokens, int32_t k_is_pre_rope, int32_t old_start_pos,
                                  float rope_base, void* stream);

/* Eq. (1): score[j] = 1 - mean_h cos(cache V row (offset + j, h), v_fresh[j][h]); H = KV heads;
 * cos = dot / max(|a||b|, 1e-12).  Accumulated in float; above the floor 1 - cos is evaluated in the
 * equivalent cancellation-free form 0.5 |a/|a| - b/|b||^2.  v_fresh [n_tokens][Hkv][dh] of T.
 * workspace: device scratch of rc_stage_workspace_bytes(0, head_dim). */
RC_API rc_status rc_vdev_score(const void* v_fresh, const rc_kv_layer* cache, int32_t seq, int32_t offset,
                        int32_t n_tokens, float* score, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Budget selection: a fixed recompute budget of k tokens in place of the paper's thresholds (Eq. 5), the way its
 * budgeted comparison system is configured (Appendix "Baseline Descriptions": a fixed recompute ratio, rounded
 * down): indices of the k largest of score[0..n), equal scores to the lower index, written ascending to
 * idx_out[k].  n <= 2^20.  NaN scores order above +inf. */
RC_API rc_status rc_topk(const float* score, int32_t n, int32_t k, int32_t* idx_out, void* stream);

/* Threshold selection (Eq. 5 / Eq. 7): idx_out receives, ascending, every j with
 * score[j] >= tau * mean(score); *count_out (device int32) their number.  idx_out holds n entries. */
RC_API rc_status rc_threshold_select(const float* score, int32_t n, float tau, int32_t* idx_out,
                              int32_t* count_out, void* stream);

/* The complete selector, Eq. (5)-(10): idx_out receives, ascending, every j with
 * s_dev[j] >= tau_dev * mean(s_dev), or s_inf[j] >= tau_inf * mean(s_inf) (s_inf may be NULL: no such
 * term), or j >= n - k_suf; *count_out (device int32) their number.  idx_out holds n entries.
 * Means and comparisons are taken in double on the given float scores. */
RC_API rc_status rc_final_select(const float* s_dev, const float* s_inf, int32_t n, float tau_dev, float tau_inf,
                          int32_t k_suf, int32_t* idx_out, int32_t* count_out, void* stream);

/* Causal grouped-query attention of n arbitrary query rows over one layer of a cache
 * (sparse rectification, Section 4.2): row i (already rotated, at position q_pos[i], ascending)
 * attends over cache rows 0..q_pos[i] of `seq`.  q, out: [n][Hq][dh] of T.
 * workspace (optional, device, 256-byte aligned, rc_sparse_attention_workspace_bytes): lets the bf16
 * kernel cut long KV ranges into chunks when there are few query rows; NULL runs every query tile
 * in one workgroup. */
RC_API size_t rc_sparse_attention_workspace_bytes(int32_t n, int32_t n_q_heads, const rc_kv_layer* cache);
RC_API rc_status rc_sparse_attention(const void* q, const int32_t* q_pos, int32_t n, int32_t n_q_heads,
                                     const rc_kv_layer* cache, int32_t seq, void* out, void* workspace,
                                     size_t workspace_bytes, void* stream);

/* C[M][N] (float) = A[M][K] (T) * W[N][K]^T (T): the gathered-row projection GEMM.
 * workspace (optional, device, 256-byte aligned, rc_gemm_workspace_bytes()): lets the bf16 kernel cut the
 * last, partial round of output tiles along K (results are summed in a fixed order); NULL: one workgroup
 * per output tile. */
RC_API size_t rc_gemm_workspace_bytes(void);
RC_API rc_status rc_gemm_rows(int32_t dtype, const void* a, const void* w, float* c, int32_t m, int32_t n,
                              int32_t k, void* workspace, size_t workspace_bytes, void* stream);

/* The same GEMM with the epilogues the decoder layer applies in place (the layer function whose outputs
 * Eq. (1) compares: attention and SwiGLU MLP sub-blocks with residual connections):
 *   RC_GEMM_STORE   c (float [M][N])  = A W^T
 *   RC_GEMM_STORE_T c (T [M][N])      = A W^T                          (fresh value rows)
 *   RC_GEMM_ADD     c (float [M][N]) += A W^T                          (residual add of the o and down projections)
 *   RC_GEMM_SWIGLU  c (T [M][N])      = silu(A W^T) * (A W2^T)         (gate and up projections in one pass)
 * w2 [N][K] of T is read by RC_GEMM_SWIGLU only (NULL otherwise).  Other arguments as for rc_gemm_rows. */
typedef enum { RC_GEMM_STORE = 0, RC_GEMM_STORE_T = 1, RC_GEMM_ADD = 2, RC_GEMM_SWIGLU = 3 } rc_gemm_epilogue;
RC_API rc_status rc_gemm_rows_fused(int32_t dtype, int32_t epilogue, const void* a, const void* w, const void* w2,
                                    void* c, int32_t m, int32_t n, int32_t k, void* workspace,
                                    size_t workspace_bytes, void* stream);

/* The step of the hot path between the q|k|v projection and attention, on its own (the kernel rc_reuse runs in
 * every layer; Figure "Overview", item 3: recomputed rows are written back into the cache): qkv [n][Hq*dh | Hkv*dh |
 * Hkv*dh] float holds the projections of n live rows at positions pos[i] (device int32, each below the capacity of
 * `seq`); queries and keys are rotated to their positions (pairs (i, i + dh/2), angle pos * base^(-2i/dh)), the
 * rotated queries go to q_out [n][Hq][dh] of T, rotated keys and the values into the cache rows pos[i] of `seq`.
 * workspace: device scratch of rc_rope_scatter_workspace_bytes(n, dst) (request table and the rotary table of the
 * whole sequence capacity, at most 2^24 positions, else RC_E_CAPACITY). */
RC_API size_t rc_rope_scatter_workspace_bytes(int32_t n, const rc_kv_layer* dst);
RC_API rc_status rc_rope_scatter(const float* qkv, const int32_t* pos, int32_t n, int32_t n_q_heads, float rope_base,
                          const rc_kv_layer* dst, int32_t seq, void* q_out, void* workspace,
                          size_t workspace_bytes, void* stream);

/* Write n recomputed rows into one layer of a paged cache: k_rows/v_rows [n][Hkv][dh] of T go to
 * positions pos[i] of `seq` (keys as given, i.e. already rotated). */
RC_API rc_status rc_scatter_paged(const void* k_rows, const void* v_rows, const int32_t* pos, int32_t n,
                           const rc_kv_layer* dst, int32_t seq, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RELAYCACHE_H */
