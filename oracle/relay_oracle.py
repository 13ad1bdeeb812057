"""CPU oracle for the selective-recompute prefill of RelayCaching.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
HIP library must compute.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does, and this module
imports nothing from the product.

Everything is numpy float64, one step after another in the paper's order, with
no blocking, fusion or reordering.  `numpy.matmul` and `numpy.lexsort` are the
only library primitives used as steps.

What follows the paper, and where:
  * deviation score            -- Section 4.2, Eq. (1)
  * layer-wise similarity      -- Section 4.2, Eq. (2)
  * layer roles (reuse / dense detect / sparse rectify) -- Section 4.2, the
    paragraph after Eq. (4); Figure "Overview of RelayCaching", item (3)
  * pre-RoPE key storage, hidden states cached at L_start -- Figure "Overview
    of RelayCaching", item (2); Section 4.2 "Start layer"
  * budget selection top floor(budget*S) -- the floor convention of the
    CacheBlend setting in Appendix "Baseline Descriptions"
  * threshold / influence / suffix selection -- Section 4.3, Eq. (5)-(10)
  * decoding step with un-rotated keys, captured hidden state and influence
    accumulation -- Figure "Overview of RelayCaching", item (2); Eq. (6)
  * layer-range profiler (start / end / detection layer) -- Section 4.2,
    Eq. (2)-(4); Appendix table "Hyperparameters for Critical Layer Selection"
  * prompts with several reused segments (relay chains) -- Appendix "Agent
    Configuration" (cumulative context chain); each segment scored and selected
    on its own
  * FULL and ZERO baselines    -- Appendix "Baseline Descriptions"
  * reuse rate                 -- Section 5.1 "Metrics"

The paper runs stock decoder models and does not restate their arithmetic; the
decoder layer here is the usual pre-norm one (RMSNorm, rotary GQA attention,
SwiGLU), with the rotate-half rotary convention.

Readings taken where the paper is silent (all restated in the design notes):
  * H in Eq. (1) counts KV heads (value vectors exist per KV head).
  * cos(a, b) = a.b / max(|a||b|, 1e-12).
  * The layer triple is 0-based; h_start is the input of layer l_start; layers
    [l_start, l_det) are dense, [l_det, l_end] sparse, both ends of the latter
    included.
  * New tokens (prefix, optional suffix) are active in every layer.
  * With no suffix, the last segment token is always active from l_start to
    the last layer: it carries the first-token logits.  It is not counted in k
    and not reported among the selected indices.
  * Selected rows write their fresh K/V into the cache before any row of that
    layer attends.
  * k = 0 skips the dense detect layers as well (pure reuse).
  * Influence (Eq. 6) sums over query heads and includes the new token's
    weight on itself.
  * Profiler: "deepest layer with s >= tau_st" is searched at or before the
    minimum-similarity layer; standard deviations are population ones; ranks
    of equal deviations are averaged; rho_l compares layers l-1 and l; the
    "min rise samples" hyper-parameter is listed but never used by the text.

    l* is the first layer whose second difference alpha is negative directly
    after a positive one, and l_det = l* + 1.

Pins: tests/test_oracle_pins.py.  No function here is unpinned, except that
nothing fixes the numeric values of scores on trained models (the paper prints
none): that part is "parity unpinned" by necessity; and the index base of
rho / alpha in the profiler's detection rule, which the rule's hand-worked
example fixes for this reading only: the table "Model-specific layer
configurations" lists detection layers 3 and 4, which this reading reaches
only through its l_start + 1 fallback ("parity unpinned").
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# model container
# --------------------------------------------------------------------------
@dataclass
class OracleModel:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float
    layers: List[dict]        # each: wq wk wv wo w_gate w_up w_down ([out][in]), g_attn g_ffn
    g_final: np.ndarray
    w_lm: np.ndarray          # [vocab][d]

    @staticmethod
    def from_shape(shape, weights: dict) -> "OracleModel":
        return OracleModel(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                           shape.head_dim, shape.d_ffn, shape.vocab, float(shape.rope_base),
                           float(shape.rms_eps), weights["layers"], weights["g_final"], weights["w_lm"])


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y = x W^T with W stored [out][in]; float64."""
    return np.matmul(np.asarray(x, F64), np.asarray(w, F64).T)


# --------------------------------------------------------------------------
# decoder-layer pieces
# --------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def rope_rotate(x: np.ndarray, angle_pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate vectors x[n][heads][head_dim] by the rotary angles of `angle_pos[n]`.

    Pair i couples elements (i, i + head_dim/2); its angle is pos * base^(-2i/head_dim).
    `angle_pos` may be negative or a difference of positions: rotations compose
    additively, which is what moving a key from an old to a new position uses.
    """
    x = np.asarray(x, F64)
    dh = x.shape[-1]
    half = dh // 2
    theta = np.asarray(base, F64) ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.asarray(angle_pos, F64)[:, None] * theta[None, :]          # [n][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def causal_gqa_attention(q: np.ndarray, q_pos: np.ndarray, k_cache: np.ndarray,
                         v_cache: np.ndarray) -> np.ndarray:
    """Attention of arbitrary query rows over a cache whose row index is the position.

    q[n][Hq][dh] at positions q_pos[n]; k_cache, v_cache [T][Hkv][dh].  Query
    head i reads KV head i // (Hq/Hkv).  A query at position p sees rows 0..p.
    Returns [n][Hq][dh].
    """
    n, hq, dh = q.shape
    t, hkv, _ = k_cache.shape
    g = hq // hkv
    visible = np.arange(t)[None, :] <= np.asarray(q_pos)[:, None]       # [n][T]
    out = np.empty((n, hq, dh), F64)
    for h in range(hq):
        kh, vh = k_cache[:, h // g, :], v_cache[:, h // g, :]
        s = np.matmul(q[:, h, :], kh.T) / np.sqrt(F64(dh))
        s = np.where(visible, s, -np.inf)
        s = s - np.max(s, axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=-1, keepdims=True)
        out[:, h, :] = np.matmul(p, vh)
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def decoder_layer(m: OracleModel, l: int, h: np.ndarray, pos: np.ndarray,
                  k_cache: np.ndarray, v_cache: np.ndarray, rope_shift: int = 0) -> np.ndarray:
    """One pre-norm decoder layer on the rows h[n][d] sitting at positions pos[n].

    The rows' fresh K (rotated to `pos`) and V are written into the layer's cache
    first; then every row attends over cache rows 0..its own position.
    k_cache / v_cache [T][Hkv][dh] are updated in place.  Returns the new h.
    `rope_shift` adds a constant to the rotary positions only (cache rows and the
    causal mask still use `pos`); it exists to state shift invariance in a test.
    """
    w = m.layers[l]
    n = h.shape[0]
    a = rmsnorm(h, w["g_attn"], m.rms_eps)
    q = linear(a, w["wq"]).reshape(n, m.n_q_heads, m.head_dim)
    k = linear(a, w["wk"]).reshape(n, m.n_kv_heads, m.head_dim)
    v = linear(a, w["wv"]).reshape(n, m.n_kv_heads, m.head_dim)
    q = rope_rotate(q, pos + rope_shift, m.rope_base)
    k = rope_rotate(k, pos + rope_shift, m.rope_base)
    k_cache[pos] = k
    v_cache[pos] = v
    o = causal_gqa_attention(q, pos, k_cache, v_cache).reshape(n, m.n_q_heads * m.head_dim)
    h = h + linear(o, w["wo"])
    f = rmsnorm(h, w["g_ffn"], m.rms_eps)
    h = h + linear(silu(linear(f, w["w_gate"])) * linear(f, w["w_up"]), w["w_down"])
    return h


def first_token_logits(m: OracleModel, h_last: np.ndarray) -> np.ndarray:
    return linear(rmsnorm(h_last, m.g_final, m.rms_eps), m.w_lm)


# --------------------------------------------------------------------------
# FULL baseline and the earlier agent's record
# --------------------------------------------------------------------------
@dataclass
class PrefillResult:
    k_cache: np.ndarray       # [L][T][Hkv][dh] keys rotated to their positions
    v_cache: np.ndarray       # [L][T][Hkv][dh]
    k_pre_rope: np.ndarray    # [L][T][Hkv][dh] keys before rotation
    h_in: np.ndarray          # [L+1][T][d]: h_in[l] enters layer l; h_in[L] leaves the last
    logits: np.ndarray        # [vocab] from the last position


def full_prefill(m: OracleModel, x: np.ndarray, pos0: int = 0) -> PrefillResult:
    """FULL baseline: every token of x[T][d] runs through every layer, causally.

    `pos0` shifts every rotary position by a constant (default 0)."""
    x = np.asarray(x, F64)
    t = x.shape[0]
    pos = np.arange(t)
    shape = (m.n_layers, t, m.n_kv_heads, m.head_dim)
    kc, vc, kpre = np.zeros(shape, F64), np.zeros(shape, F64), np.zeros(shape, F64)
    h_in = np.empty((m.n_layers + 1, t, m.d_model), F64)
    h = x
    for l in range(m.n_layers):
        h_in[l] = h
        a = rmsnorm(h, m.layers[l]["g_attn"], m.rms_eps)
        kpre[l][pos] = linear(a, m.layers[l]["wk"]).reshape(t, m.n_kv_heads, m.head_dim)
        h = decoder_layer(m, l, h, pos, kc[l], vc[l], rope_shift=pos0)
    h_in[m.n_layers] = h
    return PrefillResult(kc, vc, kpre, h_in, first_token_logits(m, h[-1]))


@dataclass
class SegmentRecord:
    """What the earlier agent's cache manager keeps for the shared segment."""
    k: np.ndarray             # [L][S][Hkv][dh]: pre-RoPE keys, or keys rotated at old positions
    v: np.ndarray             # [L][S][Hkv][dh]
    h_start: np.ndarray       # [S][d] hidden states entering layer l_start
    k_is_pre_rope: bool
    old_start_pos: int        # position of the segment's first token in the earlier run


def decode_record(m: OracleModel, x_alt: np.ndarray, x_seg: np.ndarray, l_start: int,
                  k_is_pre_rope: bool = True) -> SegmentRecord:
    """The segment record of an earlier agent that saw `x_alt` before the segment.

    Under causal attention the K/V and hidden state of a token depend only on
    the tokens before it, so token-by-token decoding and a prefill of
    [x_alt ; x_seg] give the same segment rows.
    """
    n_alt = x_alt.shape[0]
    r = full_prefill(m, np.concatenate([np.asarray(x_alt, F64), np.asarray(x_seg, F64)], axis=0))
    k = r.k_pre_rope if k_is_pre_rope else r.k_cache
    return SegmentRecord(k[:, n_alt:].copy(), r.v_cache[:, n_alt:].copy(),
                         r.h_in[l_start][n_alt:].copy(), k_is_pre_rope, n_alt)


def decode_step(m: OracleModel, x_new: np.ndarray, pos: int, k_cache: np.ndarray, v_cache: np.ndarray,
                k_pre_rope: Optional[np.ndarray] = None, capture_layer: int = -1,
                s_inf: Optional[np.ndarray] = None):
    """One decoding step of the earlier agent with the cache manager's bookkeeping
    (Figure "Overview", item 2; Eq. 6).

    The token x_new[d] sits at position `pos`; k_cache / v_cache [L][cap][Hkv][dh]
    already hold rows 0..pos-1 and receive row `pos`.  Optionally stores the key
    before rotation in k_pre_rope[l][pos], returns the hidden state entering
    `capture_layer`, and adds to s_inf[j], j = 0..pos, the attention weight this
    step's query puts on position j, summed over all layers and query heads
    (the token's weight on itself included).
    Returns (logits[vocab], h_captured[d] or None).
    """
    h = np.asarray(x_new, F64).reshape(1, m.d_model)
    g = m.n_q_heads // m.n_kv_heads
    captured = None
    for l in range(m.n_layers):
        w = m.layers[l]
        if l == capture_layer:
            captured = h[0].copy()
        a = rmsnorm(h, w["g_attn"], m.rms_eps)
        q = linear(a, w["wq"]).reshape(1, m.n_q_heads, m.head_dim)
        k = linear(a, w["wk"]).reshape(1, m.n_kv_heads, m.head_dim)
        v = linear(a, w["wv"]).reshape(1, m.n_kv_heads, m.head_dim)
        if k_pre_rope is not None:
            k_pre_rope[l][pos] = k[0]
        q = rope_rotate(q, np.array([pos]), m.rope_base)[0]
        k_cache[l][pos] = rope_rotate(k, np.array([pos]), m.rope_base)[0]
        v_cache[l][pos] = v[0]
        o = np.empty((m.n_q_heads, m.head_dim), F64)
        for i in range(m.n_q_heads):
            keys = k_cache[l][:pos + 1, i // g, :]
            sc = np.matmul(keys, q[i]) / np.sqrt(F64(m.head_dim))
            alpha = np.exp(sc - np.max(sc))
            alpha = alpha / np.sum(alpha)
            if s_inf is not None:
                s_inf[:pos + 1] += alpha
            o[i] = np.matmul(alpha, v_cache[l][:pos + 1, i // g, :])
        h = h + linear(o.reshape(1, -1), w["wo"])
        f = rmsnorm(h, w["g_ffn"], m.rms_eps)
        h = h + linear(silu(linear(f, w["w_gate"])) * linear(f, w["w_up"]), w["w_down"])
    return first_token_logits(m, h[0]), captured


# --------------------------------------------------------------------------
# scoring and selection
# --------------------------------------------------------------------------
def vdev_score(v_reuse: np.ndarray, v_full: np.ndarray) -> np.ndarray:
    """Eq. (1): d_j = 1 - (1/H) sum_h cos(v_reuse[j][h], v_full[j][h]); inputs [S][H][dh]."""
    a, b = np.asarray(v_reuse, F64), np.asarray(v_full, F64)
    dot = np.sum(a * b, axis=-1)
    na = np.sqrt(np.sum(a * a, axis=-1))
    nb = np.sqrt(np.sum(b * b, axis=-1))
    cos = dot / np.maximum(na * nb, 1e-12)
    return 1.0 - np.mean(cos, axis=-1)


def layer_similarity(d_jl: np.ndarray) -> np.ndarray:
    """Eq. (2): s_l = mean_j (1 - d_{j,l}); d_jl is [S][L]."""
    return np.mean(1.0 - np.asarray(d_jl, F64), axis=0)


def average_ranks(x: np.ndarray) -> np.ndarray:
    """Ranks 1..n of x, equal values sharing the mean of the ranks they occupy."""
    x = np.asarray(x, F64)
    order = np.argsort(x, kind="stable")
    ranks = np.empty(x.shape[0], F64)
    i = 0
    while i < x.shape[0]:
        j = i
        while j + 1 < x.shape[0] and x[order[j + 1]] == x[order[i]]:
            j += 1
        ranks[order[i:j + 1]] = 0.5 * (i + j) + 1.0
        i = j + 1
    return ranks


def spearman_adjacent(d_jl: np.ndarray) -> np.ndarray:
    """rho_l, l = 1..L-1: Spearman rank correlation of the token-wise deviations of layers l-1 and l
    (Section 4.2, "Detection layer"); rho_0 is set to 0 (undefined).  d_jl is [S][L].
    A layer whose deviations are all equal has no ranking: its correlations are 0."""
    d = np.asarray(d_jl, F64)
    n_layers = d.shape[1]
    ranks = np.stack([average_ranks(d[:, l]) for l in range(n_layers)], axis=1)
    rho = np.zeros(n_layers, F64)
    for l in range(1, n_layers):
        a = ranks[:, l - 1] - np.mean(ranks[:, l - 1])
        b = ranks[:, l] - np.mean(ranks[:, l])
        den = np.sqrt(np.sum(a * a) * np.sum(b * b))
        rho[l] = np.sum(a * b) / den if den > 0 else 0.0
    return rho


@dataclass
class LayerProfile:
    l_start: int
    l_det: int
    l_end: int
    s: np.ndarray        # Eq. (2) per layer
    rho: np.ndarray      # Spearman correlation of layers l-1 and l
    alpha: np.ndarray    # Eq. (4); 0 where undefined (l < 3)


def profile_layers(d_jl: np.ndarray, tau_st: float = 0.99, tail: int = 5, lam: float = 2.0,
                   consecutive: int = 2) -> LayerProfile:
    """The offline layer-range profiler (Section 4.2, Eq. 2-4) on deviations d_jl [S][L].

    Start: the deepest layer at or before l_min = argmin s with s >= tau_st (0 if none).
    End:   b = mean - std of s over the last `tail` layers; scanning l = l_min, l_min+1, ...: the
           first l whose next `consecutive` layers all have s >= b and |s_l' - s_{l'-1}| < lam * std
           (the last layer if no such l).
    Detection: alpha_l = rho_l - 2 rho_{l-1} + rho_{l-2} (l >= 3); l* = the first l with
           alpha_{l-1} > 0 and alpha_l < 0 for which l* + 1 lies in (l_start, l_end]; l_det = l* + 1
           (l_start + 1 if there is none).
    All indices are layer indices of the deviation matrix."""
    d = np.asarray(d_jl, F64)
    n_layers = d.shape[1]
    s = layer_similarity(d)
    l_min = int(np.argmin(s))
    l_start = 0
    for l in range(l_min + 1):
        if s[l] >= tau_st:
            l_start = l
    last = s[max(0, n_layers - tail):]
    mu, sigma = float(np.mean(last)), float(np.sqrt(np.mean((last - np.mean(last)) ** 2)))
    b = mu - sigma
    l_end = n_layers - 1
    for l in range(l_min, n_layers - consecutive):
        if all(s[l2] >= b and abs(s[l2] - s[l2 - 1]) < lam * sigma for l2 in range(l + 1, l + 1 + consecutive)):
            l_end = l
            break
    l_end = max(l_end, min(l_start + 1, n_layers - 1))
    rho = spearman_adjacent(d)
    alpha = np.zeros(n_layers, F64)
    for l in range(3, n_layers):
        alpha[l] = rho[l] - 2.0 * rho[l - 1] + rho[l - 2]
    l_det = min(l_start + 1, l_end)
    for l in range(4, n_layers):
        if alpha[l - 1] > 0.0 and alpha[l] < 0.0 and l_start < l + 1 <= l_end:
            l_det = l + 1
            break
    return LayerProfile(l_start, l_det, l_end, s, rho, alpha)


def topk_select(score: Sequence[float], k: int) -> np.ndarray:
    """Indices of the k largest scores, equal scores resolved to the lower index; ascending."""
    score = np.asarray(score)
    order = np.lexsort((np.arange(score.shape[0]), -score))      # by -score, then by index
    return np.sort(order[:k]).astype(np.int32)


def threshold_select(score: Sequence[float], tau: float) -> np.ndarray:
    """Eq. (5) / Eq. (7): {j : score_j >= tau * mean(score)}; ascending."""
    score = np.asarray(score, F64)
    return np.nonzero(score >= tau * np.mean(score))[0].astype(np.int32)


def final_selection(s_dev: Sequence[float], s_inf: Optional[Sequence[float]], tau_dev: float,
                    tau_inf: float, k_suf: int) -> np.ndarray:
    """Eq. (5)-(10): I_dev united with I_inf-score and the last k_suf tokens; ascending."""
    n = len(s_dev)
    chosen = set(threshold_select(s_dev, tau_dev).tolist())
    if s_inf is not None:
        chosen |= set(threshold_select(s_inf, tau_inf).tolist())
    chosen |= set(range(max(0, n - k_suf), n))
    return np.array(sorted(chosen), dtype=np.int32)


def reuse_rate(n_layers: int, n_seg: int, l_start: int, l_det: int, l_end: int, k: int) -> float:
    """Fraction of the segment's KV entries kept as they came from the earlier agent."""
    recomputed = (l_det - l_start) * n_seg + (l_end - l_det + 1) * k
    return 1.0 - recomputed / float(n_layers * n_seg)


# --------------------------------------------------------------------------
# the selective-recompute prefill
# --------------------------------------------------------------------------
@dataclass
class RelayResult:
    k_cache: np.ndarray       # [L][T][Hkv][dh], T = P + S + n_suffix
    v_cache: np.ndarray
    sel_idx: np.ndarray       # selected segment indices, ascending (int32)
    score: Optional[np.ndarray]   # [S] deviation at l_det (None when k = 0)
    logits: np.ndarray        # [vocab]
    active_rows: List[int]    # rows run in each layer (for accounting)


def relay_prefill(m: OracleModel, x_prefix: np.ndarray, seg: SegmentRecord, l_start: int,
                  l_det: int, l_end: int, k: int, x_suffix: Optional[np.ndarray] = None,
                  forced_idx: Optional[Sequence[int]] = None,
                  thresholds: Optional[Tuple[float, float, int]] = None,
                  s_inf: Optional[Sequence[float]] = None) -> RelayResult:
    """Prefill of [x_prefix ; segment ; x_suffix] that takes over the segment's KV.

    1. every layer: reused keys moved to positions P..P+S-1, values copied;
    2. new tokens (prefix, suffix) run through every layer;
    3. layers [l_start, l_det): all S segment tokens recomputed from seg.h_start;
    4. at l_det: fresh values of all S tokens -> Eq. (1) score -> top-k;
    5. layers [l_det, l_end]: only the selected tokens (and the logits-carrying
       last token when there is no suffix) are recomputed, their K/V rows written
       back before that layer's attention;
    6. layers > l_end: only new tokens (and that last token) continue.
    `forced_idx` replaces the top-k result (the score is still computed).
    `thresholds` = (tau_dev, tau_inf, k_suf) switches step 4 from the fixed budget to the
    selector of Eq. (5)-(10), with the influence scores `s_inf` of Eq. (6) if given; `k` is
    then ignored and the dense layers always run.
    """
    assert 0 <= l_start < l_det <= l_end < m.n_layers
    x_prefix = np.asarray(x_prefix, F64)
    p, s = x_prefix.shape[0], seg.v.shape[1]
    n_suf = 0 if x_suffix is None else x_suffix.shape[0]
    t = p + s + n_suf
    assert 0 <= k <= s
    dense = k > 0 if thresholds is None else s > 0
    shape = (m.n_layers, t, m.n_kv_heads, m.head_dim)
    kc, vc = np.zeros(shape, F64), np.zeros(shape, F64)

    # 1. take over the segment: keys re-rotated to the new positions, values as they are
    seg_pos = p + np.arange(s)
    for l in range(m.n_layers):
        if seg.k_is_pre_rope:
            kc[l][seg_pos] = rope_rotate(seg.k[l], seg_pos, m.rope_base)
        else:
            old_pos = seg.old_start_pos + np.arange(s)
            kc[l][seg_pos] = rope_rotate(seg.k[l], seg_pos - old_pos, m.rope_base)
        vc[l][seg_pos] = np.asarray(seg.v[l], F64)

    h_pre = x_prefix
    pos_pre = np.arange(p)
    h_suf = np.zeros((0, m.d_model), F64) if n_suf == 0 else np.asarray(x_suffix, F64)
    pos_suf = p + s + np.arange(n_suf)
    carries_logits = n_suf == 0           # last segment token stands in for a suffix

    seg_rows = np.zeros(0, dtype=np.int64)        # segment indices active in the current layer
    h_seg = np.zeros((0, m.d_model), F64)
    score = None
    sel = np.zeros(0, dtype=np.int32)
    active_rows = []

    for l in range(m.n_layers):
        if l == l_start:
            if dense:
                seg_rows = np.arange(s)
                h_seg = np.asarray(seg.h_start, F64).copy()
            elif carries_logits:
                seg_rows = np.array([s - 1])
                h_seg = np.asarray(seg.h_start, F64)[s - 1:s].copy()
        if l == l_det and dense:
            w = m.layers[l]
            v_fresh = linear(rmsnorm(h_seg, w["g_attn"], m.rms_eps), w["wv"])
            v_fresh = v_fresh.reshape(s, m.n_kv_heads, m.head_dim)
            score = vdev_score(vc[l][seg_pos], v_fresh)
            if thresholds is not None:
                sel = final_selection(score, s_inf, thresholds[0], thresholds[1], thresholds[2])
            elif forced_idx is not None:
                sel = np.sort(np.asarray(forced_idx, np.int32))
            else:
                sel = topk_select(score, k)
            keep = set(sel.tolist())
            if carries_logits:
                keep.add(s - 1)
            keep = np.array(sorted(keep), dtype=np.int64)
            h_seg, seg_rows = h_seg[keep], keep
        if l == l_end + 1:
            if carries_logits:
                h_seg, seg_rows = h_seg[-1:], seg_rows[-1:]       # s-1 is the largest index
            else:
                h_seg, seg_rows = h_seg[:0], seg_rows[:0]

        h_all = np.concatenate([h_pre, h_seg, h_suf], axis=0)
        pos_all = np.concatenate([pos_pre, p + seg_rows, pos_suf]).astype(np.int64)
        active_rows.append(int(h_all.shape[0]))
        h_all = decoder_layer(m, l, h_all, pos_all, kc[l], vc[l])
        n_seg_rows = seg_rows.shape[0]
        h_pre = h_all[:p]
        h_seg = h_all[p:p + n_seg_rows]
        h_suf = h_all[p + n_seg_rows:]

    h_last = h_suf[-1] if n_suf > 0 else h_seg[-1]
    return RelayResult(kc, vc, sel, score, first_token_logits(m, h_last), active_rows)


# --------------------------------------------------------------------------
# several reused segments in one prompt (relay chains)
# --------------------------------------------------------------------------
@dataclass
class MultiRelayResult:
    k_cache: np.ndarray            # [L][T][Hkv][dh]
    v_cache: np.ndarray
    sel_idx: List[np.ndarray]      # per segment, ascending, relative to the segment
    score: List[Optional[np.ndarray]]
    logits: np.ndarray
    active_rows: List[int]


def relay_prefill_multi(m: OracleModel, pieces: Sequence[tuple], l_start: int, l_det: int,
                        l_end: int) -> MultiRelayResult:
    """Prefill of a prompt made of new text and several reused segments, in one pass over the layers.

    pieces: ("new", x[n][d]) or ("seg", SegmentRecord, k) in prompt order; every segment has its own
    record (own old position), its own Eq. (1) scores at l_det and its own top-k.  The steps per layer
    are those of relay_prefill with "the segment" read as "every segment": all new tokens are live in
    every layer; a segment with k > 0 has all tokens live in [l_start, l_det) and its selected tokens
    in [l_det, l_end]; if the prompt ends with a segment, that segment's last token is live from
    l_start to the last layer and yields the logits.
    """
    assert 0 <= l_start < l_det <= l_end < m.n_layers
    spans = []                                  # (kind, first position, length, payload...)
    t = 0
    for pc in pieces:
        n = pc[1].shape[0] if pc[0] == "new" else pc[1].v.shape[1]
        spans.append((pc, t, n))
        t += n
    shape = (m.n_layers, t, m.n_kv_heads, m.head_dim)
    kc, vc = np.zeros(shape, F64), np.zeros(shape, F64)
    segs = [(pc[1], p0, n, pc[2]) for pc, p0, n in spans if pc[0] == "seg"]
    for rec, p0, n, _ in segs:
        new_pos = p0 + np.arange(n)
        for l in range(m.n_layers):
            if rec.k_is_pre_rope:
                kc[l][new_pos] = rope_rotate(rec.k[l], new_pos, m.rope_base)
            else:
                kc[l][new_pos] = rope_rotate(rec.k[l], new_pos - (rec.old_start_pos + np.arange(n)), m.rope_base)
            vc[l][new_pos] = np.asarray(rec.v[l], F64)
    ends_with_seg = len(spans) > 0 and spans[-1][0][0] == "seg"
    hidden = {}                                  # position -> hidden state of the rows that are live
    for pc, p0, n in spans:
        if pc[0] == "new":
            for i in range(n):
                hidden[p0 + i] = np.asarray(pc[1][i], F64)
    sel = [np.zeros(0, np.int32) for _ in segs]
    score: List[Optional[np.ndarray]] = [None for _ in segs]
    active_rows = []
    last_pos = t - 1
    for l in range(m.n_layers):
        if l == l_start:
            for si, (rec, p0, n, k) in enumerate(segs):
                if k > 0:
                    for j in range(n):
                        hidden[p0 + j] = np.asarray(rec.h_start[j], F64)
                elif ends_with_seg and si == len(segs) - 1:
                    hidden[p0 + n - 1] = np.asarray(rec.h_start[n - 1], F64)
        if l == l_det:
            w = m.layers[l]
            for si, (rec, p0, n, k) in enumerate(segs):
                if k <= 0:
                    continue
                h_seg = np.stack([hidden[p0 + j] for j in range(n)])
                v_fresh = linear(rmsnorm(h_seg, w["g_attn"], m.rms_eps), w["wv"]).reshape(n, m.n_kv_heads, m.head_dim)
                score[si] = vdev_score(vc[l][p0:p0 + n], v_fresh)
                sel[si] = topk_select(score[si], k)
                keep = set(sel[si].tolist())
                if ends_with_seg and si == len(segs) - 1:
                    keep.add(n - 1)
                for j in range(n):
                    if j not in keep:
                        del hidden[p0 + j]
        if l == l_end + 1:
            for si, (rec, p0, n, k) in enumerate(segs):
                for j in range(n):
                    if p0 + j in hidden and not (ends_with_seg and p0 + j == last_pos):
                        del hidden[p0 + j]
        pos = np.array(sorted(hidden), dtype=np.int64)
        h_all = np.stack([hidden[p] for p in pos])
        active_rows.append(int(pos.shape[0]))
        h_all = decoder_layer(m, l, h_all, pos, kc[l], vc[l])
        hidden = {int(p): h_all[i] for i, p in enumerate(pos)}
    return MultiRelayResult(kc, vc, sel, score, first_token_logits(m, hidden[last_pos]), active_rows)
