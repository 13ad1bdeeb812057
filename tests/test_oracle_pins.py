"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each test names the passage it leans on.  Expected values never come from the
HIP path: they are closed forms, paper-printed figures (tests/golden/), a scalar
token-at-a-time reference (tests/brute_force.py), or invariants of the method.
"""
import math
import os

import numpy as np
import pytest

from oracle import relay_oracle as R
from synth import ModelShape, Workload, make_hidden, make_weights
from tests import brute_force as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def _tiny(n_layers=3, d=16, hq=4, hkv=2, dh=4, f=24, vocab=20, name="pin", std=0.35):
    shape = ModelShape(n_layers, d, hq, hkv, dh, f, vocab, 10000.0, dtype="f32")
    w = Workload(name, shape, 0, 0, 0, 0, 1, 1, 20)
    # a larger weight scale than the benchmark's makes attention and the FFN matter at d=16
    return w, R.OracleModel.from_shape(shape, make_weights(w, std=std))


# ----------------------------------------------------------------------------
# Eq. (1): closed forms
# ----------------------------------------------------------------------------
def test_score_closed_forms():
    rng = np.random.default_rng(1)
    H, dh = 4, 8
    v = rng.standard_normal((5, H, dh))
    assert np.allclose(R.vdev_score(v * 3.7, v), 0.0, atol=1e-14)          # positive scaling: cos = 1
    assert np.allclose(R.vdev_score(-v, v), 2.0, atol=1e-14)               # negation: cos = -1
    flipped = v.copy()
    flipped[:, 1] *= -1.0                                                  # one of H heads flipped
    assert np.allclose(R.vdev_score(flipped, v), 2.0 / H, atol=1e-14)
    a = np.zeros((1, 2, 4)); b = np.zeros((1, 2, 4))
    a[0, :, 0] = 1.0; b[0, :, 1] = 2.0                                     # orthogonal: cos = 0
    assert np.allclose(R.vdev_score(a, b), 1.0)
    # a 3-4-5 angle in one head, aligned in the other: 1 - (0.6 + 1)/2
    a = np.array([[[1.0, 0.0], [1.0, 1.0]]]); b = np.array([[[3.0, 4.0], [2.0, 2.0]]])
    assert np.allclose(R.vdev_score(a, b), 1.0 - 0.8)
    # zero vector: cos defined as 0 through the floor on the denominator
    z = np.zeros((1, 1, 4))
    assert np.allclose(R.vdev_score(z, np.ones((1, 1, 4))), 1.0)
    # not symmetric-in-heads mistakes: mean over heads, not over elements
    a = np.zeros((1, 2, 2)); b = np.zeros((1, 2, 2))
    a[0, 0] = [1, 0]; b[0, 0] = [100, 0]; a[0, 1] = [1, 0]; b[0, 1] = [0, 1e-3]
    assert np.allclose(R.vdev_score(a, b), 0.5)


def test_layer_similarity_eq2():
    d = np.array([[0.0, 0.5], [0.2, 0.1], [0.4, 0.0]])
    assert np.allclose(R.layer_similarity(d), [0.8, 0.8])


# ----------------------------------------------------------------------------
# selection: budget top-k (tie rule), Eq. (5)-(10)
# ----------------------------------------------------------------------------
def test_topk_against_sorted_and_ties():
    rng = np.random.default_rng(2)
    for n in (1, 2, 7, 64, 257):
        s = rng.integers(0, 6, size=n).astype(np.float64)       # many ties
        for k in (0, 1, n // 3, n):
            want = sorted(sorted(range(n), key=lambda j: (-s[j], j))[:k])
            assert R.topk_select(s, k).tolist() == want
    assert R.topk_select([1.0, 3.0, 3.0, 3.0, 0.0], 2).tolist() == [1, 2]    # lower index wins
    assert R.topk_select([5.0, 1.0, 9.0], 2).tolist() == [0, 2]              # ascending output
    assert R.topk_select([5.0, 1.0, 9.0], 0).tolist() == []
    assert R.topk_select([0.0, -0.0, 0.0], 2).tolist() == [0, 1]             # -0 == +0


def test_threshold_and_union_selectors():
    g = _golden("paper_selector_defaults.txt")
    s_dev = [1.0, 1.0, 1.0, 5.0]                      # mean 2, 1.5 * mean = 3
    assert R.threshold_select(s_dev, g["tau_dev"]).tolist() == [3]
    assert R.threshold_select([2.0, 2.0], 1.0).tolist() == [0, 1]            # >= is inclusive
    n = 30
    s_dev = np.ones(n); s_dev[4] = 10.0
    s_inf = np.ones(n); s_inf[7] = 10.0
    got = R.final_selection(s_dev, s_inf, g["tau_dev"], g["tau_inf"], int(g["k_suf"]))
    assert got.tolist() == [4, 7] + list(range(20, 30))
    assert R.final_selection(s_dev, None, 1.5, 1.45, 0).tolist() == [4]


# ----------------------------------------------------------------------------
# reuse rate: the paper's ablation figure pins the layer-range convention
# ----------------------------------------------------------------------------
def test_reuse_rate_matches_paper_ablation():
    g = _golden("paper_reuse_rate.txt")
    L = int(g["n_layers"])
    # the paper's triple indexes hidden states; as 0-based layers with l_end included it is (a, c, b-1)
    l_start, l_det, l_end = int(g["paper_l_start"]), int(g["paper_l_det"]), int(g["paper_l_end"]) - 1
    S = 1000
    dense = R.reuse_rate(L, S, l_start, l_det, l_end, k=S)
    assert round(100 * dense, 2) == g["dense_range_reuse_pct"]              # 15/32 = 46.875 -> 46.88
    # the full method's 85.35 % then implies a selected fraction between 15 % and 20 %
    f = (L * (1 - g["full_method_reuse_pct"] / 100) - (l_det - l_start)) / (l_end - l_det + 1)
    assert 0.15 < f < 0.20
    assert R.reuse_rate(L, S, 7, 8, 24, 0) == 1.0 - 1.0 / 32
    assert abs(R.reuse_rate(32, 4096, 7, 8, 24, 614) - (1 - (4096 + 17 * 614) / (32 * 4096))) < 1e-15


# ----------------------------------------------------------------------------
# rotary algebra
# ----------------------------------------------------------------------------
def test_rope_algebra():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 3, 16))
    a = np.array([0, 1, 5, 17, 300, 4095])
    b = np.array([3, 0, 9, -17, 11, -4000])
    base = 10000.0
    assert np.allclose(R.rope_rotate(R.rope_rotate(x, a, base), b, base), R.rope_rotate(x, a + b, base), atol=1e-12)
    assert np.allclose(np.linalg.norm(R.rope_rotate(x, a, base), axis=-1), np.linalg.norm(x, axis=-1))
    assert np.array_equal(R.rope_rotate(x, np.zeros(6), base), x)
    # complex-number statement of the same rotation: (x_i + i x_{i+half}) * exp(i pos theta_i)
    half = 8
    theta = base ** (-2.0 * np.arange(half) / 16)
    z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * a[:, None, None] * theta[None, None, :])
    assert np.allclose(R.rope_rotate(x, a, base), np.concatenate([z.real, z.imag], -1), atol=1e-12)
    # first pair rotates by exactly pos radians; the dot product of rotated q, k depends on pos difference only
    q = rng.standard_normal((1, 1, 16)); k = rng.standard_normal((1, 1, 16))
    d1 = np.sum(R.rope_rotate(q, [10], base) * R.rope_rotate(k, [4], base))
    d2 = np.sum(R.rope_rotate(q, [1006], base) * R.rope_rotate(k, [1000], base))
    assert abs(d1 - d2) < 1e-9
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    r = R.rope_rotate(e, [0.5], base)
    assert np.allclose([r[0, 0, 0], r[0, 0, 8]], [math.cos(0.5), math.sin(0.5)])


# ----------------------------------------------------------------------------
# attention special cases
# ----------------------------------------------------------------------------
def test_attention_special_cases():
    rng = np.random.default_rng(4)
    T, hkv, g, dh = 9, 2, 3, 8
    K = rng.standard_normal((T, hkv, dh)); V = rng.standard_normal((T, hkv, dh))
    q = rng.standard_normal((4, hkv * g, dh))
    pos = np.array([0, 3, 3, 8])
    out = R.causal_gqa_attention(q, pos, K, V)
    # a query at position 0 sees one key: output is that value, for every head of the group
    for h in range(hkv * g):
        assert np.allclose(out[0, h], V[0, h // g])
    # textbook softmax attention written with scalar loops
    for n in range(4):
        for h in range(hkv * g):
            sc = [float(q[n, h] @ K[t, h // g]) / math.sqrt(dh) for t in range(pos[n] + 1)]
            mx = max(sc); e = [math.exp(s - mx) for s in sc]; z = sum(e)
            want = sum(e[t] / z * V[t, h // g] for t in range(pos[n] + 1))
            assert np.allclose(out[n, h], want, atol=1e-12)
    # grouped-query attention equals multi-head attention over KV heads repeated g times
    Kr, Vr = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)
    assert np.allclose(R.causal_gqa_attention(q, pos, Kr, Vr), out, atol=1e-13)
    # rows after the query position never matter
    K2, V2 = K.copy(), V.copy()
    K2[4:] += 7.0; V2[4:] -= 3.0
    assert np.allclose(R.causal_gqa_attention(q[:3], pos[:3], K2, V2), out[:3], atol=1e-13)
    # large logits do not overflow
    big = R.causal_gqa_attention(q * 1e4, pos, K, V)
    assert np.all(np.isfinite(big))


# ----------------------------------------------------------------------------
# brute force on tiny inputs (token-at-a-time scalar reference)
# ----------------------------------------------------------------------------
def _nested(a):
    return np.asarray(a).tolist()


def _cache_from_dicts(dicts, T, hkv, dh):
    out = np.zeros((len(dicts), T, hkv, dh))
    for l, dct in enumerate(dicts):
        for t, rows in dct.items():
            out[l, t] = np.asarray(rows)
    return out


def test_full_prefill_equals_token_by_token():
    w, m = _tiny()
    x = make_hidden(w, "x", 11).astype(np.float64)
    r = R.full_prefill(m, x)
    tm = B.TinyModel(m)
    kc, vc, h_in, logits = B.brute_full_prefill(tm, _nested(x))
    assert np.allclose(r.k_cache, _cache_from_dicts(kc, 11, 2, 4), atol=1e-11)
    assert np.allclose(r.v_cache, _cache_from_dicts(vc, 11, 2, 4), atol=1e-11)
    assert np.allclose(r.h_in, np.asarray(h_in), atol=1e-11)
    assert np.allclose(r.logits, logits, atol=1e-11)
    # and the model is not degenerate: attention and FFN move the hidden state
    assert np.max(np.abs(r.h_in[-1] - r.h_in[0])) > 0.05


@pytest.mark.parametrize("triple,k", [((0, 1, 2), 3), ((1, 2, 2), 5), ((0, 2, 3), 0), ((0, 1, 1), 14)])
def test_relay_equals_scalar_reference(triple, k):
    w, m = _tiny(n_layers=4, name="pin4")
    P, S, A = 6, 14, 4
    xp = make_hidden(w, "xp", P).astype(np.float64)
    xa = make_hidden(w, "xa", A).astype(np.float64)
    xs = make_hidden(w, "xs", S).astype(np.float64)
    seg = R.decode_record(m, xa, xs, triple[0])
    got = R.relay_prefill(m, xp, seg, *triple, k)
    tm = B.TinyModel(m)
    kc, vc, sel, score, logits = B.brute_relay(tm, _nested(xp), _nested(seg.k), _nested(seg.v),
                                               _nested(seg.h_start), *triple, k)
    assert got.sel_idx.tolist() == sel
    if k > 0:
        assert np.allclose(got.score, score, atol=1e-12)
        assert np.max(got.score) > 1e-4          # different prefixes do produce deviation
    assert np.allclose(got.k_cache, _cache_from_dicts(kc, P + S, 2, 4), atol=1e-10)
    assert np.allclose(got.v_cache, _cache_from_dicts(vc, P + S, 2, 4), atol=1e-10)
    assert np.allclose(got.logits, logits, atol=1e-10)


# ----------------------------------------------------------------------------
# invariants of the method
# ----------------------------------------------------------------------------
def _setup(n_layers=4, P=9, S=17, A=5, l_start=0, same_prefix=False, pre_rope=True, name="inv"):
    w, m = _tiny(n_layers=n_layers, d=32, hq=4, hkv=2, dh=8, f=40, name=name, std=0.25)
    xp = make_hidden(w, "xp", P).astype(np.float64)
    xa = xp if same_prefix else make_hidden(w, "xa", A).astype(np.float64)
    xs = make_hidden(w, "xs", S).astype(np.float64)
    seg = R.decode_record(m, xa, xs, l_start, k_is_pre_rope=pre_rope)
    full = R.full_prefill(m, np.concatenate([xp, xs]))
    return m, xp, xs, seg, full


def test_full_budget_reproduces_full_prefill():
    """FULL baseline: budget 100 % over all layers, from the token inputs themselves."""
    m, xp, xs, seg, full = _setup()
    seg.h_start = xs.copy()                      # l_start = 0: the hidden state entering layer 0 is the input
    S = xs.shape[0]
    got = R.relay_prefill(m, xp, seg, 0, 1, m.n_layers - 1, S)
    assert np.allclose(got.k_cache, full.k_cache, atol=1e-10)
    assert np.allclose(got.v_cache, full.v_cache, atol=1e-10)
    assert np.allclose(got.logits, full.logits, atol=1e-10)
    assert got.sel_idx.tolist() == list(range(S))
    assert got.active_rows == [9 + 17] * m.n_layers


@pytest.mark.parametrize("l_start,l_det,l_end", [(1, 2, 3), (1, 3, 3), (2, 3, 3)])
def test_full_budget_with_true_hidden_states(l_start, l_det, l_end):
    """With h_start taken from the full-prefill run itself, the recomputed layers equal it exactly."""
    m, xp, xs, seg, full = _setup(l_start=l_start)
    P, S = xp.shape[0], xs.shape[0]
    seg.h_start = full.h_in[l_start][P:].copy()
    got = R.relay_prefill(m, xp, seg, l_start, l_det, l_end, S)
    for l in range(l_start, l_end + 1):
        assert np.allclose(got.k_cache[l], full.k_cache[l], atol=1e-10)
        assert np.allclose(got.v_cache[l], full.v_cache[l], atol=1e-10)
    # layers before l_start keep what the earlier agent wrote (different prefix => different values)
    assert not np.allclose(got.v_cache[l_start - 1][P:], full.v_cache[l_start - 1][P:], atol=1e-6) or l_start == 1
    # layer 0's V of a token does not depend on its prefix at all
    assert np.allclose(got.v_cache[0], full.v_cache[0], atol=1e-12)


@pytest.mark.parametrize("pre_rope", [True, False])
def test_zero_budget_is_pure_reuse(pre_rope):
    """ZERO baseline: nothing rectified; segment rows are the rotated record, bit for bit."""
    m, xp, xs, seg, full = _setup(pre_rope=pre_rope, A=5)
    P, S = xp.shape[0], xs.shape[0]
    suffix = np.random.default_rng(7).standard_normal((2, m.d_model))
    got = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, x_suffix=suffix)
    new_pos = P + np.arange(S)
    for l in range(m.n_layers):
        if pre_rope:
            want_k = R.rope_rotate(seg.k[l], new_pos, m.rope_base)
        else:
            want_k = R.rope_rotate(seg.k[l], np.full(S, P - 5), m.rope_base)
        assert np.array_equal(got.k_cache[l][P:P + S], want_k)
        assert np.array_equal(got.v_cache[l][P:P + S], seg.v[l])
    assert got.sel_idx.size == 0 and got.score is None
    assert got.active_rows == [P + 2] * m.n_layers
    # prefix rows equal a plain prefill of the prefix alone
    alone = R.full_prefill(m, xp)
    assert np.allclose(got.k_cache[:, :P], alone.k_cache, atol=1e-12)
    # without a suffix only the last segment row is touched, from l_start on
    got2 = R.relay_prefill(m, xp, seg, 1, 2, 3, 0)
    for l in range(m.n_layers):
        assert np.array_equal(got2.v_cache[l][P:P + S - 1], seg.v[l][:S - 1])
    assert np.array_equal(got2.v_cache[0][P + S - 1], seg.v[0][S - 1])
    assert got2.active_rows == [P, P + 1, P + 1, P + 1]


def test_threshold_selector_reduces_to_forced_indices():
    """Eq. (5)-(10) inside the prefill: whatever set the selector yields, the pass equals the budget pass
    forced onto that same set (which the scalar reference pins), and the set is the hand-checkable one."""
    m, xp, xs, seg, _ = _setup()
    S = xs.shape[0]
    # suffix rule alone: cuts nobody can reach, last 3 tokens
    a = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, thresholds=(1e9, 1e9, 3))
    assert a.sel_idx.tolist() == [S - 3, S - 2, S - 1]
    b = R.relay_prefill(m, xp, seg, 1, 2, 3, 3, forced_idx=[S - 3, S - 2, S - 1])
    assert np.array_equal(a.k_cache, b.k_cache) and np.array_equal(a.logits, b.logits)
    assert a.active_rows == b.active_rows and np.array_equal(a.score, b.score)
    # everything selected == full budget
    c = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, thresholds=(1e9, 1e9, S))
    d = R.relay_prefill(m, xp, seg, 1, 2, 3, S)
    assert c.sel_idx.tolist() == list(range(S)) and np.array_equal(c.v_cache, d.v_cache)
    # influence alone: a spike at tokens 2 and 5 (mean 12/17, cut 1.45 * mean ~ 1.02), no suffix rule
    s_inf = np.zeros(S)
    s_inf[[2, 5]] = 6.0
    e = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, thresholds=(1e9, 1.45, 0), s_inf=s_inf)
    assert e.sel_idx.tolist() == [2, 5]
    f = R.relay_prefill(m, xp, seg, 1, 2, 3, 2, forced_idx=[2, 5])
    assert np.array_equal(e.k_cache, f.k_cache) and np.array_equal(e.logits, f.logits)
    # deviation rule: the cut is tau * mean of the scores the pass itself computed
    g = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, thresholds=(1.5, 1.45, 0))
    want = [j for j in range(S) if g.score[j] >= 1.5 * sum(g.score) / S]
    assert g.sel_idx.tolist() == want and 0 < len(want) < S
    # nobody selected: only the logits-carrying last token stays active after the detection layer
    h = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, thresholds=(1e9, 1e9, 0))
    assert h.sel_idx.size == 0 and h.active_rows == [9, 9 + S, 9 + 1, 9 + 1]


def test_pre_rope_and_delta_rotation_agree():
    m, xp, xs, seg_pre, _ = _setup(pre_rope=True)
    _, _, _, seg_rot, _ = _setup(pre_rope=False)
    a = R.relay_prefill(m, xp, seg_pre, 1, 2, 3, 4)
    b = R.relay_prefill(m, xp, seg_rot, 1, 2, 3, 4)
    assert np.allclose(a.k_cache, b.k_cache, atol=1e-10)
    assert np.allclose(a.logits, b.logits, atol=1e-10)
    assert a.sel_idx.tolist() == b.sel_idx.tolist()


def test_same_prefix_gives_zero_scores_and_full_prefill():
    m, xp, xs, seg, full = _setup(same_prefix=True, l_start=1)
    for k in (1, 5, 17):
        got = R.relay_prefill(m, xp, seg, 1, 2, 3, k)
        assert np.max(np.abs(got.score)) < 1e-12
        assert np.allclose(got.k_cache, full.k_cache, atol=1e-10)
        assert np.allclose(got.v_cache, full.v_cache, atol=1e-10)
        assert np.allclose(got.logits, full.logits, atol=1e-10)


def test_layer0_values_do_not_depend_on_prefix():
    m, xp, xs, seg, full = _setup()
    P = xp.shape[0]
    d0 = R.vdev_score(seg.v[0], full.v_cache[0][P:])
    assert np.max(np.abs(d0)) < 1e-13
    d1 = R.vdev_score(seg.v[1], full.v_cache[1][P:])
    assert np.max(d1) > 1e-5
    # pre-RoPE keys of layer 0 likewise
    assert np.allclose(seg.k[0], full.k_pre_rope[0][P:], atol=1e-13)


def test_position_shift_leaves_full_prefill_logits_unchanged():
    w, m = _tiny()
    x = make_hidden(w, "x", 9).astype(np.float64)
    a = R.full_prefill(m, x).logits
    b = R.full_prefill(m, x, pos0=37).logits
    assert np.allclose(a, b, atol=1e-10)


def test_causality_and_prefix_independence():
    m, xp, xs, seg, _ = _setup()
    P, S = xp.shape[0], xs.shape[0]
    base = R.relay_prefill(m, xp, seg, 1, 2, 3, 5)
    # perturb the record of the last few segment tokens: earlier rows of every layer stay put
    seg2 = R.SegmentRecord(seg.k.copy(), seg.v.copy(), seg.h_start.copy(), seg.k_is_pre_rope, seg.old_start_pos)
    cut = S - 4
    seg2.k[:, cut:] += 0.3; seg2.v[:, cut:] -= 0.2; seg2.h_start[cut:] += 0.1
    forced = [j for j in base.sel_idx.tolist()]
    a = R.relay_prefill(m, xp, seg, 1, 2, 3, 5, forced_idx=forced)
    b = R.relay_prefill(m, xp, seg2, 1, 2, 3, 5, forced_idx=forced)
    assert np.allclose(a.k_cache[:, :P + cut], b.k_cache[:, :P + cut], atol=1e-12)
    assert np.allclose(a.v_cache[:, :P + cut], b.v_cache[:, :P + cut], atol=1e-12)
    assert not np.allclose(a.logits, b.logits, atol=1e-9)
    # prefix rows never depend on the segment
    assert np.allclose(a.k_cache[:, :P], R.full_prefill(m, xp).k_cache, atol=1e-12)


def test_selected_rows_move_towards_full_prefill():
    """Rectifying more tokens cannot leave the selected rows further from FULL than pure reuse."""
    m, xp, xs, seg, full = _setup(l_start=1)
    P, S = xp.shape[0], xs.shape[0]
    seg.h_start = full.h_in[1][P:].copy()        # exact hidden states isolate the effect of selection
    zero = R.relay_prefill(m, xp, seg, 1, 2, 3, 0, x_suffix=np.zeros((1, m.d_model)))
    some = R.relay_prefill(m, xp, seg, 1, 2, 3, 6, x_suffix=np.zeros((1, m.d_model)))
    sel = some.sel_idx
    assert len(sel) == 6 and len(set(sel.tolist())) == 6
    for l in (2, 3):
        err_zero = np.abs(zero.v_cache[l][P + sel] - full.v_cache[l][P + sel]).max()
        err_some = np.abs(some.v_cache[l][P + sel] - full.v_cache[l][P + sel]).max()
        assert err_some < err_zero
    # unselected rows in sparse layers are untouched
    rest = np.setdiff1d(np.arange(S), sel)
    assert np.array_equal(some.v_cache[3][P + rest], zero.v_cache[3][P + rest])
    # the dense layer is recomputed for everyone and is exact here
    assert np.allclose(some.v_cache[1], full.v_cache[1][:P + S + 0].tolist() + [some.v_cache[1][-1].tolist()], atol=1e-10)


# ----------------------------------------------------------------------------
# decoding with the cache manager's bookkeeping (Figure "Overview" item 2, Eq. 6)
# ----------------------------------------------------------------------------
def test_decode_chain_equals_prefill_and_scalar_influence():
    w, m = _tiny(n_layers=3, name="dec3")
    T, n_prompt = 9, 4
    x = make_hidden(w, "x", T).astype(np.float64)
    full = R.full_prefill(m, x)
    pre = R.full_prefill(m, x[:n_prompt])
    shape = (m.n_layers, T, m.n_kv_heads, m.head_dim)
    kc, vc, kpre = np.zeros(shape), np.zeros(shape), np.zeros(shape)
    kc[:, :n_prompt], vc[:, :n_prompt], kpre[:, :n_prompt] = pre.k_cache, pre.v_cache, pre.k_pre_rope
    s_inf = np.zeros(T)
    caps = []
    for t in range(n_prompt, T):
        logits, cap = R.decode_step(m, x[t], t, kc, vc, k_pre_rope=kpre, capture_layer=1, s_inf=s_inf)
        caps.append(cap)
    # token-by-token decoding leaves the same cache, un-rotated keys, captured states and logits as a prefill
    assert np.allclose(kc, full.k_cache, atol=1e-11) and np.allclose(vc, full.v_cache, atol=1e-11)
    assert np.allclose(kpre, full.k_pre_rope, atol=1e-11)
    assert np.allclose(np.array(caps), full.h_in[1][n_prompt:], atol=1e-11)
    assert np.allclose(logits, full.logits, atol=1e-10)
    # every (step, layer, head) distributes exactly one unit of attention
    assert abs(np.sum(s_inf) - (T - n_prompt) * m.n_layers * m.n_q_heads) < 1e-9
    # a position can only have collected weight from steps at or after it
    assert s_inf[T - 1] <= m.n_layers * m.n_q_heads + 1e-12 and np.all(s_inf > 0)
    # scalar reference with explicit loops over steps, layers, heads and keys
    tm = B.TinyModel(m)
    want, blogits = B.brute_decode_influence(tm, _nested(x), n_prompt)
    assert np.allclose(s_inf, want, atol=1e-11)
    assert np.allclose(logits, blogits, atol=1e-10)


def test_decode_first_token_puts_all_weight_on_itself():
    w, m = _tiny(n_layers=2, name="dec1")
    x = make_hidden(w, "x", 1).astype(np.float64)
    shape = (m.n_layers, 1, m.n_kv_heads, m.head_dim)
    kc, vc = np.zeros(shape), np.zeros(shape)
    s_inf = np.zeros(1)
    logits, cap = R.decode_step(m, x[0], 0, kc, vc, s_inf=s_inf)
    assert s_inf[0] == m.n_layers * m.n_q_heads and cap is None
    assert np.allclose(logits, R.full_prefill(m, x).logits, atol=1e-12)


# ----------------------------------------------------------------------------
# layer-range profiler (Section 4.2, Eq. 2-4)
# ----------------------------------------------------------------------------
def _deviations_with_profile(s_target, n=40, seed=3):
    """d[j][l] whose layer means are exactly 1 - s_target[l] (token-wise factors sum to zero)."""
    rng = np.random.default_rng(seed)
    eps = rng.standard_normal((n, len(s_target))) * 0.2
    eps -= eps.mean(axis=0, keepdims=True)
    return (1.0 - np.asarray(s_target))[None, :] * (1.0 + eps)


def test_profiler_start_and_end_layer_hand_example():
    # U-shaped profile; worked by hand:
    #   l_min = 5.  Deepest layer <= 5 with s >= 0.99 is 2.
    #   last 5 layers: 0.93 0.95 0.955 0.953 0.956 -> mean 0.9488, population std 0.00962, b = 0.93918,
    #   lambda * std = 0.01924.  l = 5: s6 < b.  l = 6: s7 = 0.93 < b.  l = 7: |s8 - s7| = 0.02 too large.
    #   l = 8: s9, s10 >= b with steps 0.005 and 0.002 -> l_end = 8.
    s = [1.0, 0.995, 0.992, 0.97, 0.90, 0.85, 0.88, 0.93, 0.95, 0.955, 0.953, 0.956]
    prof = R.profile_layers(_deviations_with_profile(s))
    assert np.allclose(prof.s, s, atol=1e-12)
    assert (prof.l_start, prof.l_end) == (2, 8)
    assert prof.l_start < prof.l_det <= prof.l_end
    # a stricter stability rule moves the end later; a laxer threshold moves the start deeper
    assert R.profile_layers(_deviations_with_profile(s), consecutive=3).l_end == 8
    assert R.profile_layers(_deviations_with_profile(s), lam=0.4).l_end == 9      # 0.00385: the step 0.005 into layer 9 is too large
    assert R.profile_layers(_deviations_with_profile(s), lam=0.1).l_end == 11     # 0.00096: no step is small enough
    assert R.profile_layers(_deviations_with_profile(s), tau_st=0.96).l_start == 3
    assert R.profile_layers(_deviations_with_profile(s), tau_st=1.5).l_start == 0


def test_profiler_detection_layer_hand_example():
    """Eq. (4) and the choice of l* on rankings written out by hand (tests/hand_profiles.py): rho, alpha and the
    triple are typed-in numbers, not recomputed by any rule."""
    from tests import hand_profiles as H
    prof = R.profile_layers(H.deviations())
    assert np.allclose(prof.s, H.S, atol=1e-12)
    assert np.allclose(prof.rho, H.RHO, atol=1e-12)
    assert np.allclose(prof.alpha, H.ALPHA, atol=1e-12)
    assert (prof.l_start, prof.l_det, prof.l_end) == H.TRIPLE == (2, 6, 8)
    # rankings that never change from layer 1 on: rho = 1, alpha = 0, no sign change -> l_start + 1
    flat = R.profile_layers(H.deviations(ranks=[H.RANKS[0]] + [H.RANKS[5]] * 11))
    assert (flat.l_start, flat.l_det, flat.l_end) == (2, 3, 8)
    # another similarity profile under the same rankings (start and end move, l* does not), worked by hand:
    #   minimum at layer 4; tau_st 0.96: deepest layer <= 4 with s >= 0.96 is 3.
    #   last five layers 0.952 0.951 0.952 0.951 0.952: mean 0.9516, population std 0.00049, b = 0.95111.
    #   l = 4: s5 = 0.950 < b.  l = 5: s6 = 0.951 < b.  l = 6: s7 ok, s8 = 0.951 < b.  l = 7: s8 < b.
    #   l = 8: s9 ok, s10 < b.  l = 9: s10 < b.  No layer qualifies: l_end = 11, and 6 lies inside (3, 11].
    s_short = [0.999, 0.995, 0.992, 0.97, 0.90, 0.95, 0.951, 0.952, 0.951, 0.952, 0.951, 0.952]
    short = R.profile_layers(H.deviations(s=s_short), tau_st=0.96, lam=50.0)
    assert (short.l_start, short.l_det, short.l_end) == (3, 6, 11)


def test_profiler_rank_correlation_against_library_and_sign_change():
    import scipy.stats
    rng = np.random.default_rng(5)
    n, L = 200, 14
    base = rng.random(n)
    # the ranking settles with depth: the share of the common pattern rises quickly, then saturates
    share = 1.0 - np.exp(-0.55 * np.arange(L))
    d = np.stack([share[l] * base + (1 - share[l]) * rng.random(n) for l in range(L)], axis=1) * 0.05
    d[:25, 6] = d[0, 6]                                     # ties in one layer
    rho = R.spearman_adjacent(d)
    for l in range(1, L):
        assert abs(rho[l] - scipy.stats.spearmanr(d[:, l - 1], d[:, l]).statistic) < 1e-12
    assert np.array_equal(R.average_ranks([3.0, 1.0, 3.0, 2.0]), [3.5, 1.0, 3.5, 2.0])
    # second difference by an independent route, then the first + -> - change inside the range
    second = np.zeros(L)
    second[3:] = np.diff(rho[1:], n=2)
    prof = R.profile_layers(d, tau_st=0.0)                   # l_start = l_min (every layer passes the threshold)
    assert np.allclose(prof.alpha, second, atol=1e-14)
    want = next((l + 1 for l in range(4, L) if second[l - 1] > 0 > second[l] and prof.l_start < l + 1 <= prof.l_end),
                min(prof.l_start + 1, prof.l_end))
    assert prof.l_det == want
    # constant deviations in a layer: no ranking, correlation 0 on both sides
    d2 = d.copy()
    d2[:, 4] = 0.01
    rho2 = R.spearman_adjacent(d2)
    assert rho2[4] == 0.0 and rho2[5] == 0.0


# ----------------------------------------------------------------------------
# prompts with several reused segments
# ----------------------------------------------------------------------------
def _multi_setup(n_layers=4, l_start=1):
    w, m = _tiny(n_layers=n_layers, name="multi")
    sizes = dict(a=5, s1=9, b=4, s2=7, c=3, alt1=6, alt2=2)
    x = {k: make_hidden(w, k, n).astype(np.float64) for k, n in sizes.items()}
    rec1 = R.decode_record(m, x["alt1"], x["s1"], l_start)
    rec2 = R.decode_record(m, x["alt2"], x["s2"], l_start, k_is_pre_rope=False)
    return m, x, rec1, rec2


def test_multi_segment_reduces_to_single_segment_and_is_prefix_closed():
    m, x, rec1, rec2 = _multi_setup()
    one = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 3), ("new", x["b"])], 1, 2, 3)
    ref = R.relay_prefill(m, x["a"], rec1, 1, 2, 3, 3, x_suffix=x["b"])
    assert np.allclose(one.k_cache, ref.k_cache, atol=1e-12) and np.allclose(one.v_cache, ref.v_cache, atol=1e-12)
    assert one.sel_idx[0].tolist() == ref.sel_idx.tolist() and np.allclose(one.logits, ref.logits, atol=1e-11)
    assert one.active_rows == ref.active_rows
    # ending with the segment: its last token carries the logits, as in the single-segment pass
    tail = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 3)], 1, 2, 3)
    ref2 = R.relay_prefill(m, x["a"], rec1, 1, 2, 3, 3)
    assert np.allclose(tail.logits, ref2.logits, atol=1e-11) and tail.active_rows == ref2.active_rows
    # causality: what a longer prompt leaves in the rows of its first pieces is what those pieces alone leave
    both = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 3), ("new", x["b"]), ("seg", rec2, 2),
                                     ("new", x["c"])], 1, 2, 3)
    n1 = one.k_cache.shape[1]
    assert np.allclose(both.k_cache[:, :n1], one.k_cache, atol=1e-12)
    assert np.allclose(both.v_cache[:, :n1], one.v_cache, atol=1e-12)
    assert both.sel_idx[0].tolist() == one.sel_idx[0].tolist() and len(both.sel_idx[1]) == 2


def test_multi_segment_full_budget_is_full_prefill_and_zero_budget_is_reuse():
    m, x, rec1, rec2 = _multi_setup(l_start=0)
    prompt = np.concatenate([x["a"], x["s1"], x["b"], x["s2"], x["c"]])
    full = R.full_prefill(m, prompt)
    rec1.h_start, rec2.h_start = x["s1"].copy(), x["s2"].copy()       # l_start = 0: inputs are the hidden states
    got = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 9), ("new", x["b"]), ("seg", rec2, 7),
                                    ("new", x["c"])], 0, 1, m.n_layers - 1)
    assert np.allclose(got.k_cache, full.k_cache, atol=1e-10) and np.allclose(got.v_cache, full.v_cache, atol=1e-10)
    assert np.allclose(got.logits, full.logits, atol=1e-10)
    zero = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 0), ("new", x["b"]), ("seg", rec2, 0),
                                     ("new", x["c"])], 0, 1, 2)
    p1, p2 = 5, 5 + 9 + 4
    for l in range(m.n_layers):
        assert np.array_equal(zero.v_cache[l][p1:p1 + 9], rec1.v[l]) and np.array_equal(zero.v_cache[l][p2:p2 + 7], rec2.v[l])
        assert np.array_equal(zero.k_cache[l][p1:p1 + 9], R.rope_rotate(rec1.k[l], p1 + np.arange(9), m.rope_base))
        # the second record stores keys rotated at their old positions 2..8: moved by the position difference
        assert np.array_equal(zero.k_cache[l][p2:p2 + 7], R.rope_rotate(rec2.k[l], np.full(7, p2 - 2), m.rope_base))
    assert zero.active_rows == [5 + 4 + 3] * m.n_layers


def test_multi_segment_equals_scalar_reference():
    m, x, rec1, _ = _multi_setup()
    rec2 = R.decode_record(m, x["alt2"], x["s2"], 1)
    got = R.relay_prefill_multi(m, [("new", x["a"]), ("seg", rec1, 3), ("new", x["b"]), ("seg", rec2, 2),
                                    ("new", x["c"])], 1, 2, 2)
    tm = B.TinyModel(m)
    pieces = [("new", _nested(x["a"])), ("seg", _nested(rec1.k), _nested(rec1.v), _nested(rec1.h_start), 3),
              ("new", _nested(x["b"])), ("seg", _nested(rec2.k), _nested(rec2.v), _nested(rec2.h_start), 2),
              ("new", _nested(x["c"]))]
    kc, vc, sels, logits = B.brute_relay_multi(tm, pieces, 1, 2, 2)
    T = 5 + 9 + 4 + 7 + 3
    assert [s.tolist() for s in got.sel_idx] == sels
    assert np.allclose(got.k_cache, _cache_from_dicts(kc, T, 2, 4), atol=1e-10)
    assert np.allclose(got.v_cache, _cache_from_dicts(vc, T, 2, 4), atol=1e-10)
    assert np.allclose(got.logits, logits, atol=1e-10)
