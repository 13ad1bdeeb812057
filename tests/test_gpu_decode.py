"""Decoding steps with the cache manager's bookkeeping (rc_decode_step) against the CPU oracle, and the closed
loop: a segment record and influence scores produced by decoding on the GPU feed the selective-recompute prefill."""
import numpy as np
import pytest
import torch

from oracle import relay_oracle as R
from synth import WORKLOADS, make_block_table, make_hidden, make_weights
from tests.harness import TOL, rel_err, round_store, threshold_margin, to_np

pytestmark = pytest.mark.gpu


def _setup(name):
    from paper_2603_13289_amd import binding as rc
    w = WORKLOADS[name]
    weights = make_weights(w)
    om = R.OracleModel.from_shape(w.shape, weights)
    model = rc.rc_model_create(w.shape, weights)
    return rc, w, om, model


def _up(rc, w, x):
    td = rc.torch_dtype(rc.rc_dtype_of(w.shape.dtype))
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda().to(td).contiguous()


def _oracle_chain(om, x, n_prompt, capture_layer):
    """Prefill of the prompt, then one decode_step per remaining token."""
    T = x.shape[0]
    pre = R.full_prefill(om, x[:n_prompt])
    shape = (om.n_layers, T, om.n_kv_heads, om.head_dim)
    kc, vc, kpre = np.zeros(shape), np.zeros(shape), np.zeros(shape)
    kc[:, :n_prompt], vc[:, :n_prompt], kpre[:, :n_prompt] = pre.k_cache, pre.v_cache, pre.k_pre_rope
    s_inf = np.zeros(T)
    caps, logits = [], []
    for t in range(n_prompt, T):
        lg, cap = R.decode_step(om, x[t], t, kc, vc, k_pre_rope=kpre, capture_layer=capture_layer, s_inf=s_inf)
        caps.append(cap)
        logits.append(lg)
    return kc, vc, kpre, np.array(caps), np.array(logits), s_inf


def _hip_chain(rc, w, model, xs, n_prompts, capture_layer, paged):
    """The same on the GPU for a batch of sequences of different lengths (one decoding step per call)."""
    sh = w.shape
    dt = rc.rc_dtype_of(sh.dtype)
    td = rc.torch_dtype(dt)
    n = len(xs)
    lens = [x.shape[0] for x in xs]
    if paged:
        tab, nb = make_block_table(lens, 16, seed=5)
        cache = rc.PagedKV(sh.n_layers, nb, 16, sh.n_kv_heads, sh.head_dim, dt, tab)
        kpre = rc.PagedKV(sh.n_layers, nb, 16, sh.n_kv_heads, sh.head_dim, dt, tab)
    else:
        cache = rc.PagedKV.contiguous(sh.n_layers, n, max(lens), sh.n_kv_heads, sh.head_dim, dt)
        kpre = rc.PagedKV.contiguous(sh.n_layers, n, max(lens), sh.n_kv_heads, sh.head_dim, dt)
    xd = [_up(rc, w, x) for x in xs]
    lg = torch.zeros((n, sh.vocab), dtype=torch.float32, device="cuda")
    ws = rc.alloc_workspace(rc.rc_prefill_workspace_bytes(model, n_prompts))
    rc.rc_prefill(model, [xd[b][:n_prompts[b]].contiguous() for b in range(n)], list(range(n)), cache, lg, ws, k_pre=kpre)
    s_inf = [torch.zeros(lens[b], dtype=torch.float32, device="cuda") for b in range(n)]
    caps = [torch.zeros((lens[b], sh.d_model), dtype=td, device="cuda") for b in range(n)]
    logits = [[] for _ in range(n)]
    step = 0
    while True:
        live = [b for b in range(n) if n_prompts[b] + step < lens[b]]
        if not live:
            break
        reqs = [rc.DecodeReq(xd[b][n_prompts[b] + step], n_prompts[b] + step, b, caps[b][n_prompts[b] + step], s_inf[b])
                for b in live]
        ws = rc.alloc_workspace(rc.rc_decode_workspace_bytes(model, reqs))
        out = torch.zeros((len(live), sh.vocab), dtype=torch.float32, device="cuda")
        rc.rc_decode_step(model, reqs, cache, out, ws, k_pre=kpre, capture_layer=capture_layer)
        torch.cuda.synchronize()
        for i, b in enumerate(live):
            logits[b].append(to_np(out[i]))
        step += 1
    return cache, kpre, caps, logits, s_inf


@pytest.mark.parametrize("name,paged", [("tiny5_f32", False), ("tiny5_f32", True), ("small_bf16", True),
                                        ("mistral7b_trunc", False)])
def test_decode_chain_matches_oracle(name, paged):
    rc, w, om, model = _setup(name)
    tol = TOL[w.shape.dtype]
    lens, prompts = [41, 23], [17, 20]
    xs = [make_hidden(w, "x_dec", lens[b], b) for b in range(2)]
    cap_layer = 1
    cache, kpre, caps, logits, s_inf = _hip_chain(rc, w, model, xs, prompts, cap_layer, paged)
    for b in range(2):
        kc, vc, kp, ocaps, ologits, os_inf = _oracle_chain(om, xs[b].astype(np.float64), prompts[b], cap_layer)
        for l in range(w.shape.n_layers):
            assert rel_err(to_np(cache.read("k", l, b, lens[b])), kc[l]) <= tol
            assert rel_err(to_np(cache.read("v", l, b, lens[b])), vc[l]) <= tol
            assert rel_err(to_np(kpre.read("k", l, b, lens[b])), kp[l]) <= tol
        assert rel_err(to_np(caps[b][prompts[b]:]), ocaps) <= tol
        assert rel_err(np.array(logits[b]), ologits) <= tol
        got = to_np(s_inf[b])
        assert rel_err(got, os_inf) <= tol
        # every (step, layer, query head) hands out one unit of attention
        units = (lens[b] - prompts[b]) * w.shape.n_layers * w.shape.n_q_heads
        assert abs(float(got.astype(np.float64).sum()) - units) <= 1e-4 * units
    model.close()


def test_decode_without_bookkeeping_and_first_position():
    """No un-rotated keys, no capture, no influence; a sequence that starts empty (position 0)."""
    rc, w, om, model = _setup("tiny5_f32")
    sh = w.shape
    x = make_hidden(w, "x_dec0", 3)
    cache = rc.PagedKV.contiguous(sh.n_layers, 1, 8, sh.n_kv_heads, sh.head_dim, rc.RC_F32)
    full = R.full_prefill(om, x.astype(np.float64))
    for t in range(3):
        req = [rc.DecodeReq(_up(rc, w, x[t]), t, 0)]
        lg = torch.zeros((1, sh.vocab), dtype=torch.float32, device="cuda")
        rc.rc_decode_step(model, req, cache, lg, rc.alloc_workspace(rc.rc_decode_workspace_bytes(model, req)))
    torch.cuda.synchronize()
    for l in range(sh.n_layers):
        assert rel_err(to_np(cache.read("k", l, 0, 3)), full.k_cache[l]) <= TOL["f32"]
    assert rel_err(to_np(lg)[0], full.logits) <= TOL["f32"]
    # capacity is checked on the host
    with pytest.raises(rc.RcError) as e:
        rc.rc_decode_step(model, [rc.DecodeReq(_up(rc, w, x[0]), 8, 0)], cache, lg, rc.alloc_workspace(1 << 20))
    assert e.value.status == rc.RC_E_CAPACITY
    model.close()


def test_closed_loop_record_from_decoding_feeds_threshold_selector():
    """Stage i-1 on the GPU: prefill of its own prompt, then the segment is generated token by token while the
    cache manager keeps un-rotated keys, hidden states at l_start and influence scores.  Stage i takes that
    record over (different prefix) with the selector of Eq. (5)-(10).  The oracle does the same chain."""
    rc, w, om, model = _setup("tiny5_f32")
    sh = w.shape
    A, S, P = 19, 37, 26
    l_start, l_det, l_end = 1, 2, 3
    x_alt, x_seg, x_new = make_hidden(w, "loop_alt", A), make_hidden(w, "loop_seg", S), make_hidden(w, "loop_new", P)
    x_old = np.concatenate([x_alt, x_seg])
    # --- oracle chain
    kc, vc, kp, ocaps, _, os_inf = _oracle_chain(om, x_old.astype(np.float64), A, l_start)
    seg = R.SegmentRecord(round_store(kp[:, A:], "f32").astype(np.float64), round_store(vc[:, A:], "f32").astype(np.float64),
                          round_store(ocaps, "f32").astype(np.float64), True, A)
    s_inf_seg = os_inf[A:].astype(np.float32)
    probe = R.relay_prefill(om, x_new, seg, l_start, l_det, l_end, 0, thresholds=(1.5, 1.45, 4), s_inf=s_inf_seg)
    tau_dev = next(t for t in (1.5 * (1 + 0.01 * i) for i in range(40)) if threshold_margin(probe.score, t) > 2e-3)
    tau_inf = next(t for t in (1.45 * (1 + 0.01 * i) for i in range(40)) if threshold_margin(s_inf_seg, t) > 2e-3)
    want = R.relay_prefill(om, x_new, seg, l_start, l_det, l_end, 0, thresholds=(tau_dev, tau_inf, 4), s_inf=s_inf_seg)
    assert 4 <= len(want.sel_idx) < S
    # --- the library
    cache, kpre, caps, _, s_inf = _hip_chain(rc, w, model, [x_old], [A], l_start, paged=True)
    record = rc.PagedKV.from_pools(kpre.k, cache.v, cache.block_table, rc.RC_F32)
    dst = rc.PagedKV.contiguous(sh.n_layers, 1, P + S, sh.n_kv_heads, sh.head_dim, rc.RC_F32)
    req = rc.Request(_up(rc, w, x_new), caps[0][A:].contiguous(), None, src_seq=0, src_offset=A, k_is_pre_rope=True,
                     seg_old_start_pos=A, s_inf=s_inf[0][A:].contiguous())
    plan = rc.Plan(l_start, l_det, l_end, None, None, rc.RC_SELECT_THRESHOLD, tau_dev, tau_inf, 4)
    ws = rc.alloc_workspace(rc.rc_reuse_workspace_bytes(model, [req], plan))
    logits = torch.zeros((1, sh.vocab), dtype=torch.float32, device="cuda")
    sel = torch.full((S,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc.rc_reuse(model, [req], plan, record, dst, logits, sel, None, ws, sel_cnt=cnt)
    torch.cuda.synchronize()
    c = int(cnt.item())
    assert np.array_equal(sel.cpu().numpy()[:c], want.sel_idx)
    for l in range(sh.n_layers):
        assert rel_err(to_np(dst.read("k", l, 0, P + S)), want.k_cache[l]) <= TOL["f32"]
        assert rel_err(to_np(dst.read("v", l, 0, P + S)), want.v_cache[l]) <= TOL["f32"]
    assert rel_err(to_np(logits)[0], want.logits) <= TOL["f32"]
    model.close()
