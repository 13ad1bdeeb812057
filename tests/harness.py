"""Shared helpers of the GPU parity tests: build a seeded case, run the oracle, run the HIP path.

The oracle side and the HIP side only share the seeded inputs (synth/) and the
earlier agent's segment record, which the oracle produces and which is rounded
to the workload's storage type once before either side consumes it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from oracle import relay_oracle as R
from synth import (WORKLOADS, Workload, budget_to_k, make_block_table, make_hidden, make_weights, ragged_lengths,
                   round_to_bf16)

TOL = {"f32": 1e-4, "bf16": 2e-2}      # max |x - y| / max |y| per tensor


def rel_err(got, want) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-30))


def row_rel_err(got, want, floor_frac: float = 0.05) -> float:
    """Worst row of max|x - y| over a row divided by that row's own max|y|, rows being the vectors along the
    last axis (one token and head of a cache, one logits vector).  The divisor is at least floor_frac of the
    tensor's max|y|, so a row that is small against the rest of the tensor is still held to an absolute bound."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    err = np.max(np.abs(got - want), axis=-1)
    ref = np.maximum(np.max(np.abs(want), axis=-1), floor_frac * max(np.max(np.abs(want)), 1e-30))
    return float(np.max(err / ref))


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def round_store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


@dataclass
class ReqCase:
    P: int
    S: int
    A: int
    xp: np.ndarray
    xa: np.ndarray
    xs: np.ndarray
    xsuf: Optional[np.ndarray]
    seg: R.SegmentRecord            # record after storage rounding
    k: int


@dataclass
class Case:
    w: Workload
    weights: dict
    om: R.OracleModel
    reqs: List[ReqCase]


def build_case(name: str, k_override: Optional[int] = None, pre_rope: bool = True, n_suffix: int = 0,
               l_triple=None, max_req: Optional[int] = None, seed: Optional[int] = None) -> Case:
    """seed: master seed of the token hidden states, one for all requests or a list with one per request (weights
    keep the default seed); None = the default."""
    w = WORKLOADS[name]
    if l_triple is not None:
        from dataclasses import replace
        w = replace(w, l_start=l_triple[0], l_det=l_triple[1], l_end=l_triple[2])
    weights = make_weights(w)
    om = R.OracleModel.from_shape(w.shape, weights)
    reqs = []
    lens = ragged_lengths(w)
    if max_req is not None:
        lens = lens[:max_req]
    for b, (P, S, A) in enumerate(lens):
        hs = {} if seed is None else {"seed": seed[b] if isinstance(seed, (list, tuple)) else seed}
        xp = make_hidden(w, "x_prefix", P, b, **hs)
        xa = make_hidden(w, "x_alt", A, b, **hs)
        xs = make_hidden(w, "x_seg", S, b, **hs)
        xsuf = make_hidden(w, "x_suffix", n_suffix, b, **hs) if n_suffix else None
        seg = R.decode_record(om, xa, xs, w.l_start, k_is_pre_rope=pre_rope)
        dt = w.shape.dtype
        seg = R.SegmentRecord(round_store(seg.k, dt).astype(np.float64), round_store(seg.v, dt).astype(np.float64),
                              round_store(seg.h_start, dt).astype(np.float64), pre_rope, A)
        k = budget_to_k(S, w.budget_pct) if k_override is None else min(k_override, S)
        reqs.append(ReqCase(P, S, A, xp, xa, xs, xsuf, seg, k))
    return Case(w, weights, om, reqs)


def oracle_relay(case: Case, b: int = 0, forced_idx=None, thresholds=None, s_inf=None) -> R.RelayResult:
    rq = case.reqs[b]
    w = case.w
    return R.relay_prefill(case.om, rq.xp, rq.seg, w.l_start, w.l_det, w.l_end, rq.k, x_suffix=rq.xsuf,
                           forced_idx=forced_idx, thresholds=thresholds, s_inf=s_inf)


def build_case_with_margin(name: str, margin: float, **kw):
    """A case whose oracle selection is safe to compare bit for bit across precisions: every request's input seed
    is bumped until the oracle's k-th and (k+1)-th largest scores of that request are further apart (relatively)
    than `margin` (requests are independent, so each is bumped on its own; k = 0 and k = S always qualify).
    Returns (case, [oracle result per request], [seed per request])."""
    from dataclasses import replace
    from synth.workloads import MASTER_SEED
    def safe(case, b, want):
        kb = case.reqs[b].k
        # scores that are rounding noise around zero (identical prefixes) have no meaningful ranking
        real = kb in (0, case.reqs[b].S) or np.sort(want.score)[::-1][kb - 1] > 1e-9
        return real and selection_margin(want.score, kb) > margin

    case = build_case(name, **kw)
    n_req = len(case.reqs)
    seeds = [MASTER_SEED] * n_req
    reqs = list(case.reqs)
    wants = [oracle_relay(case, b) for b in range(n_req)]
    for b in range(n_req):
        bump = 0
        while not safe(case, b, wants[b]):
            bump += 1
            if bump >= 64:
                raise AssertionError(f"{name} request {b}: no seed in 64 gives a selection margin above {margin}")
            seeds[b] = MASTER_SEED + bump
            case = build_case(name, seed=list(seeds), **kw)
            wants[b] = oracle_relay(case, b)
            reqs[b] = case.reqs[b]
    return replace(case, reqs=reqs), wants, seeds


def threshold_margin(score: np.ndarray, tau: float) -> float:
    """Smallest relative distance of a score from the cut tau * mean(score) of Eq. (5) / Eq. (7)."""
    score = np.asarray(score, np.float64)
    cut = tau * float(np.mean(score))
    return float(np.min(np.abs(score - cut)) / max(abs(cut), 1e-300))


def selection_margin(score: np.ndarray, k: int) -> float:
    """Relative gap between the k-th and (k+1)-th largest score (inf when k is 0 or all)."""
    if k <= 0 or k >= score.shape[0]:
        return float("inf")
    s = np.sort(score)[::-1]
    return float((s[k - 1] - s[k]) / max(abs(s[k - 1]), 1e-300))


# ------------------------------------------------------------------ HIP side
@dataclass
class HipRun:
    k_cache: List[List[np.ndarray]]      # [req][layer] -> [T][Hkv][dh]
    v_cache: List[List[np.ndarray]]
    logits: np.ndarray                   # [n_req][vocab]
    sel: List[np.ndarray]
    scores: List[np.ndarray]


def hip_relay(case: Case, forced: Optional[List[np.ndarray]] = None, paged_src: bool = True,
              thresholds=None, s_inf: Optional[List[Optional[np.ndarray]]] = None) -> HipRun:
    """thresholds = (tau_dev, tau_inf, k_suf) runs the selector of Eq. (5)-(10) instead of the budget."""
    from paper_2603_13289_amd import binding as rc
    w, sh = case.w, case.w.shape
    dt = rc.rc_dtype_of(sh.dtype)
    td = rc.torch_dtype(dt)
    dev = "cuda"
    model = rc.rc_model_create(sh, case.weights)
    n_req = len(case.reqs)

    def up(x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev).to(td).contiguous()

    # the earlier agents' caches: sequence b holds [alt_b ; seg_b]; only the segment rows are filled
    src_lens = [r.A + r.S for r in case.reqs]
    dst_lens = [r.P + r.S + (0 if r.xsuf is None else r.xsuf.shape[0]) for r in case.reqs]
    if w.block_size > 0:
        st, sn = make_block_table(src_lens, w.block_size, seed=1)
        dtab, dn = make_block_table(dst_lens, w.block_size, seed=2)
        src = rc.PagedKV(sh.n_layers, sn, w.block_size, sh.n_kv_heads, sh.head_dim, dt, st)
        dst = rc.PagedKV(sh.n_layers, dn, w.block_size, sh.n_kv_heads, sh.head_dim, dt, dtab, fill=7.0)
    else:
        src = rc.PagedKV.contiguous(sh.n_layers, n_req, max(src_lens), sh.n_kv_heads, sh.head_dim, dt)
        dst = rc.PagedKV.contiguous(sh.n_layers, n_req, max(dst_lens), sh.n_kv_heads, sh.head_dim, dt, fill=7.0)
    reqs = []
    for b, r in enumerate(case.reqs):
        for l in range(sh.n_layers):
            src.write("k", l, b, up(r.seg.k[l]), start=r.A)
            src.write("v", l, b, up(r.seg.v[l]), start=r.A)
        reqs.append(rc.Request(up(r.xp) if r.P else None, up(r.seg.h_start), None if r.xsuf is None else up(r.xsuf),
                               src_seq=b, src_offset=r.A, k_is_pre_rope=r.seg.k_is_pre_rope,
                               seg_old_start_pos=r.seg.old_start_pos, dst_seq=b,
                               s_inf=None if s_inf is None or s_inf[b] is None else
                               torch.from_numpy(np.ascontiguousarray(s_inf[b], np.float32)).to(dev)))
    ks = [r.k for r in case.reqs]
    fidx = None
    if forced is not None:
        fidx = torch.from_numpy(np.concatenate([np.asarray(f, np.int32) for f in forced])).to(dev)
    sum_seg = sum(r.S for r in case.reqs)
    cnt = None
    if thresholds is None:
        plan = rc.Plan(w.l_start, w.l_det, w.l_end, ks, fidx)
    else:
        plan = rc.Plan(w.l_start, w.l_det, w.l_end, None, None, rc.RC_SELECT_THRESHOLD, float(thresholds[0]),
                       float(thresholds[1]), int(thresholds[2]))
        cnt = torch.full((n_req,), -1, dtype=torch.int32, device=dev)
    ws = rc.alloc_workspace(rc.rc_reuse_workspace_bytes(model, reqs, plan))
    logits = torch.zeros((n_req, sh.vocab), dtype=torch.float32, device=dev)
    sel = torch.full((max(sum(ks) if thresholds is None else sum_seg, 1),), -1, dtype=torch.int32, device=dev)
    scores = torch.full((sum_seg,), -5.0, dtype=torch.float32, device=dev)
    rc.rc_reuse(model, reqs, plan, src, dst, logits, sel, scores, ws, sel_cnt=cnt)
    torch.cuda.synchronize()
    cnt_h = None if cnt is None else cnt.cpu().numpy()
    out_k, out_v, out_sel, out_sc = [], [], [], []
    so = ko = 0
    for b, r in enumerate(case.reqs):
        out_k.append([to_np(dst.read("k", l, b, dst_lens[b])) for l in range(sh.n_layers)])
        out_v.append([to_np(dst.read("v", l, b, dst_lens[b])) for l in range(sh.n_layers)])
        if cnt_h is None:
            out_sel.append(sel[ko:ko + r.k].cpu().numpy())
        else:
            out_sel.append(sel[so:so + max(int(cnt_h[b]), 0)].cpu().numpy())
        out_sc.append(scores[so:so + r.S].cpu().numpy())
        ko += r.k
        so += r.S
    res = HipRun(out_k, out_v, to_np(logits), out_sel, out_sc)
    model.close()
    return res


def hip_full_prefill(case: Case, b: int = 0, capture_layer: int = 0):
    """rc_prefill of [prefix ; segment] of request b; returns (k, v, k_pre, h_capture, logits)."""
    from paper_2603_13289_amd import binding as rc
    sh = case.w.shape
    dt = rc.rc_dtype_of(sh.dtype)
    td = rc.torch_dtype(dt)
    model = rc.rc_model_create(sh, case.weights)
    r = case.reqs[b]
    x = torch.from_numpy(np.concatenate([r.xp, r.xs]).astype(np.float32)).to("cuda").to(td).contiguous()
    T = x.shape[0]
    bs = case.w.block_size
    if bs > 0:
        tab, nb = make_block_table([T], bs, seed=3)
        dst = rc.PagedKV(sh.n_layers, nb, bs, sh.n_kv_heads, sh.head_dim, dt, tab)
        kpre = rc.PagedKV(sh.n_layers, nb, bs, sh.n_kv_heads, sh.head_dim, dt, tab)
    else:
        dst = rc.PagedKV.contiguous(sh.n_layers, 1, T, sh.n_kv_heads, sh.head_dim, dt)
        kpre = rc.PagedKV.contiguous(sh.n_layers, 1, T, sh.n_kv_heads, sh.head_dim, dt)
    hcap = torch.zeros((T, sh.d_model), dtype=td, device="cuda")
    logits = torch.zeros((1, sh.vocab), dtype=torch.float32, device="cuda")
    ws = rc.alloc_workspace(rc.rc_prefill_workspace_bytes(model, [T]))
    rc.rc_prefill(model, [x], [0], dst, logits, ws, k_pre=kpre, capture_layer=capture_layer, h_capture=[hcap])
    torch.cuda.synchronize()
    k = [to_np(dst.read("k", l, 0, T)) for l in range(sh.n_layers)]
    v = [to_np(dst.read("v", l, 0, T)) for l in range(sh.n_layers)]
    kp = [to_np(kpre.read("k", l, 0, T)) for l in range(sh.n_layers)]
    model.close()
    return k, v, kp, to_np(hcap), to_np(logits)[0]
