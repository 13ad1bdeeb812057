"""CPU-only checks of the C ABI: the library loads, exports what the header declares, and rejects
bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

from paper_2603_13289_amd import binding as rc
from synth import ModelShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "relaycache.h")).read()
    return re.findall(r"RC_API\s+[\w\s\*]+?\b(rc_\w+)\(", text)


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 16
    assert sorted(names) == sorted(rc.EXPORTS)
    lib = C.CDLL(rc.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in rc.build_info()
    assert rc.status_str(0) == "ok" and "argument" in rc.status_str(-1)


def _cpu_model(shape):
    d, hq, hkv, dh, f = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn
    z = lambda *s: np.zeros(s, np.float32)
    layers = [dict(wq=z(hq * dh, d), wk=z(hkv * dh, d), wv=z(hkv * dh, d), wo=z(d, hq * dh), w_gate=z(f, d),
                   w_up=z(f, d), w_down=z(d, f), g_attn=z(d), g_ffn=z(d)) for _ in range(shape.n_layers)]
    return rc.rc_model_create(shape, {"layers": layers, "g_final": z(d), "w_lm": z(shape.vocab, d)}, device="cpu")


SHAPE = ModelShape(3, 64, 2, 1, 64, 64, 32, 1e4, dtype="f32")


def test_model_create_rejects_bad_shapes():
    from dataclasses import replace
    for bad, code in [(replace(SHAPE, head_dim=48), rc.RC_E_UNSUPPORTED),
                      (replace(SHAPE, n_q_heads=3, n_kv_heads=2), rc.RC_E_INVALID_ARG),
                      (replace(SHAPE, d_model=60), rc.RC_E_UNSUPPORTED),
                      (replace(SHAPE, dtype="bf16"), rc.RC_E_UNSUPPORTED),      # bf16 needs head_dim 128
                      (replace(SHAPE, n_layers=0), rc.RC_E_INVALID_ARG),
                      (replace(SHAPE, n_layers=500), rc.RC_E_CAPACITY)]:
        with pytest.raises(rc.RcError) as e:
            _cpu_model(bad)
        assert e.value.status == code


def _req(P=4, S=6, suf=0):
    t = lambda n: torch.zeros((n, SHAPE.d_model)) if n else None
    return rc.Request(t(P), t(S), t(suf), src_seq=0, src_offset=2, dst_seq=0)


def test_reuse_argument_errors_are_reported_before_any_launch():
    m = _cpu_model(SHAPE)
    kv = rc.PagedKV.contiguous(3, 1, 16, 1, 64, rc.RC_F32, device="cpu")
    logits = torch.zeros((1, 32)); sel = torch.zeros(8, dtype=torch.int32)
    ws = torch.zeros(1 << 22, dtype=torch.uint8)

    def call(reqs, plan, src=kv, dst=kv, workspace=ws, logits_=logits):
        rc.rc_reuse(m, reqs, plan, src, dst, logits_, sel, None, workspace)

    def status(fn):
        with pytest.raises(rc.RcError) as e:
            fn()
        return e.value.status

    ok_plan = rc.Plan(0, 1, 2, [2])
    assert rc.rc_reuse_workspace_bytes(m, [_req()], ok_plan) > 0
    assert rc.rc_reuse_workspace_bytes(m, [_req()], rc.Plan(1, 1, 2, [2])) == 0
    assert status(lambda: call([_req()], rc.Plan(1, 1, 2, [2]))) == rc.RC_E_INVALID_ARG      # l_det <= l_start
    assert status(lambda: call([_req()], rc.Plan(0, 2, 1, [2]))) == rc.RC_E_INVALID_ARG      # l_end < l_det
    assert status(lambda: call([_req()], rc.Plan(0, 1, 3, [2]))) == rc.RC_E_INVALID_ARG      # l_end >= n_layers
    assert status(lambda: call([_req()], rc.Plan(0, 1, 2, [7]))) == rc.RC_E_INVALID_ARG      # k > S
    assert status(lambda: call([_req()], rc.Plan(0, 1, 2, [-1]))) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()] * 33, rc.Plan(0, 1, 2, [1] * 33))) == rc.RC_E_CAPACITY
    assert status(lambda: call([_req(P=20)], ok_plan)) == rc.RC_E_CAPACITY                   # sequence > table
    r = _req(); r.dst_seq = 3
    assert status(lambda: call([r], ok_plan)) == rc.RC_E_CAPACITY
    assert status(lambda: call([_req()], ok_plan, workspace=torch.zeros(256, dtype=torch.uint8))) == rc.RC_E_WORKSPACE
    assert status(lambda: call([_req()], ok_plan, logits_=None)) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()], ok_plan, src=None)) == rc.RC_E_INVALID_ARG
    # threshold selector: no forced indices, no negative suffix count or cut, a count output is required
    thr = lambda **kw: rc.Plan(0, 1, 2, None, None, rc.RC_SELECT_THRESHOLD, **kw)
    assert rc.rc_reuse_workspace_bytes(m, [_req()], thr()) >= rc.rc_reuse_workspace_bytes(m, [_req()], ok_plan)
    assert status(lambda: call([_req()], thr(k_suf=-1))) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()], thr(tau_dev=-0.5))) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()], thr(tau_inf=float("nan")))) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()], rc.Plan(0, 1, 2, None, sel, rc.RC_SELECT_THRESHOLD))) == rc.RC_E_INVALID_ARG
    assert status(lambda: call([_req()], thr())) == rc.RC_E_INVALID_ARG                      # sel_cnt missing
    assert status(lambda: call([_req()], rc.Plan(0, 1, 2, [2], None, 7))) == rc.RC_E_INVALID_ARG   # unknown selector
    assert status(lambda: call([_req()], rc.Plan(0, 1, 2, None))) == rc.RC_E_INVALID_ARG     # budget without counts
    m.close()


def test_reuse_in_shared_pools_needs_a_block_aligned_move():
    """Source and destination in the same pools: allowed only when the segment moves by whole blocks."""
    m = _cpu_model(SHAPE)
    table = [[0, 1, 2, 3], [4, 5, 6, 7]]
    kv = rc.PagedKV(3, 8, 4, 1, 64, rc.RC_F32, table, device="cpu")
    other = rc.PagedKV(3, 8, 4, 1, 64, rc.RC_F32, table, device="cpu")
    logits = torch.zeros((1, 32)); sel = torch.zeros(8, dtype=torch.int32)
    raw = torch.zeros((1 << 22) + 256, dtype=torch.uint8)
    ws = raw[(-raw.data_ptr()) % 256:]                    # the workspace check wants 256-byte alignment
    plan = rc.Plan(0, 1, 2, [2])

    def status(req, src, dst):
        try:
            rc.rc_reuse(m, [req], plan, src, dst, logits, sel, None, ws)
        except rc.RcError as e:
            return e.status
        return rc.RC_OK

    t = lambda n: torch.zeros((n, SHAPE.d_model))
    moved_by_3 = rc.Request(t(5), t(6), None, src_seq=0, src_offset=2, dst_seq=1)          # 5 - 2 = 3, blocks of 4
    assert status(moved_by_3, kv, kv) == rc.RC_E_UNSUPPORTED
    cached = rc.Request(t(1), t(6), None, src_seq=0, src_offset=2, dst_seq=1, n_cached=2)  # 2 + 1 - 2 = 1
    assert status(cached, kv, kv) == rc.RC_E_UNSUPPORTED
    mixed = rc.PagedKV.from_pools(kv.k, other.v, kv.block_table, rc.RC_F32)                 # only the key pools shared
    assert status(moved_by_3, kv, mixed) == rc.RC_E_UNSUPPORTED
    # (an aligned move in shared pools and any move between separate caches pass this check; they go on to launch
    # kernels, which the GPU tests cover)
    m.close()


def test_stage_argument_errors():
    def status(fn):
        with pytest.raises(rc.RcError) as e:
            fn()
        return e.value.status
    s = torch.zeros(8); idx = torch.zeros(8, dtype=torch.int32)
    assert status(lambda: rc.rc_topk(s, 8, 9, idx)) == rc.RC_E_INVALID_ARG
    assert status(lambda: rc.rc_topk(s, (1 << 20) + 1, 1, idx)) == rc.RC_E_CAPACITY
    rc.rc_topk(s, 8, 0, idx)       # k = 0 is a no-op, no launch
    kv = rc.PagedKV.contiguous(1, 1, 16, 2, 64, rc.RC_F32, device="cpu")
    lay = kv.layer(0)
    assert status(lambda: rc.rc_sparse_attention(s, idx, 1, 3, lay, 0, s, None)) == rc.RC_E_INVALID_ARG   # 3 % 2 heads
    assert status(lambda: rc.rc_sparse_attention(s, idx, 1, 2, lay, 5, s, None)) == rc.RC_E_CAPACITY
    assert status(lambda: rc.rc_gemm_rows(rc.RC_F32, s, s, s, 1, 1, 4, None)) == rc.RC_E_UNSUPPORTED      # k % 8
    assert status(lambda: rc.rc_gemm_rows_fused(rc.RC_F32, 4, s, s, None, s, 1, 1, 8)) == rc.RC_E_INVALID_ARG   # epilogue
    assert status(lambda: rc.rc_gemm_rows_fused(rc.RC_F32, rc.RC_GEMM_SWIGLU, s, s, None, s, 1, 1, 8)) == rc.RC_E_INVALID_ARG
    assert status(lambda: rc.rc_gemm_rows_fused(rc.RC_F32, rc.RC_GEMM_ADD, s, s, s, s, 1, 1, 8)) == rc.RC_E_INVALID_ARG
    assert rc.rc_stage_workspace_bytes(10, 64) > 0
    assert status(lambda: rc.rc_ceiling_stream_copy(s, s, 24)) == rc.RC_E_INVALID_ARG                      # not 16-byte units
    assert status(lambda: rc.rc_ceiling_mfma_loop(s, 0, 10)) == rc.RC_E_INVALID_ARG
    assert rc.rc_ceiling_mfma_loop_out_bytes(2) == 2 * 512 * 4


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
