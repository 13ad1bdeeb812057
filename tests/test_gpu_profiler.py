"""Calibration pass of the layer-range profiler on the GPU: Eq. (1) of every segment token at every layer
(full prefill of [new prefix ; segment] against the record left by [other prefix ; segment]), then the
host-side rules of Eq. (2)-(4), against the oracle."""
import numpy as np
import pytest
import torch

from oracle import relay_oracle as R
from synth import WORKLOADS, make_hidden, make_weights
from tests.harness import TOL, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny5_f32", "small_bf16"])
def test_calibration_pass_and_profile(name):
    from paper_2603_13289_amd import binding as rc
    w = WORKLOADS[name]
    sh = w.shape
    dt = rc.rc_dtype_of(sh.dtype)
    td = rc.torch_dtype(dt)
    weights = make_weights(w)
    om = R.OracleModel.from_shape(sh, weights)
    model = rc.rc_model_create(sh, weights)
    A, P, S = 23, 31, 90
    x_alt, x_new, x_seg = make_hidden(w, "cal_alt", A), make_hidden(w, "cal_new", P), make_hidden(w, "cal_seg", S)
    up = lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda().to(td).contiguous()

    def prefill(x):
        T = x.shape[0]
        kv = rc.PagedKV.contiguous(sh.n_layers, 1, T, sh.n_kv_heads, sh.head_dim, dt)
        lg = torch.zeros((1, sh.vocab), dtype=torch.float32, device="cuda")
        rc.rc_prefill(model, [up(x)], [0], kv, lg, rc.alloc_workspace(rc.rc_prefill_workspace_bytes(model, [T])))
        return kv

    reuse = prefill(np.concatenate([x_alt, x_seg]))       # what the earlier agent left behind
    full = prefill(np.concatenate([x_new, x_seg]))        # the reference the segment should have had
    ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(0, sh.head_dim))
    d = torch.zeros((sh.n_layers, S), dtype=torch.float32, device="cuda")
    for l in range(sh.n_layers):
        v_full = full.read("v", l, 0, S, start=P).contiguous()
        rc.rc_vdev_score(v_full, reuse.layer(l), 0, A, S, d[l], ws)
    torch.cuda.synchronize()
    d_gpu = d.cpu().numpy()
    # oracle deviations from its own two prefills
    o_reuse = R.full_prefill(om, np.concatenate([x_alt, x_seg]).astype(np.float64))
    o_full = R.full_prefill(om, np.concatenate([x_new, x_seg]).astype(np.float64))
    d_want = np.stack([R.vdev_score(o_reuse.v_cache[l][A:], o_full.v_cache[l][P:]) for l in range(sh.n_layers)])
    assert np.allclose(d_gpu[0], 0.0, atol=1e-6 if sh.dtype == "f32" else 1e-4)      # layer-0 values ignore the prefix
    tol = TOL[sh.dtype]
    assert np.max(np.abs(d_gpu - d_want)) <= tol * max(np.max(d_want), 1e-3)
    # the rules, applied by the library and by the oracle to the same deviations
    params = (0.99, 2, 2.0, 1) if sh.n_layers < 8 else (0.99, 5, 2.0, 2)
    (l_start, l_det, l_end), s, rho = rc.rc_layer_profile(d_gpu, *params)
    want = R.profile_layers(d_gpu.T.astype(np.float64), tau_st=float(np.float32(params[0])), tail=params[1],
                            lam=params[2], consecutive=params[3])
    assert (l_start, l_det, l_end) == (want.l_start, want.l_det, want.l_end)
    assert np.allclose(s, want.s, atol=1e-12) and np.allclose(rho, want.rho, atol=1e-12)
    assert np.allclose(s, R.layer_similarity(d_want.T), atol=tol)
    model.close()
