"""Stage-level parity: each kernel family through the C ABI against the CPU oracle's stage function."""
import numpy as np
import pytest
import torch

from oracle import relay_oracle as R
from synth import make_block_table, round_to_bf16, stream_rng
from tests.harness import TOL, rel_err, to_np

pytestmark = pytest.mark.gpu


def _rc():
    from paper_2603_13289_amd import binding as rc
    return rc


def _td(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def _rand(shape, dtype, name, scale=1.0):
    x = stream_rng("stage", name).standard_normal(shape, dtype=np.float32) * np.float32(scale)
    return round_to_bf16(x) if dtype == "bf16" else x


def _up(x, dtype):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda().to(_td(dtype)).contiguous()


def _cache(dtype, hkv, dh, lens, block_size, name, fill_random=True):
    """A one-layer cache with random content; returns (PagedKV, [seq] -> K rows, V rows as numpy)."""
    rc = _rc()
    dt = rc.rc_dtype_of(dtype)
    if block_size:
        tab, nb = make_block_table(lens, block_size, seed=11)
        kv = rc.PagedKV(1, nb, block_size, hkv, dh, dt, tab)
    else:
        kv = rc.PagedKV.contiguous(1, len(lens), max(lens), hkv, dh, dt)
    ks, vs = [], []
    for s, n in enumerate(lens):
        k = _rand((n, hkv, dh), dtype, f"{name}k{s}")
        v = _rand((n, hkv, dh), dtype, f"{name}v{s}")
        if fill_random:
            kv.write("k", 0, s, _up(k, dtype))
            kv.write("v", 0, s, _up(v, dtype))
        ks.append(k)
        vs.append(v)
    return kv, ks, vs


# ------------------------------------------------------------------ K1
@pytest.mark.parametrize("dtype,hkv,dh", [("f32", 2, 64), ("bf16", 8, 128), ("f32", 3, 128)])
@pytest.mark.parametrize("block_size", [0, 16])
@pytest.mark.parametrize("pre_rope", [True, False])
def test_rope_rerotate(dtype, hkv, dh, block_size, pre_rope):
    rc = _rc()
    n, src_off, dst_off, old = 203, 37, 129, 37
    base = 10000.0 if dtype == "f32" else 1.0e6
    src, ks, vs = _cache(dtype, hkv, dh, [src_off + n + 5, 50], block_size, "rr_src")
    dst, _, _ = _cache(dtype, hkv, dh, [30, dst_off + n], block_size, "rr_dst", fill_random=False)
    ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(dst_off + n, dh))
    rc.rc_rope_rerotate(src.layer(0), 0, src_off, dst.layer(0), 1, dst_off, n, pre_rope, old, base, ws)
    torch.cuda.synchronize()
    k_src, v_src = ks[0][src_off:src_off + n], vs[0][src_off:src_off + n]
    ang = dst_off + np.arange(n) if pre_rope else np.full(n, dst_off - old)
    want_k = R.rope_rotate(k_src, ang, base)
    got_k = to_np(dst.read("k", 0, 1, n, start=dst_off))
    got_v = to_np(dst.read("v", 0, 1, n, start=dst_off))
    assert rel_err(got_k, want_k) <= (1e-6 if dtype == "f32" else 4e-3)
    assert np.array_equal(got_v, v_src)                       # values are copied bit for bit
    # rows outside the destination range are untouched (zeros)
    assert float(dst.read("k", 0, 1, dst_off, start=0).abs().max()) == 0.0
    assert float(dst.read("k", 0, 0, 30, start=0).abs().max()) == 0.0


def test_rope_rerotate_large_positions_keep_float_accuracy():
    rc = _rc()
    n, dst_off, dh = 64, 36800, 128
    src, ks, _ = _cache("f32", 1, dh, [n], 0, "rr_big")
    dst, _, _ = _cache("f32", 1, dh, [dst_off + n], 0, "rr_big_dst", fill_random=False)
    ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(dst_off + n, dh))
    rc.rc_rope_rerotate(src.layer(0), 0, 0, dst.layer(0), 0, dst_off, n, True, 0, 1.0e6, ws)
    torch.cuda.synchronize()
    want = R.rope_rotate(ks[0], dst_off + np.arange(n), 1.0e6)
    assert rel_err(to_np(dst.read("k", 0, 0, n, start=dst_off)), want) <= 1e-6


# ------------------------------------------------------------------ K4
@pytest.mark.parametrize("dtype,hkv,dh", [("f32", 2, 64), ("bf16", 8, 128), ("f32", 5, 128), ("bf16", 3, 128)])
@pytest.mark.parametrize("block_size", [0, 16])
def test_vdev_score(dtype, hkv, dh, block_size):
    rc = _rc()
    n, off = 301, 77
    cache, _, vs = _cache(dtype, hkv, dh, [40, off + n], block_size, "sc")
    v_reuse = vs[1][off:off + n]
    fresh = v_reuse + _rand((n, hkv, dh), dtype, "sc_noise", 0.3)
    fresh[5] = v_reuse[5] * 2.0            # scaled copy -> 0
    fresh[6] = -v_reuse[6]                 # negation -> 2
    fresh[7] = 0.0                         # zero vector -> cos := 0 -> score 1
    if dtype == "bf16":
        fresh = round_to_bf16(fresh)
    score = torch.full((n,), -9.0, device="cuda")
    ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(0, dh))
    rc.rc_vdev_score(_up(fresh, dtype), cache.layer(0), 1, off, n, score, ws)
    torch.cuda.synchronize()
    want = R.vdev_score(v_reuse, fresh)
    got = score.cpu().numpy()
    assert np.max(np.abs(got - want)) <= 2e-6        # float accumulation of <= 128-term dot products
    assert abs(got[5]) <= 1e-6 and abs(got[6] - 2.0) <= 1e-6 and got[7] == 1.0


# ------------------------------------------------------------------ K5
@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 1000, 4096, 16384, 32768, 40001])
def test_topk_matches_oracle_bit_exactly(n):
    rc = _rc()
    g = stream_rng("stage", f"topk{n}")
    score = g.random(n, dtype=np.float32)
    score[g.integers(0, n, size=max(1, n // 7))] = score[0]          # many exact ties
    if n > 10:
        score[3] = -0.0; score[4] = 0.0; score[9] = -1.5e-7
    dev = torch.from_numpy(score).cuda()
    for k in sorted({0, 1, n // 7, (n * 15) // 100, n // 2, n - 1, n}):
        if k < 0 or k > n:
            continue
        out = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
        rc.rc_topk(dev, n, k, out)
        torch.cuda.synchronize()
        want = R.topk_select(score, k)
        assert np.array_equal(out.cpu().numpy()[:k], want), (n, k)


def test_topk_all_equal_and_descending_inputs():
    rc = _rc()
    n = 5000
    for arr in (np.full(n, 0.25, np.float32), np.linspace(1, 0, n, dtype=np.float32),
                np.linspace(0, 1, n, dtype=np.float32)):
        out = torch.zeros(777, dtype=torch.int32, device="cuda")
        rc.rc_topk(torch.from_numpy(arr).cuda(), n, 777, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), R.topk_select(arr, 777))


@pytest.mark.parametrize("n", [10, 1000, 33333])
def test_threshold_select(n):
    rc = _rc()
    g = stream_rng("stage", f"thr{n}")
    score = (g.random(n, dtype=np.float32) ** 4).astype(np.float32)       # sparse large values
    for tau in (1.5, 1.45, 0.0, 50.0):
        idx = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        rc.rc_threshold_select(torch.from_numpy(score).cuda(), n, tau, idx, cnt)
        torch.cuda.synchronize()
        want = R.threshold_select(score.astype(np.float64), float(np.float32(tau)))
        c = int(cnt.item())
        assert c == len(want)
        assert np.array_equal(idx.cpu().numpy()[:c], want)


@pytest.mark.parametrize("n", [1, 7, 1000, 33333])
def test_final_select(n):
    rc = _rc()
    g = stream_rng("stage", f"fin{n}")
    s_dev = (g.random(n, dtype=np.float32) ** 4).astype(np.float32)
    s_inf = np.exp(g.standard_normal(n)).astype(np.float32)
    for tau_dev, tau_inf, k_suf, use_inf in ((1.5, 1.45, 10, True), (1.5, 1.45, 0, False), (50.0, 50.0, 0, True),
                                             (1.0, 1.0, n + 5, True), (2.0, 0.5, 3, True)):
        idx = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        rc.rc_final_select(torch.from_numpy(s_dev).cuda(), torch.from_numpy(s_inf).cuda() if use_inf else None, n,
                           tau_dev, tau_inf, k_suf, idx, cnt)
        torch.cuda.synchronize()
        want = R.final_selection(s_dev.astype(np.float64), s_inf.astype(np.float64) if use_inf else None,
                                 float(np.float32(tau_dev)), float(np.float32(tau_inf)), k_suf)
        c = int(cnt.item())
        assert c == len(want)
        assert np.array_equal(idx.cpu().numpy()[:c], want)


# ------------------------------------------------------------------ K6
@pytest.mark.parametrize("dtype,hq,hkv,dh", [("f32", 4, 2, 64), ("bf16", 8, 2, 128), ("bf16", 10, 2, 128),
                                              ("bf16", 4, 4, 128), ("f32", 2, 1, 128),
                                              # every width of a query-head group the bf16 kernel is built for (1 ... 8), and
                                              # one beyond (served in passes)
                                              ("bf16", 4, 2, 128), ("bf16", 6, 2, 128), ("bf16", 12, 2, 128),
                                              ("bf16", 14, 2, 128), ("bf16", 16, 2, 128), ("bf16", 18, 2, 128)])
@pytest.mark.parametrize("block_size", [0, 16])
@pytest.mark.parametrize("split", [False, True])
def test_sparse_attention(dtype, hq, hkv, dh, block_size, split):
    rc = _rc()
    T = 333
    cache, ks, vs = _cache(dtype, hkv, dh, [20, T], block_size, "att")
    g = stream_rng("stage", "att_pos")
    pos = np.sort(np.concatenate([np.arange(0, 70), g.choice(np.arange(70, T), size=57, replace=False), [T - 1, T - 1]]))
    n = len(pos)
    q = _rand((n, hq, dh), dtype, "att_q", 0.5)
    out = torch.zeros((n, hq, dh), dtype=_td(dtype), device="cuda")
    ws = None
    if split:      # the bf16 kernel cuts long KV ranges into chunks and merges partial results
        if dtype != "bf16":
            pytest.skip("the float path has no KV split")
        rc.rc_tune_set(rc.RC_TUNE_ATTN_CHUNK_TILES, 2)     # chunks of 128 keys, so that T = 333 is "long"
        assert rc.rc_sparse_attention_workspace_bytes(n, hq, cache.layer(0)) > 0
        ws = rc.alloc_workspace(rc.rc_sparse_attention_workspace_bytes(n, hq, cache.layer(0)))
    try:
        rc.rc_sparse_attention(_up(q, dtype), torch.from_numpy(pos.astype(np.int32)).cuda(), n, hq, cache.layer(0), 1,
                               out, ws)
        torch.cuda.synchronize()
    finally:
        rc.rc_tune_set(rc.RC_TUNE_ATTN_CHUNK_TILES, 0)
    want = R.causal_gqa_attention(q.astype(np.float64), pos, ks[1].astype(np.float64), vs[1].astype(np.float64))
    assert rel_err(to_np(out), want) <= (2e-5 if dtype == "f32" else 1e-2)
    # the first query sees a single key: its output is that value row
    assert rel_err(to_np(out)[0, 0], vs[1][0, 0]) <= (1e-6 if dtype == "f32" else 4e-3)


@pytest.mark.parametrize("case", ["growing", "shrinking", "flat", "spiky"])
@pytest.mark.parametrize("split", [False, True])
def test_sparse_attention_wide_score_range(case, split):
    """Scores whose running maximum moves by far more (or less) than the slack the bf16 kernel allows before it
    rescales its running sums: logits that grow or fall along the context, identical scores, rare spikes."""
    rc = _rc()
    hq, hkv, dh, T = 8, 2, 128, 1500
    g = stream_rng("stage", f"att_range_{case}")
    k = g.standard_normal((T, hkv, dh), dtype=np.float32)
    v = g.standard_normal((T, hkv, dh), dtype=np.float32)
    ramp = np.linspace(0.05, 3.0, T, dtype=np.float32)[:, None, None]
    if case == "growing":
        k = np.abs(k) * ramp               # against an all-positive query: logits rise along the context
    elif case == "shrinking":
        k = np.abs(k) * ramp[::-1]
    elif case == "flat":
        k[:] = 0.0                         # every visible key gets the same weight: output = mean of V
    else:
        k *= 0.1
        k[g.choice(T, size=12, replace=False)] *= 60.0
    k, v = round_to_bf16(k), round_to_bf16(v)
    kv = rc.PagedKV.contiguous(1, 1, T, hkv, dh, rc.RC_BF16)
    kv.write("k", 0, 0, _up(k, "bf16"))
    kv.write("v", 0, 0, _up(v, "bf16"))
    pos = np.sort(np.concatenate([np.arange(0, 40), g.choice(np.arange(40, T), size=85, replace=False), [T - 1]]))
    n = len(pos)
    q = round_to_bf16(np.abs(g.standard_normal((n, hq, dh), dtype=np.float32)) * (1.5 if case != "spiky" else 1.0))
    out = torch.zeros((n, hq, dh), dtype=torch.bfloat16, device="cuda")
    ws = None
    if split:
        rc.rc_tune_set(rc.RC_TUNE_ATTN_CHUNK_TILES, 4)
        ws = rc.alloc_workspace(rc.rc_sparse_attention_workspace_bytes(n, hq, kv.layer(0)))
    try:
        rc.rc_sparse_attention(_up(q, "bf16"), torch.from_numpy(pos.astype(np.int32)).cuda(), n, hq, kv.layer(0), 0,
                               out, ws)
        torch.cuda.synchronize()
    finally:
        rc.rc_tune_set(rc.RC_TUNE_ATTN_CHUNK_TILES, 0)
    got = to_np(out)
    assert np.isfinite(got).all()
    want = R.causal_gqa_attention(q.astype(np.float64), pos, k.astype(np.float64), v.astype(np.float64))
    assert rel_err(got, want) <= 1e-2
    if case == "flat":
        want_mean = np.stack([v[: p + 1].astype(np.float64).mean(axis=0) for p in pos])      # [n][hkv][dh]
        assert rel_err(got, np.repeat(want_mean, hq // hkv, axis=1)) <= 1e-2


@pytest.mark.parametrize("split", [False, True])
def test_sparse_attention_over_more_blocks_than_the_lds_table_holds(split):
    """A paged cache whose sequence spans 2063 blocks of 16 tokens.  A workgroup keeps the block-table slice of its KV
    range in LDS when it has at most 2048 entries; an unsplit query tile near the end of this sequence needs more and
    looks its blocks up in global memory instead.  With a workspace the range is cut into chunks whose slices fit."""
    rc = _rc()
    hq, hkv, dh, T = 8, 2, 128, 33001
    cache, ks, vs = _cache("bf16", hkv, dh, [5, T], 16, "att_long")
    g = stream_rng("stage", "att_long_pos")
    pos = np.sort(np.concatenate([np.arange(0, 33), g.choice(np.arange(33, T), size=30, replace=False), [T - 1]]))
    n = len(pos)
    q = _rand((n, hq, dh), "bf16", "att_long_q", 0.5)
    out = torch.zeros((n, hq, dh), dtype=torch.bfloat16, device="cuda")
    ws = None
    if split:
        assert rc.rc_sparse_attention_workspace_bytes(n, hq, cache.layer(0)) > 0
        ws = rc.alloc_workspace(rc.rc_sparse_attention_workspace_bytes(n, hq, cache.layer(0)))
    rc.rc_sparse_attention(_up(q, "bf16"), torch.from_numpy(pos.astype(np.int32)).cuda(), n, hq, cache.layer(0), 1, out, ws)
    torch.cuda.synchronize()
    want = R.causal_gqa_attention(q.astype(np.float64), pos, ks[1].astype(np.float64), vs[1].astype(np.float64))
    assert rel_err(to_np(out), want) <= 1e-2


# ------------------------------------------------------------------ K3
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m,n,k", [(1, 64, 64), (51, 192, 256), (129, 1000, 688), (300, 257, 1408), (1639, 512, 1024),
                                   (700, 2100, 512),
                                   # few rows: the weight-streaming kernel of the decoding path (bf16)
                                   (1, 64, 256), (16, 1024, 512), (17, 4096, 1024), (32, 96, 14336), (5, 6144, 4096)])
@pytest.mark.parametrize("tail_split", [False, True])
def test_gemm_rows(dtype, m, n, k, tail_split):
    rc = _rc()
    a = _rand((m, k), dtype, f"ga{m}{k}")
    w = _rand((n, k), dtype, f"gw{n}{k}", 0.05)
    c = torch.zeros((m, n), dtype=torch.float32, device="cuda")
    ws = None
    if tail_split:          # the partial last round of output tiles is cut along K and summed by a fix-up kernel
        if dtype != "bf16":
            pytest.skip("only the bf16 MFMA GEMM has a K-split tail")
        ws = rc.alloc_workspace(rc.rc_gemm_workspace_bytes())
    rc.rc_gemm_rows(rc.rc_dtype_of(dtype), _up(a, dtype), _up(w, dtype), c, m, n, k, ws)
    torch.cuda.synchronize()
    want = a.astype(np.float64) @ w.astype(np.float64).T
    assert rel_err(to_np(c), want) <= 2e-6 * np.sqrt(k)


@pytest.mark.parametrize("tile", [5, 6, 7])
@pytest.mark.parametrize("epilogue", ["store", "add", "swiglu"])
@pytest.mark.parametrize("m,n,k", [(300, 258, 1408), (1639, 576, 1024), (700, 2100, 512), (2049, 6144, 256)])
def test_gemm_forced_tile_shapes(tile, epilogue, m, n, k):
    """Every direct-to-LDS tile shape of the bf16 GEMM (normally chosen per launch by a time model), with the
    K-split tail where the shape has one."""
    rc = _rc()
    a = _rand((m, k), "bf16", f"ta{m}{k}")
    w = _rand((n, k), "bf16", f"tw{n}{k}", 0.05)
    w2 = _rand((n, k), "bf16", f"tu{n}{k}", 0.05)
    ws = rc.alloc_workspace(rc.rc_gemm_workspace_bytes())
    prod = R.linear(a.astype(np.float64), w.astype(np.float64))
    rc.rc_tune_set(rc.RC_TUNE_GEMM_TILE, tile)
    try:
        if epilogue == "store":
            c = torch.zeros((m, n), dtype=torch.float32, device="cuda")
            rc.rc_gemm_rows(rc.RC_BF16, _up(a, "bf16"), _up(w, "bf16"), c, m, n, k, ws)
            want, tol = prod, 2e-6 * np.sqrt(k)
        elif epilogue == "add":
            c0 = _rand((m, n), "f32", f"tc{m}{n}")
            c = torch.from_numpy(c0).cuda()
            rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_ADD, _up(a, "bf16"), _up(w, "bf16"), None, c, m, n, k, ws)
            want, tol = c0.astype(np.float64) + prod, 2e-6 * np.sqrt(k)
        else:
            c = torch.zeros((m, n), dtype=torch.bfloat16, device="cuda")
            rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_SWIGLU, _up(a, "bf16"), _up(w, "bf16"), _up(w2, "bf16"), c,
                                  m, n, k, ws)
            want, tol = R.silu(prod) * R.linear(a.astype(np.float64), w2.astype(np.float64)), 4e-3
        torch.cuda.synchronize()
    finally:
        rc.rc_tune_set(rc.RC_TUNE_GEMM_TILE, 0)
    assert rel_err(to_np(c), want) <= tol


@pytest.mark.parametrize("epilogue", ["store", "add", "swiglu"])
@pytest.mark.parametrize("m", [1025, 1057, 1088, 1089, 1153, 1639])
def test_gemm_ragged_last_tile_row(epilogue, m):
    """Launches with at least one full round of 256x256 tiles whose last tile row has 1 ... 129 live rows: up to
    64 of them are multiplied by the thin tile body, more by the full body."""
    rc = _rc()
    k = 256
    n = 8192 if epilogue == "swiglu" else (16384 if epilogue == "store" else 16344)    # 16344: ragged last tile column
    a = _rand((m, k), "bf16", f"ra{m}")
    w = _rand((n, k), "bf16", f"rw{n}", 0.05)
    ws = rc.alloc_workspace(rc.rc_gemm_workspace_bytes())
    prod = R.linear(a.astype(np.float64), w.astype(np.float64))
    if epilogue == "store":
        c = torch.full((m, n), 7.0, dtype=torch.float32, device="cuda")
        rc.rc_gemm_rows(rc.RC_BF16, _up(a, "bf16"), _up(w, "bf16"), c, m, n, k, ws)
        want, tol = prod, 2e-6 * np.sqrt(k)
    elif epilogue == "add":
        c0 = _rand((m, n), "f32", f"rc{m}")
        c = torch.from_numpy(c0).cuda()
        rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_ADD, _up(a, "bf16"), _up(w, "bf16"), None, c, m, n, k, ws)
        want, tol = c0.astype(np.float64) + prod, 2e-6 * np.sqrt(k)
    else:
        w2 = _rand((n, k), "bf16", f"ru{n}", 0.05)
        c = torch.zeros((m, n), dtype=torch.bfloat16, device="cuda")
        rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_SWIGLU, _up(a, "bf16"), _up(w, "bf16"), _up(w2, "bf16"), c, m, n, k,
                              ws)
        want, tol = R.silu(prod) * R.linear(a.astype(np.float64), w2.astype(np.float64)), 4e-3
    torch.cuda.synchronize()
    assert rel_err(to_np(c), want) <= tol
    if epilogue == "store":     # without a workspace: no K-split tail, every tile is done by one workgroup
        c1 = torch.zeros_like(c)
        rc.rc_gemm_rows(rc.RC_BF16, _up(a, "bf16"), _up(w, "bf16"), c1, m, n, k, None)
        torch.cuda.synchronize()
        assert rel_err(to_np(c1), want) <= tol
    # the same launch with the thin bodies switched off (only the K-split tail may fall on other tiles)
    rc.rc_tune_set(rc.RC_TUNE_GEMM_THIN_TILES, 0)
    try:
        if epilogue == "store":
            c2 = torch.zeros_like(c)
            rc.rc_gemm_rows(rc.RC_BF16, _up(a, "bf16"), _up(w, "bf16"), c2, m, n, k, ws)
        elif epilogue == "add":
            c2 = torch.from_numpy(c0).cuda()
            rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_ADD, _up(a, "bf16"), _up(w, "bf16"), None, c2, m, n, k, ws)
        else:
            c2 = torch.zeros_like(c)
            rc.rc_gemm_rows_fused(rc.RC_BF16, rc.RC_GEMM_SWIGLU, _up(a, "bf16"), _up(w, "bf16"), _up(w2, "bf16"), c2, m, n,
                                  k, ws)
        torch.cuda.synchronize()
    finally:
        rc.rc_tune_set(rc.RC_TUNE_GEMM_THIN_TILES, 1)
    assert rel_err(to_np(c), to_np(c2)) <= (1e-6 if epilogue != "swiglu" else 8e-3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("epilogue", ["store_t", "add", "swiglu"])
@pytest.mark.parametrize("m,n,k", [(51, 192, 256), (129, 1000, 688), (300, 258, 1408), (1639, 512, 1024),
                                   (700, 2100, 512), (17, 4096, 1024)])
def test_gemm_rows_fused(dtype, epilogue, m, n, k):
    """The epilogues the layer applies in place: type-T store, residual add, SwiGLU of a gate/up pair."""
    rc = _rc()
    a = _rand((m, k), dtype, f"fa{m}{k}")
    w = _rand((n, k), dtype, f"fw{n}{k}", 0.05)
    w2 = _rand((n, k), dtype, f"fu{n}{k}", 0.05)
    ws = rc.alloc_workspace(rc.rc_gemm_workspace_bytes()) if dtype == "bf16" else None
    t = rc.rc_dtype_of(dtype)
    prod = R.linear(a.astype(np.float64), w.astype(np.float64))
    if epilogue == "add":
        c0 = _rand((m, n), "f32", f"fc{m}{n}")
        c = torch.from_numpy(c0).cuda()
        rc.rc_gemm_rows_fused(t, rc.RC_GEMM_ADD, _up(a, dtype), _up(w, dtype), None, c, m, n, k, ws)
        want, tol = c0.astype(np.float64) + prod, 2e-6 * np.sqrt(k)
    elif epilogue == "store_t":
        c = torch.zeros((m, n), dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
        rc.rc_gemm_rows_fused(t, rc.RC_GEMM_STORE_T, _up(a, dtype), _up(w, dtype), None, c, m, n, k, ws)
        want, tol = prod, (2e-6 * np.sqrt(k) if dtype == "f32" else 4e-3)
    else:
        c = torch.zeros((m, n), dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
        rc.rc_gemm_rows_fused(t, rc.RC_GEMM_SWIGLU, _up(a, dtype), _up(w, dtype), _up(w2, dtype), c, m, n, k, ws)
        want = R.silu(prod) * R.linear(a.astype(np.float64), w2.astype(np.float64))
        tol = 4e-6 * np.sqrt(k) if dtype == "f32" else 4e-3     # bf16: one rounding of the stored product
    torch.cuda.synchronize()
    assert rel_err(to_np(c), want) <= tol


# ------------------------------------------------------------------ K7
@pytest.mark.parametrize("dtype,hkv,dh", [("f32", 2, 64), ("bf16", 8, 128)])
@pytest.mark.parametrize("block_size", [0, 16])
def test_scatter_paged(dtype, hkv, dh, block_size):
    rc = _rc()
    T = 500
    cache, ks, vs = _cache(dtype, hkv, dh, [T, 33], block_size, "scat")
    g = stream_rng("stage", "scat_pos")
    pos = np.sort(g.choice(T, size=75, replace=False)).astype(np.int32)
    kr = _rand((75, hkv, dh), dtype, "scat_k")
    vr = _rand((75, hkv, dh), dtype, "scat_v")
    rc.rc_scatter_paged(_up(kr, dtype), _up(vr, dtype), torch.from_numpy(pos).cuda(), 75, cache.layer(0), 0)
    torch.cuda.synchronize()
    want_k, want_v = ks[0].copy(), vs[0].copy()
    want_k[pos], want_v[pos] = kr, vr
    assert np.array_equal(to_np(cache.read("k", 0, 0, T)), want_k)
    assert np.array_equal(to_np(cache.read("v", 0, 0, T)), want_v)
    assert np.array_equal(to_np(cache.read("k", 0, 1, 33)), ks[1])     # other sequences untouched


@pytest.mark.parametrize("dtype,hq,hkv,dh", [("f32", 4, 2, 64), ("bf16", 32, 8, 128), ("bf16", 10, 2, 128)])
@pytest.mark.parametrize("block_size", [0, 16])
def test_rope_scatter_of_the_hot_path(dtype, hq, hkv, dh, block_size):
    """The kernel rc_reuse runs between the q|k|v projection and attention, through its own stage call: rotary on
    queries and keys at scattered positions, fresh K/V rows written into the paged cache."""
    rc = _rc()
    T, n = 700, 131
    base = 10000.0 if dtype == "f32" else 1.0e6
    cache, ks, vs = _cache(dtype, hkv, dh, [T, 40], block_size, "rs")
    g = stream_rng("stage", "rs_pos")
    pos = np.sort(g.choice(T, size=n, replace=False)).astype(np.int32)
    nq, nkv = hq * dh, hkv * dh
    qkv = stream_rng("stage", "rs_qkv").standard_normal((n, nq + 2 * nkv), dtype=np.float32)
    q_out = torch.zeros((n, hq, dh), dtype=_td(dtype), device="cuda")
    ws = rc.alloc_workspace(rc.rc_rope_scatter_workspace_bytes(n, cache.layer(0)))
    rc.rc_rope_scatter(torch.from_numpy(qkv).cuda(), torch.from_numpy(pos).cuda(), n, hq, base, cache.layer(0), 0, q_out, ws)
    torch.cuda.synchronize()
    q_want = R.rope_rotate(qkv[:, :nq].reshape(n, hq, dh), pos, base)
    k_want = R.rope_rotate(qkv[:, nq:nq + nkv].reshape(n, hkv, dh), pos, base)
    v_want = qkv[:, nq + nkv:].reshape(n, hkv, dh)
    tol = 1e-6 if dtype == "f32" else 4e-3                   # one rounding to bf16
    assert rel_err(to_np(q_out), q_want) <= tol
    got_k, got_v = to_np(cache.read("k", 0, 0, T)), to_np(cache.read("v", 0, 0, T))
    assert rel_err(got_k[pos], k_want) <= tol and rel_err(got_v[pos], v_want) <= tol
    rest = np.setdiff1d(np.arange(T), pos)
    assert np.array_equal(got_k[rest], ks[0][rest]) and np.array_equal(got_v[rest], vs[0][rest])   # other rows untouched
    assert np.array_equal(to_np(cache.read("k", 0, 1, 40)), ks[1])


# ------------------------------------------------------------------ machine ceilings (benchmark report helpers)
def test_ceiling_kernels_run_and_copy_is_exact():
    rc = _rc()
    g = stream_rng("stage", "ceil")
    n = (1 << 22) + 16 * 37
    src = torch.from_numpy(g.integers(0, 256, size=n, dtype=np.uint8)).cuda()
    dst = torch.zeros_like(src)
    rc.rc_ceiling_stream_copy(src, dst, n)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    out = torch.zeros(rc.rc_ceiling_mfma_loop_out_bytes(4) // 4, dtype=torch.float32, device="cuda")
    flops = rc.rc_ceiling_mfma_loop(out, 4, 10)
    torch.cuda.synchronize()
    assert flops == 4 * 8 * 10 * 32 * 2 * 16 * 16 * 32
    assert torch.isfinite(out).all() and float(out.abs().max()) > 0.0
