"""The allocation-free re-rotation entry point against the one that takes a caller's workspace.

rc_rope_rerotate_static keeps its scratch (request table, rotary tables) in a device array of the library;
both entry points launch the same kernels, so keys must agree bit for bit and values are copied unchanged.
Two calls in a row share the array; the second is smaller, so stale table entries of the first lie behind
the ones it uses.
"""
import numpy as np
import pytest
import torch

from synth import make_block_table, round_to_bf16, stream_rng

pytestmark = pytest.mark.gpu


def _cache(rc, dtype, hkv, dh, lens, block_size, name, fill=True):
    dt = rc.rc_dtype_of(dtype)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    if block_size:
        tab, nb = make_block_table(lens, block_size, seed=23)
        kv = rc.PagedKV(1, nb, block_size, hkv, dh, dt, tab)
    else:
        kv = rc.PagedKV.contiguous(1, len(lens), max(lens), hkv, dh, dt)
    if fill:
        for s, n in enumerate(lens):
            for which in ("k", "v"):
                x = stream_rng("no_alloc", f"{name}{which}{s}").standard_normal((n, hkv, dh), dtype=np.float32)
                if dtype == "bf16":
                    x = round_to_bf16(x)
                kv.write(which, 0, s, torch.from_numpy(x).cuda().to(td).contiguous())
    return kv


@pytest.mark.parametrize("dtype,hkv,dh,block_size", [("bf16", 8, 128, 16), ("f32", 2, 64, 0)])
@pytest.mark.parametrize("pre_rope", [True, False])
def test_static_scratch_rerotate_equals_workspace_rerotate(dtype, hkv, dh, block_size, pre_rope):
    from paper_2603_13289_amd import binding as rc
    base = 1.0e6 if dtype == "bf16" else 1.0e4
    # (tokens, source offset, destination offset, old start position): a larger call, then a smaller one
    calls = [(1500, 40, 700, 40), (203, 37, 129, 21)]
    src = _cache(rc, dtype, hkv, dh, [max(o + n for n, o, _, _ in calls) + 3, 64], block_size, "src")
    for n, src_off, dst_off, old in calls:
        dst_ws = _cache(rc, dtype, hkv, dh, [30, dst_off + n + 5], block_size, "dst", fill=False)
        dst_st = _cache(rc, dtype, hkv, dh, [30, dst_off + n + 5], block_size, "dst", fill=False)
        ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(dst_off + n, dh))
        rc.rc_rope_rerotate(src.layer(0), 0, src_off, dst_ws.layer(0), 1, dst_off, n, pre_rope, old, base, ws)
        rc.rc_rope_rerotate_static(src.layer(0), 0, src_off, dst_st.layer(0), 1, dst_off, n, pre_rope, old, base)
        torch.cuda.synchronize()
        for which in ("k", "v"):
            a = dst_ws.read(which, 0, 1, dst_off + n + 5)
            b = dst_st.read(which, 0, 1, dst_off + n + 5)
            assert torch.equal(a, b), (which, n)
        assert float(dst_st.read("k", 0, 1, n, start=dst_off).float().abs().max()) > 0.0
        assert float(dst_st.read("k", 0, 1, dst_off, start=0).float().abs().max()) == 0.0   # rows before: untouched


def test_static_scratch_rejects_sizes_beyond_its_limit():
    from paper_2603_13289_amd import binding as rc
    limit = rc.RC_REROTATE_STATIC_MAX_POSITIONS
    n = 64
    src = _cache(rc, "f32", 1, 64, [n], 0, "lim_src")
    dst = _cache(rc, "f32", 1, 64, [limit + n], 0, "lim_dst", fill=False)
    with pytest.raises(rc.RcError) as e:
        rc.rc_rope_rerotate_static(src.layer(0), 0, 0, dst.layer(0), 0, limit - n + 1, n, True, 0, 1.0e4)
    assert e.value.status == rc.RC_E_CAPACITY
    torch.cuda.synchronize()
    assert float(dst.read("k", 0, 0, limit + n).abs().max()) == 0.0        # nothing was launched
    # the largest size it takes
    rc.rc_rope_rerotate_static(src.layer(0), 0, 0, dst.layer(0), 0, limit - n, n, True, 0, 1.0e4)
    ws = rc.alloc_workspace(rc.rc_stage_workspace_bytes(limit, 64))
    dst2 = _cache(rc, "f32", 1, 64, [limit + n], 0, "lim_dst", fill=False)
    rc.rc_rope_rerotate(src.layer(0), 0, 0, dst2.layer(0), 0, limit - n, n, True, 0, 1.0e4, ws)
    torch.cuda.synchronize()
    assert torch.equal(dst.read("k", 0, 0, limit + n), dst2.read("k", 0, 0, limit + n))
    assert rc.rc_rope_rerotate_static_scratch_bytes() <= 17 << 20
