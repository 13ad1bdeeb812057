"""ctypes binding of librelaycache.so: argument marshalling only.

Function names match the C ABI in include/relaycache.h.  PyTorch is used for
device memory and streams; every step of the method runs inside the library's
HIP kernels.  There is no CPU fallback: if the shared library is missing the
import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librelaycache.so")

RC_OK, RC_E_INVALID_ARG, RC_E_UNSUPPORTED, RC_E_WORKSPACE, RC_E_HIP, RC_E_CAPACITY = 0, -1, -2, -3, -4, -5
RC_F32, RC_BF16 = 0, 1
RC_MAX_REQ = 32
RC_SELECT_BUDGET, RC_SELECT_THRESHOLD = 0, 1

EXPORTS = [
    "rc_status_str", "rc_build_info", "rc_model_create", "rc_model_destroy", "rc_reuse_workspace_bytes",
    "rc_reuse", "rc_prefill_workspace_bytes", "rc_prefill", "rc_decode_workspace_bytes", "rc_decode_step", "rc_layer_profile", "rc_stage_workspace_bytes", "rc_rope_rerotate",
    "rc_vdev_score", "rc_topk", "rc_threshold_select", "rc_final_select", "rc_sparse_attention", "rc_gemm_rows", "rc_gemm_rows_fused", "rc_ceiling_stream_copy",
    "rc_ceiling_mfma_loop_out_bytes", "rc_ceiling_mfma_loop", "rc_gemm_plan_check",
    "rc_scatter_paged", "rc_profile_enable", "rc_profile_class_count", "rc_profile_class_name", "rc_profile_read",
    "rc_tune_set", "rc_sparse_attention_workspace_bytes",
    "rc_gemm_workspace_bytes", "rc_rope_rerotate_static", "rc_rope_rerotate_static_scratch_bytes",
    "rc_rope_scatter", "rc_rope_scatter_workspace_bytes",
]


class RcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} ({status})")


# ------------------------------------------------------------------ C structs
class rc_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class rc_layer_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_ffn")]


class rc_paged_kv(C.Structure):
    _fields_ = [("k_pool", C.POINTER(C.c_void_p)), ("v_pool", C.POINTER(C.c_void_p)), ("n_blocks", C.c_int32),
                ("block_size", C.c_int32), ("block_table", C.c_void_p), ("n_seq", C.c_int32),
                ("max_blocks_per_seq", C.c_int32)]


class rc_kv_layer(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("n_blocks", C.c_int32), ("block_size", C.c_int32),
                ("block_table", C.c_void_p), ("n_seq", C.c_int32), ("max_blocks_per_seq", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32)]


class rc_request(C.Structure):
    _fields_ = [("n_prefix", C.c_int32), ("x_prefix", C.c_void_p), ("n_seg", C.c_int32), ("h_start", C.c_void_p),
                ("n_suffix", C.c_int32), ("x_suffix", C.c_void_p), ("src_seq", C.c_int32), ("src_offset", C.c_int32),
                ("k_is_pre_rope", C.c_int32), ("seg_old_start_pos", C.c_int32), ("dst_seq", C.c_int32),
                ("s_inf", C.c_void_p), ("n_cached", C.c_int32), ("no_logits", C.c_int32)]


class rc_decode_req(C.Structure):
    _fields_ = [("x", C.c_void_p), ("pos", C.c_int32), ("seq", C.c_int32), ("h_capture", C.c_void_p),
                ("s_inf", C.c_void_p)]


class rc_layer_profile_params(C.Structure):
    _fields_ = [("tau_st", C.c_float), ("tail", C.c_int32), ("lam", C.c_float), ("consecutive", C.c_int32)]


class rc_layer_triple(C.Structure):
    _fields_ = [("l_start", C.c_int32), ("l_det", C.c_int32), ("l_end", C.c_int32)]


class rc_plan(C.Structure):
    _fields_ = [("l_start", C.c_int32), ("l_det", C.c_int32), ("l_end", C.c_int32),
                ("k_per_req", C.POINTER(C.c_int32)), ("forced_idx", C.c_void_p),
                ("selector", C.c_int32), ("tau_dev", C.c_float), ("tau_inf", C.c_float), ("k_suf", C.c_int32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_13289_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.rc_status_str.restype = C.c_char_p
    lib.rc_status_str.argtypes = [C.c_int]
    lib.rc_build_info.restype = C.c_char_p
    lib.rc_build_info.argtypes = []
    lib.rc_model_create.restype = C.c_int
    lib.rc_model_create.argtypes = [C.POINTER(rc_model_desc), C.POINTER(rc_layer_w), vp, vp, C.POINTER(vp)]
    lib.rc_model_destroy.restype = C.c_int
    lib.rc_model_destroy.argtypes = [vp]
    lib.rc_reuse_workspace_bytes.restype = sz
    lib.rc_reuse_workspace_bytes.argtypes = [vp, C.POINTER(rc_request), i32, C.POINTER(rc_plan)]
    lib.rc_reuse.restype = C.c_int
    lib.rc_reuse.argtypes = [vp, C.POINTER(rc_request), i32, C.POINTER(rc_plan), C.POINTER(rc_paged_kv),
                             C.POINTER(rc_paged_kv), vp, vp, vp, vp, vp, sz, vp]
    lib.rc_decode_workspace_bytes.restype = sz
    lib.rc_decode_workspace_bytes.argtypes = [vp, C.POINTER(rc_decode_req), i32]
    lib.rc_decode_step.restype = C.c_int
    lib.rc_decode_step.argtypes = [vp, C.POINTER(rc_decode_req), i32, C.POINTER(rc_paged_kv), C.POINTER(vp), i32, vp,
                                   vp, sz, vp]
    lib.rc_layer_profile.restype = C.c_int
    lib.rc_layer_profile.argtypes = [vp, i32, i32, C.POINTER(rc_layer_profile_params), C.POINTER(rc_layer_triple), vp, vp]
    lib.rc_prefill_workspace_bytes.restype = sz
    lib.rc_prefill_workspace_bytes.argtypes = [vp, C.POINTER(i32), i32]
    lib.rc_prefill.restype = C.c_int
    lib.rc_prefill.argtypes = [vp, C.POINTER(vp), C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(rc_paged_kv),
                               C.POINTER(vp), i32, C.POINTER(vp), vp, vp, sz, vp]
    lib.rc_stage_workspace_bytes.restype = sz
    lib.rc_stage_workspace_bytes.argtypes = [i32, i32]
    lib.rc_rope_rerotate.restype = C.c_int
    lib.rc_rope_rerotate.argtypes = [C.POINTER(rc_kv_layer), i32, i32, C.POINTER(rc_kv_layer), i32, i32, i32, i32,
                                     i32, C.c_float, vp, sz, vp]
    lib.rc_rope_rerotate_static.restype = C.c_int
    lib.rc_rope_rerotate_static.argtypes = [C.POINTER(rc_kv_layer), i32, i32, C.POINTER(rc_kv_layer), i32, i32, i32,
                                            i32, i32, C.c_float, vp]
    lib.rc_rope_rerotate_static_scratch_bytes.restype = sz
    lib.rc_rope_rerotate_static_scratch_bytes.argtypes = []
    lib.rc_rope_scatter_workspace_bytes.restype = sz
    lib.rc_rope_scatter_workspace_bytes.argtypes = [i32, C.POINTER(rc_kv_layer)]
    lib.rc_rope_scatter.restype = C.c_int
    lib.rc_rope_scatter.argtypes = [vp, vp, i32, i32, C.c_float, C.POINTER(rc_kv_layer), i32, vp, vp, sz, vp]
    lib.rc_vdev_score.restype = C.c_int
    lib.rc_vdev_score.argtypes = [vp, C.POINTER(rc_kv_layer), i32, i32, i32, vp, vp, sz, vp]
    lib.rc_topk.restype = C.c_int
    lib.rc_topk.argtypes = [vp, i32, i32, vp, vp]
    lib.rc_threshold_select.restype = C.c_int
    lib.rc_threshold_select.argtypes = [vp, i32, C.c_float, vp, vp, vp]
    lib.rc_final_select.restype = C.c_int
    lib.rc_final_select.argtypes = [vp, vp, i32, C.c_float, C.c_float, i32, vp, vp, vp]
    lib.rc_sparse_attention.restype = C.c_int
    lib.rc_sparse_attention.argtypes = [vp, vp, i32, i32, C.POINTER(rc_kv_layer), i32, vp, vp, sz, vp]
    lib.rc_sparse_attention_workspace_bytes.restype = sz
    lib.rc_sparse_attention_workspace_bytes.argtypes = [i32, i32, C.POINTER(rc_kv_layer)]
    lib.rc_gemm_rows.restype = C.c_int
    lib.rc_gemm_rows.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp, sz, vp]
    lib.rc_gemm_plan_check.restype = i32
    lib.rc_gemm_plan_check.argtypes = [i32, i32, i32, i32, i32, i32, i32, C.POINTER(i32)]
    lib.rc_ceiling_stream_copy.restype = C.c_int
    lib.rc_ceiling_stream_copy.argtypes = [vp, vp, sz, vp]
    lib.rc_ceiling_mfma_loop_out_bytes.restype = sz
    lib.rc_ceiling_mfma_loop_out_bytes.argtypes = [i32]
    lib.rc_ceiling_mfma_loop.restype = C.c_int
    lib.rc_ceiling_mfma_loop.argtypes = [vp, i32, i32, C.POINTER(C.c_double), vp]
    lib.rc_gemm_rows_fused.restype = C.c_int
    lib.rc_gemm_rows_fused.argtypes = [i32, i32, vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]
    lib.rc_gemm_workspace_bytes.restype = sz
    lib.rc_gemm_workspace_bytes.argtypes = []
    lib.rc_scatter_paged.restype = C.c_int
    lib.rc_scatter_paged.argtypes = [vp, vp, vp, i32, C.POINTER(rc_kv_layer), i32, vp]
    lib.rc_tune_set.restype = C.c_int
    lib.rc_tune_set.argtypes = [i32, i32]
    lib.rc_profile_enable.restype = C.c_int
    lib.rc_profile_enable.argtypes = [i32]
    lib.rc_profile_class_count.restype = i32
    lib.rc_profile_class_count.argtypes = []
    lib.rc_profile_class_name.restype = C.c_char_p
    lib.rc_profile_class_name.argtypes = [i32]
    lib.rc_profile_read.restype = C.c_int
    lib.rc_profile_read.argtypes = [C.POINTER(C.c_float), C.POINTER(i32)]
    return lib


lib = _load()


def status_str(status: int) -> str:
    return lib.rc_status_str(status).decode()


def build_info() -> str:
    return lib.rc_build_info().decode()


def _check(status: int, where: str) -> None:
    if status != RC_OK:
        raise RcError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        if not torch.cuda.is_available():
            return None          # host-side argument checks need no stream
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def torch_dtype(dtype: int) -> torch.dtype:
    return torch.bfloat16 if dtype == RC_BF16 else torch.float32


def rc_dtype_of(name: str) -> int:
    return RC_BF16 if name in ("bf16", "bfloat16") else RC_F32


# ------------------------------------------------------------------ model
class Model:
    """rc_model handle plus the tensors it points into (kept alive here)."""

    def __init__(self, shape, layers: Sequence[dict], g_final: torch.Tensor, w_lm: torch.Tensor):
        self.shape = shape
        self.dtype = rc_dtype_of(shape.dtype)
        self._keep = (layers, g_final, w_lm)
        desc = rc_model_desc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                             shape.d_ffn, shape.vocab, float(shape.rope_base), float(shape.rms_eps), self.dtype)
        arr = (rc_layer_w * len(layers))()
        for i, lw in enumerate(layers):
            for name, _ in rc_layer_w._fields_:
                setattr(arr[i], name, _ptr(lw[name]))
        handle = C.c_void_p()
        _check(lib.rc_model_create(C.byref(desc), arr, _ptr(g_final), _ptr(w_lm), C.byref(handle)), "rc_model_create")
        self.handle = handle

    def close(self) -> None:
        if self.handle:
            lib.rc_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rc_model_create(shape, weights: dict, device="cuda") -> Model:
    """weights: {"layers": [...], "g_final", "w_lm"} of numpy float32 or torch tensors ([out][in])."""
    td = torch_dtype(rc_dtype_of(shape.dtype))

    def dev(x):
        t = x if isinstance(x, torch.Tensor) else torch.from_numpy(x)
        return t.to(device=device, dtype=td).contiguous()

    layers = [{k: dev(v) for k, v in lw.items()} for lw in weights["layers"]]
    return Model(shape, layers, dev(weights["g_final"]), dev(weights["w_lm"]))


# ------------------------------------------------------------------ paged cache
class PagedKV:
    """Per-layer K/V pools [n_blocks][Hkv][block_size][dh] plus a block table, on the device."""

    def __init__(self, n_layers: int, n_blocks: int, block_size: int, n_kv_heads: int, head_dim: int, dtype: int,
                 block_table, device="cuda", fill: Optional[float] = None):
        td = torch_dtype(dtype)
        self.n_layers, self.n_blocks, self.block_size = n_layers, n_blocks, block_size
        self.n_kv_heads, self.head_dim, self.dtype = n_kv_heads, head_dim, dtype
        shape = (n_blocks, n_kv_heads, block_size, head_dim)
        mk = (lambda: torch.zeros(shape, dtype=td, device=device)) if fill is None else \
             (lambda: torch.full(shape, fill, dtype=td, device=device))
        self.k = [mk() for _ in range(n_layers)]
        self.v = [mk() for _ in range(n_layers)]
        self.block_table = torch.as_tensor(block_table, dtype=torch.int32).to(device).contiguous()
        assert self.block_table.dim() == 2
        self.n_seq, self.max_blocks = self.block_table.shape
        self._kp = (C.c_void_p * n_layers)(*[t.data_ptr() for t in self.k])
        self._vp = (C.c_void_p * n_layers)(*[t.data_ptr() for t in self.v])
        self.c = rc_paged_kv(C.cast(self._kp, C.POINTER(C.c_void_p)), C.cast(self._vp, C.POINTER(C.c_void_p)),
                             n_blocks, block_size, self.block_table.data_ptr(), self.n_seq, self.max_blocks)

    @staticmethod
    def contiguous(n_layers, n_seq, max_len, n_kv_heads, head_dim, dtype, device="cuda", fill=None) -> "PagedKV":
        table = [[s] for s in range(n_seq)]
        return PagedKV(n_layers, n_seq, max_len, n_kv_heads, head_dim, dtype, table, device, fill)

    @staticmethod
    def from_pools(k: List[torch.Tensor], v: List[torch.Tensor], block_table: torch.Tensor, dtype: int) -> "PagedKV":
        """A cache made of existing per-layer pools (e.g. one run's pre-RoPE keys with its values)."""
        self = PagedKV.__new__(PagedKV)
        self.n_layers = len(k)
        self.n_blocks, self.n_kv_heads, self.block_size, self.head_dim = k[0].shape
        self.dtype, self.k, self.v, self.block_table = dtype, list(k), list(v), block_table
        self.n_seq, self.max_blocks = block_table.shape
        self._kp = (C.c_void_p * self.n_layers)(*[t.data_ptr() for t in self.k])
        self._vp = (C.c_void_p * self.n_layers)(*[t.data_ptr() for t in self.v])
        self.c = rc_paged_kv(C.cast(self._kp, C.POINTER(C.c_void_p)), C.cast(self._vp, C.POINTER(C.c_void_p)),
                             self.n_blocks, self.block_size, block_table.data_ptr(), self.n_seq, self.max_blocks)
        return self

    def layer(self, l: int) -> rc_kv_layer:
        return rc_kv_layer(self.k[l].data_ptr(), self.v[l].data_ptr(), self.n_blocks, self.block_size,
                           self.block_table.data_ptr(), self.n_seq, self.max_blocks, self.n_kv_heads,
                           self.head_dim, self.dtype)

    def _index(self, seq: int, n: int, start: int = 0):
        if not (0 <= seq < self.n_seq and start >= 0 and start + n <= self.max_blocks * self.block_size):
            raise IndexError(f"rows {start}..{start + n - 1} of sequence {seq} are outside the cache "
                             f"({self.n_seq} sequences of {self.max_blocks * self.block_size} rows)")
        pos = torch.arange(start, start + n, device=self.block_table.device)
        blk = self.block_table[seq][pos // self.block_size].long()
        return blk, pos % self.block_size

    def read(self, which: str, l: int, seq: int, n: int, start: int = 0) -> torch.Tensor:
        """Rows start..start+n-1 of a sequence as [n][Hkv][dh] (a gather done by torch, for tests)."""
        pool = (self.k if which == "k" else self.v)[l]
        blk, slot = self._index(seq, n, start)
        return pool[blk, :, slot, :]

    def write(self, which: str, l: int, seq: int, rows: torch.Tensor, start: int = 0) -> None:
        pool = (self.k if which == "k" else self.v)[l]
        blk, slot = self._index(seq, rows.shape[0], start)
        pool[blk, :, slot, :] = rows.to(pool.dtype)


# ------------------------------------------------------------------ the hot path
@dataclass
class Request:
    x_prefix: Optional[torch.Tensor]          # [P][d]
    h_start: Optional[torch.Tensor]           # [S][d]
    x_suffix: Optional[torch.Tensor] = None   # [n_suffix][d]
    src_seq: int = 0
    src_offset: int = 0
    k_is_pre_rope: bool = True
    seg_old_start_pos: int = 0
    dst_seq: int = 0
    s_inf: Optional[torch.Tensor] = None      # [S] float32 influence scores (threshold selector only)
    n_cached: int = 0                         # rows of dst_seq an earlier call already finished
    no_logits: bool = False                   # not the last piece of a multi-segment prompt

    def c(self) -> rc_request:
        n = lambda t: 0 if t is None else int(t.shape[0])
        return rc_request(n(self.x_prefix), _ptr(self.x_prefix), n(self.h_start), _ptr(self.h_start),
                          n(self.x_suffix), _ptr(self.x_suffix), self.src_seq, self.src_offset,
                          1 if self.k_is_pre_rope else 0, self.seg_old_start_pos, self.dst_seq, _ptr(self.s_inf), self.n_cached,
                          1 if self.no_logits else 0)


@dataclass
class Plan:
    l_start: int
    l_det: int
    l_end: int
    k_per_req: Optional[List[int]]                # budget selector; None with the threshold selector
    forced_idx: Optional[torch.Tensor] = None     # int32 device, concatenated
    selector: int = RC_SELECT_BUDGET
    tau_dev: float = 1.5
    tau_inf: float = 1.45
    k_suf: int = 10

    def c(self):
        ks = None
        if self.k_per_req is not None:
            ks = (C.c_int32 * len(self.k_per_req))(*self.k_per_req)
        return rc_plan(self.l_start, self.l_det, self.l_end,
                       C.cast(ks, C.POINTER(C.c_int32)) if ks is not None else None,
                       _ptr(self.forced_idx), self.selector, self.tau_dev, self.tau_inf, self.k_suf), ks


def _req_array(reqs: Sequence[Request]):
    arr = (rc_request * len(reqs))()
    for i, r in enumerate(reqs):
        arr[i] = r.c()
    return arr


def rc_reuse_workspace_bytes(model: Model, reqs: Sequence[Request], plan: Plan) -> int:
    cplan, _keep = plan.c()
    return int(lib.rc_reuse_workspace_bytes(model.handle, _req_array(reqs), len(reqs), C.byref(cplan)))


def rc_reuse(model: Model, reqs: Sequence[Request], plan: Plan, src: Optional[PagedKV], dst: PagedKV,
             logits: torch.Tensor, sel_idx: Optional[torch.Tensor], scores: Optional[torch.Tensor],
             workspace: torch.Tensor, stream=None, sel_cnt: Optional[torch.Tensor] = None) -> None:
    cplan, _keep = plan.c()
    st = lib.rc_reuse(model.handle, _req_array(reqs), len(reqs), C.byref(cplan),
                      C.byref(src.c) if src is not None else None, C.byref(dst.c), _ptr(logits), _ptr(sel_idx),
                      _ptr(sel_cnt), _ptr(scores), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rc_reuse")


def rc_prefill_workspace_bytes(model: Model, n_tokens: Sequence[int]) -> int:
    arr = (C.c_int32 * len(n_tokens))(*n_tokens)
    return int(lib.rc_prefill_workspace_bytes(model.handle, arr, len(n_tokens)))


def rc_prefill(model: Model, x: Sequence[torch.Tensor], dst_seq: Sequence[int], dst: PagedKV,
               logits: torch.Tensor, workspace: torch.Tensor, k_pre: Optional[PagedKV] = None,
               capture_layer: int = -1, h_capture: Optional[Sequence[torch.Tensor]] = None, stream=None) -> None:
    n = len(x)
    xs = (C.c_void_p * n)(*[_ptr(t) for t in x])
    nt = (C.c_int32 * n)(*[int(t.shape[0]) for t in x])
    ds = (C.c_int32 * n)(*dst_seq)
    hc = None if h_capture is None else (C.c_void_p * n)(*[_ptr(t) for t in h_capture])
    st = lib.rc_prefill(model.handle, xs, nt, ds, n, C.byref(dst.c), k_pre.c.k_pool if k_pre is not None else None,
                        capture_layer, hc, _ptr(logits), _ptr(workspace),
                        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rc_prefill")


@dataclass
class DecodeReq:
    x: torch.Tensor                            # [d]
    pos: int
    seq: int = 0
    h_capture: Optional[torch.Tensor] = None   # [d]
    s_inf: Optional[torch.Tensor] = None       # float32 [>= pos + 1]


def _decode_array(reqs: Sequence[DecodeReq]):
    arr = (rc_decode_req * len(reqs))()
    for i, r in enumerate(reqs):
        arr[i] = rc_decode_req(_ptr(r.x), r.pos, r.seq, _ptr(r.h_capture), _ptr(r.s_inf))
    return arr


def rc_decode_workspace_bytes(model: Model, reqs: Sequence[DecodeReq]) -> int:
    return int(lib.rc_decode_workspace_bytes(model.handle, _decode_array(reqs), len(reqs)))


def rc_decode_step(model: Model, reqs: Sequence[DecodeReq], cache: PagedKV, logits: torch.Tensor,
                   workspace: torch.Tensor, k_pre: Optional[PagedKV] = None, capture_layer: int = -1,
                   stream=None) -> None:
    st = lib.rc_decode_step(model.handle, _decode_array(reqs), len(reqs), C.byref(cache.c),
                            k_pre.c.k_pool if k_pre is not None else None, capture_layer, _ptr(logits),
                            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rc_decode_step")


def rc_layer_profile(d, tau_st: float = 0.99, tail: int = 5, lam: float = 2.0, consecutive: int = 2):
    """d: host float32 array [n_layers][n_tokens].  Returns ((l_start, l_det, l_end), s[L], rho[L])."""
    import numpy as np
    d = np.ascontiguousarray(d, dtype=np.float32)
    n_layers, n_tokens = d.shape
    params = rc_layer_profile_params(tau_st, tail, lam, consecutive)
    out = rc_layer_triple()
    s = np.zeros(n_layers, np.float64)
    rho = np.zeros(n_layers, np.float64)
    _check(lib.rc_layer_profile(d.ctypes.data, n_layers, n_tokens, C.byref(params), C.byref(out), s.ctypes.data,
                                rho.ctypes.data), "rc_layer_profile")
    return (out.l_start, out.l_det, out.l_end), s, rho


def alloc_workspace(n_bytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least n_bytes, 256-byte aligned (torch's allocator aligns to 512)."""
    return torch.empty(max(n_bytes, 256), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------ stage calls
def rc_stage_workspace_bytes(n_positions: int, head_dim: int) -> int:
    return int(lib.rc_stage_workspace_bytes(n_positions, head_dim))


def rc_rope_rerotate(src: rc_kv_layer, src_seq: int, src_offset: int, dst: rc_kv_layer, dst_seq: int,
                     dst_offset: int, n_tokens: int, k_is_pre_rope: bool, old_start_pos: int, rope_base: float,
                     workspace: torch.Tensor, stream=None) -> None:
    _check(lib.rc_rope_rerotate(C.byref(src), src_seq, src_offset, C.byref(dst), dst_seq, dst_offset, n_tokens,
                                1 if k_is_pre_rope else 0, old_start_pos, rope_base, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)), "rc_rope_rerotate")


RC_REROTATE_STATIC_MAX_POSITIONS = 32768


def rc_rope_rerotate_static_scratch_bytes() -> int:
    return int(lib.rc_rope_rerotate_static_scratch_bytes())


def rc_rope_rerotate_static(src: rc_kv_layer, src_seq: int, src_offset: int, dst: rc_kv_layer, dst_seq: int,
                            dst_offset: int, n_tokens: int, k_is_pre_rope: bool, old_start_pos: int,
                            rope_base: float, stream=None) -> None:
    _check(lib.rc_rope_rerotate_static(C.byref(src), src_seq, src_offset, C.byref(dst), dst_seq, dst_offset,
                                       n_tokens, 1 if k_is_pre_rope else 0, old_start_pos, rope_base,
                                       _stream(stream)), "rc_rope_rerotate_static")


def rc_vdev_score(v_fresh: torch.Tensor, cache: rc_kv_layer, seq: int, offset: int, n_tokens: int,
                  score: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib.rc_vdev_score(_ptr(v_fresh), C.byref(cache), seq, offset, n_tokens, _ptr(score), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream(stream)), "rc_vdev_score")


def rc_topk(score: torch.Tensor, n: int, k: int, idx_out: torch.Tensor, stream=None) -> None:
    _check(lib.rc_topk(_ptr(score), n, k, _ptr(idx_out), _stream(stream)), "rc_topk")


def rc_threshold_select(score: torch.Tensor, n: int, tau: float, idx_out: torch.Tensor, count_out: torch.Tensor,
                        stream=None) -> None:
    _check(lib.rc_threshold_select(_ptr(score), n, tau, _ptr(idx_out), _ptr(count_out), _stream(stream)),
           "rc_threshold_select")


def rc_final_select(s_dev: torch.Tensor, s_inf: Optional[torch.Tensor], n: int, tau_dev: float, tau_inf: float,
                    k_suf: int, idx_out: torch.Tensor, count_out: torch.Tensor, stream=None) -> None:
    _check(lib.rc_final_select(_ptr(s_dev), _ptr(s_inf), n, tau_dev, tau_inf, k_suf, _ptr(idx_out), _ptr(count_out),
                               _stream(stream)), "rc_final_select")


def rc_sparse_attention_workspace_bytes(n: int, n_q_heads: int, cache: rc_kv_layer) -> int:
    return int(lib.rc_sparse_attention_workspace_bytes(n, n_q_heads, C.byref(cache)))


def rc_sparse_attention(q: torch.Tensor, q_pos: torch.Tensor, n: int, n_q_heads: int, cache: rc_kv_layer, seq: int,
                        out: torch.Tensor, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.rc_sparse_attention(_ptr(q), _ptr(q_pos), n, n_q_heads, C.byref(cache), seq, _ptr(out),
                                   _ptr(workspace), nbytes, _stream(stream)), "rc_sparse_attention")


def rc_gemm_workspace_bytes() -> int:
    return int(lib.rc_gemm_workspace_bytes())


def rc_gemm_rows(dtype: int, a: torch.Tensor, w: torch.Tensor, c: torch.Tensor, m: int, n: int, k: int,
                 workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.rc_gemm_rows(dtype, _ptr(a), _ptr(w), _ptr(c), m, n, k, _ptr(workspace), nbytes, _stream(stream)),
           "rc_gemm_rows")


def rc_gemm_plan_check(m: int, n: int, k: int, swiglu: bool, tile: int, n_cus: int = 256, with_workspace: bool = True):
    """(violations, grid size) of the launch schedule of one bf16 GEMM; host only."""
    nb = C.c_int32(0)
    err = int(lib.rc_gemm_plan_check(m, n, k, 1 if swiglu else 0, tile, n_cus, 1 if with_workspace else 0, C.byref(nb)))
    return err, int(nb.value)


def rc_ceiling_stream_copy(src: torch.Tensor, dst: torch.Tensor, nbytes: int, stream=None) -> None:
    _check(lib.rc_ceiling_stream_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "rc_ceiling_stream_copy")


def rc_ceiling_mfma_loop_out_bytes(n_workgroups: int) -> int:
    return int(lib.rc_ceiling_mfma_loop_out_bytes(n_workgroups))


def rc_ceiling_mfma_loop(out: torch.Tensor, n_workgroups: int, iters: int, stream=None) -> float:
    """Launches the register-only MFMA loop; returns the floating-point operations it performs."""
    flops = C.c_double(0.0)
    _check(lib.rc_ceiling_mfma_loop(_ptr(out), n_workgroups, iters, C.byref(flops), _stream(stream)),
           "rc_ceiling_mfma_loop")
    return float(flops.value)


RC_GEMM_STORE, RC_GEMM_STORE_T, RC_GEMM_ADD, RC_GEMM_SWIGLU = 0, 1, 2, 3


def rc_gemm_rows_fused(dtype: int, epilogue: int, a: torch.Tensor, w: torch.Tensor, w2: Optional[torch.Tensor],
                       c: torch.Tensor, m: int, n: int, k: int, workspace: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.rc_gemm_rows_fused(dtype, epilogue, _ptr(a), _ptr(w), _ptr(w2), _ptr(c), m, n, k, _ptr(workspace),
                                  nbytes, _stream(stream)), "rc_gemm_rows_fused")


def rc_rope_scatter_workspace_bytes(n: int, dst: rc_kv_layer) -> int:
    return int(lib.rc_rope_scatter_workspace_bytes(n, C.byref(dst)))


def rc_rope_scatter(qkv: torch.Tensor, pos: torch.Tensor, n: int, n_q_heads: int, rope_base: float, dst: rc_kv_layer,
                    seq: int, q_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib.rc_rope_scatter(_ptr(qkv), _ptr(pos), n, n_q_heads, rope_base, C.byref(dst), seq, _ptr(q_out),
                               _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "rc_rope_scatter")


def rc_scatter_paged(k_rows: torch.Tensor, v_rows: torch.Tensor, pos: torch.Tensor, n: int, dst: rc_kv_layer,
                     seq: int, stream=None) -> None:
    _check(lib.rc_scatter_paged(_ptr(k_rows), _ptr(v_rows), _ptr(pos), n, C.byref(dst), seq, _stream(stream)),
           "rc_scatter_paged")


# ------------------------------------------------------------------ per-stage timing
def rc_profile_enable(on: bool) -> None:
    _check(lib.rc_profile_enable(1 if on else 0), "rc_profile_enable")


def rc_profile_read() -> dict:
    """{stage class: (milliseconds, launches)} accumulated since the last read."""
    n = lib.rc_profile_class_count()
    ms = (C.c_float * n)()
    cnt = (C.c_int32 * n)()
    _check(lib.rc_profile_read(ms, cnt), "rc_profile_read")
    return {lib.rc_profile_class_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


RC_TUNE_GEMM_TILE = 1
RC_TUNE_ATTN_CHUNK_TILES = 2
RC_TUNE_GEMM_XCD_REMAP = 3
RC_TUNE_GEMM_THIN_TILES = 4


def rc_tune_set(key: int, value: int) -> None:
    _check(lib.rc_tune_set(key, value), "rc_tune_set")
