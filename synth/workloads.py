"""Shapes, workloads and seeded random draws for the selective-recompute prefill.

Everything here is input preparation: which tensors exist, how large they are,
and which random numbers fill them.  Random streams are counter-based (Philox)
and keyed by (master seed, workload name, tensor name, layer), so any tensor can
be regenerated on its own and both consumers (the CPU oracle's tests and the
HIP path's tests) see bit-identical values.

Value recipe: projection weights N(0, 0.02^2), RMSNorm gains 1, token hidden
states N(0, 1) per element.  For bf16 workloads every generated tensor is
rounded to bf16 (round-to-nearest-even) once and handed out as float32 holding
bf16-representable values, so both consumers start from the same numbers.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np

MASTER_SEED = 20260313


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "f32" or "bf16": storage type of weights, activations and KV

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def gemm_params_per_layer(self) -> int:
        d, hq, hkv, dh, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        return 2 * d * hq * dh + 2 * d * hkv * dh + 3 * d * f


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    n_prefix: int          # P: tokens of the new prefix
    n_seg: int             # S: tokens of the reused segment
    n_alt: int             # length of the earlier agent's (different) prefix
    l_start: int
    l_det: int
    l_end: int
    budget_pct: int        # recompute budget in percent of S
    block_size: int = 0    # 0: contiguous cache; >0: paged with this many tokens per block
    n_req: int = 1
    prefix_range: Tuple[int, int] = (0, 0)   # ragged batches: P_i ~ U[lo, hi]
    seg_range: Tuple[int, int] = (0, 0)      # ragged batches: S_i ~ U[lo, hi]
    note: str = ""


def budget_to_k(n_seg: int, budget_pct: int) -> int:
    """Token count for a percentage budget, floor, in integer arithmetic."""
    return (n_seg * budget_pct) // 100


_TINY = ModelShape(2, 256, 4, 2, 64, 688, 1024, 1.0e4, dtype="f32")
_MISTRAL = ModelShape(32, 4096, 32, 8, 128, 14336, 32768, 1.0e6)
_LLAMA = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, 5.0e5)
_QWEN32 = ModelShape(64, 5120, 40, 8, 128, 27648, 152064, 1.0e6)

WORKLOADS: Dict[str, Workload] = {}


def _add(w: Workload) -> None:
    WORKLOADS[w.name] = w


# The five benchmark configurations.
_add(Workload("tiny_f32", _TINY, 128, 256, 96, 0, 1, 1, 20,
              note="2-layer fp32 decoder, recompute 20% in layer 1"))
_add(Workload("mistral7b_4k", _MISTRAL, 1024, 4096, 512, 7, 8, 24, 15,
              note="headline: 1k new prefix + 4k reused, 15% in layers 8-24"))
for _pct in (5, 10, 20):
    _add(Workload(f"llama8b_16k_b{_pct}", _LLAMA, 2048, 16384, 1024, 7, 8, 24, _pct))
_add(Workload("mistral7b_ragged16", _MISTRAL, 0, 0, 0, 7, 8, 24, 15, block_size=16, n_req=16,
              prefix_range=(256, 2048), seg_range=(1024, 8192),
              note="16 ragged requests, paged KV with 16-token blocks; alt prefix = P_i // 2"))
_add(Workload("qwen32b_32k", _QWEN32, 4096, 32768, 2048, 15, 16, 48, 10))

# Parity-sized relatives: same structure, sizes the CPU oracle finishes in seconds.
_add(Workload("tiny_f32_paged", _TINY, 100, 203, 77, 0, 1, 1, 20, block_size=16,
              note="ragged sizes, paged"))
_add(Workload("tiny_f32_inplace", _TINY, 112, 203, 80, 0, 1, 1, 20, block_size=16,
              note="the segment moves by exactly two 16-token blocks (80 -> 112): a take-over in place is allowed"))
_TINY5 = ModelShape(5, 256, 4, 2, 64, 688, 512, 1.0e4, dtype="f32")
_add(Workload("tiny5_f32", _TINY5, 70, 150, 33, 1, 2, 3, 20, block_size=16,
              note="5 layers so that every phase (before / dense / sparse / after) has at least one layer"))
_add(Workload("tiny5_f32_noprefix", _TINY5, 0, 120, 40, 1, 2, 3, 20, note="segment starts at position 0"))
_add(Workload("tiny5_f32_one", _TINY5, 9, 1, 5, 1, 2, 3, 100, note="one-token segment"))
_add(Workload("tiny5_f32_batch32", _TINY5, 0, 0, 0, 1, 2, 3, 8, block_size=16, n_req=32,
              prefix_range=(0, 40), seg_range=(1, 60), note="the most requests one call takes; some budgets round to 0"))
_add(Workload("small_bf16", ModelShape(4, 512, 8, 2, 128, 1408, 2048, 1.0e6), 150, 333, 70, 0, 1, 2, 15,
              note="narrow bf16 model, 4 layers, head_dim 128, group 4"))
_add(Workload("small_bf16_ragged", ModelShape(4, 512, 8, 2, 128, 1408, 2048, 1.0e6), 0, 0, 0, 0, 1, 2, 15,
              block_size=16, n_req=3, prefix_range=(40, 200), seg_range=(100, 400)))
_add(Workload("mistral7b_trunc", replace(_MISTRAL, n_layers=4, vocab=4096), 192, 640, 96, 0, 1, 2, 15,
              note="Mistral-7B widths, 4 layers, triple (0,1,2)"))
_add(Workload("mistral7b_4k_trunc", replace(_MISTRAL, n_layers=4, vocab=4096), 1024, 4096, 512, 0, 1, 2, 15,
              note="the headline token counts (1024 new + 4096 reused, k = 614) at Mistral-7B widths, 4 layers, "
                   "triple (0,1,2): dense, two sparse and one tail layer; the oracle finishes it in about a minute"))
_add(Workload("mistral7b_pair_trunc", replace(_MISTRAL, n_layers=3, vocab=4096), 0, 0, 0, 0, 1, 2, 15, block_size=16,
              n_req=2, prefix_range=(256, 1024), seg_range=(1024, 2560),
              note="two ragged requests, paged with 16-token blocks, Mistral-7B widths, 3 layers"))
_add(Workload("qwen32b_trunc", replace(_QWEN32, n_layers=3, vocab=4096), 130, 330, 64, 0, 1, 2, 10,
              note="32B widths (group 5), 3 layers"))


def stream_rng(workload: str, tensor: str, layer: int = -1, seed: int = MASTER_SEED) -> np.random.Generator:
    """Counter-based generator keyed by (seed, workload, tensor, layer)."""
    h = hashlib.sha256(f"{seed}|{workload}|{tensor}|{layer}".encode()).digest()
    key = int.from_bytes(h[:16], "little")
    return np.random.Generator(np.random.Philox(key=key))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


def _finish(x: np.ndarray, dtype: str) -> np.ndarray:
    return round_to_bf16(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def make_weights(w: Workload, seed: int = MASTER_SEED, std: float = 0.02) -> dict:
    """All model weights as float32 arrays in [out][in] layout.

    Returns {"layers": [ {wq, wk, wv, wo, w_gate, w_up, w_down, g_attn, g_ffn} ],
             "g_final": [d], "w_lm": [vocab][d]}.
    """
    s = w.shape
    d, hq, hkv, dh, f = s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ffn
    key = w.name if w.n_req == 1 else w.name  # weights are shared by all requests of a batch

    def draw(name: str, layer: int, rows: int, cols: int) -> np.ndarray:
        g = stream_rng(key, name, layer, seed)
        return _finish(g.standard_normal((rows, cols), dtype=np.float32) * np.float32(std), s.dtype)

    layers = []
    for l in range(s.n_layers):
        layers.append({
            "wq": draw("wq", l, hq * dh, d),
            "wk": draw("wk", l, hkv * dh, d),
            "wv": draw("wv", l, hkv * dh, d),
            "wo": draw("wo", l, d, hq * dh),
            "w_gate": draw("w_gate", l, f, d),
            "w_up": draw("w_up", l, f, d),
            "w_down": draw("w_down", l, d, f),
            "g_attn": np.ones(d, dtype=np.float32),
            "g_ffn": np.ones(d, dtype=np.float32),
        })
    return {"layers": layers, "g_final": np.ones(d, dtype=np.float32),
            "w_lm": draw("w_lm", -1, s.vocab, d)}


def make_hidden(w: Workload, tensor: str, n_tokens: int, req: int = 0, seed: int = MASTER_SEED) -> np.ndarray:
    """Token hidden states [n_tokens][d] ~ N(0,1) for one named input of one request."""
    g = stream_rng(w.name, f"{tensor}#{req}", -1, seed)
    return _finish(g.standard_normal((n_tokens, w.shape.d_model), dtype=np.float32), w.shape.dtype)


def make_influence(w: Workload, n_tokens: int, req: int = 0, seed: int = MASTER_SEED) -> np.ndarray:
    """Stand-in for the per-token attention mass an earlier agent accumulated while decoding
    (the input of the influence criterion): positive, heavy-tailed (log-normal), float32."""
    g = stream_rng(w.name, f"s_inf#{req}", -1, seed)
    return np.exp(g.standard_normal(n_tokens)).astype(np.float32)


def ragged_lengths(w: Workload, seed: int = MASTER_SEED) -> List[Tuple[int, int, int]]:
    """(P_i, S_i, alt_i) per request; fixed sizes for single-request workloads.  The earlier agent's prefix is half
    as long as the new one, and at least one token."""
    if w.n_req == 1 and w.prefix_range == (0, 0):
        return [(w.n_prefix, w.n_seg, w.n_alt)]
    g = stream_rng(w.name, "lengths", -1, seed)
    out = []
    for _ in range(w.n_req):
        p = int(g.integers(w.prefix_range[0], w.prefix_range[1] + 1))
        s = int(g.integers(w.seg_range[0], w.seg_range[1] + 1))
        out.append((p, s, max(p // 2, 1)))     # never the same (empty) prefix on both sides: scores would all be 0
    return out


def make_block_table(seq_lens: List[int], block_size: int, shuffle: bool = True,
                     seed: int = MASTER_SEED, extra_blocks: int = 3) -> Tuple[np.ndarray, int]:
    """Block table [n_seq][max_blocks] (int32) over one pool, and the pool's block count.

    With shuffle the pool's pages are handed out in a random order so that a
    sequence's pages are not contiguous; unused table slots hold -1.
    """
    need = [(n + block_size - 1) // block_size for n in seq_lens]
    total = sum(need) + extra_blocks
    ids = np.arange(total, dtype=np.int32)
    if shuffle:
        g = stream_rng("block_table", f"{seq_lens}|{block_size}", -1, seed)
        g.shuffle(ids)
    table = np.full((len(seq_lens), max(need)), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(need):
        table[i, :n] = ids[at:at + n]
        at += n
    return table, total
