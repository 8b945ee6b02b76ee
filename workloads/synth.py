"""Workload shapes and seeded synthetic tensors for greedy self-speculative decoding.

The paper evaluates trained checkpoints on text datasets; neither is available, so the
five workloads below stand in for them by shape only (layer count, widths, head layout,
prompt length, number of new tokens, exit layer E and number of speculations d).

Everything here is data preparation: random streams, scaling of the residual-branch
output projections of the late layers (so that an early exit often agrees with the full
model), and storage of bf16 models as raw 16-bit patterns.  No step of the decoder or
of the decoding loop lives in this module.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

WEIGHT_NAMES_PER_LAYER = (
    "wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm",
)
_GLOBAL_NAMES = ("embed", "lm_head", "final_norm")
WEIGHT_STD = 0.02


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "bf16": weights stored as bf16 bit patterns; "f32": float32

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def layer_weight_bytes(self) -> int:
        dm = self.d_model
        n = 2 * dm * self.q_dim + 2 * dm * self.kv_dim + 3 * dm * self.ffn_dim + 2 * dm
        return n * self.elem_bytes

    def head_weight_bytes(self) -> int:
        return (self.vocab * self.d_model + self.d_model) * self.elem_bytes

    def kv_bytes_per_pos_layer(self) -> int:
        return 2 * self.kv_dim * self.elem_bytes


@dataclass(frozen=True)
class Workload:
    model: ModelConfig
    exit_layer: int       # E: the draft stage runs layers 0..E-1
    draft_len: int        # d: number of speculations per round
    n_prompt: int
    n_new: int
    resid_scale: float    # multiplies wo / w_down of layers >= E
    weight_seed: int = 0
    prompt_seed: int = 1
    gain_jitter: float = 0.0   # norm gains = 1 + gain_jitter * N(0,1); 0 gives all-ones
    sweep_exit_layers: Tuple[int, ...] = ()
    sweep_draft_lens: Tuple[int, ...] = ()

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


_C1 = ModelConfig("c1-tiny-f32", 4, 256, 4, 4, 64, 688, 1024, 10000.0, 1e-5, "f32")
_C2 = ModelConfig("c2-1.5b", 24, 2048, 16, 16, 128, 5632, 32000)
_C3 = ModelConfig("c3-7b", 32, 4096, 32, 32, 128, 11008, 32000)
_C4 = ModelConfig("c4-8b-gqa", 32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0)
_C5 = ModelConfig("c5-13b", 40, 5120, 40, 40, 128, 13824, 32000)

CONFIGS: Dict[str, Workload] = {
    "c1": Workload(_C1, exit_layer=2, draft_len=4, n_prompt=32, n_new=64, resid_scale=0.05),
    "c2": Workload(_C2, exit_layer=8, draft_len=6, n_prompt=512, n_new=256, resid_scale=0.1),
    "c3": Workload(_C3, exit_layer=8, draft_len=12, n_prompt=1536, n_new=128, resid_scale=0.1),
    "c4": Workload(_C4, exit_layer=12, draft_len=6, n_prompt=256, n_new=256, resid_scale=0.1),
    "c5": Workload(_C5, exit_layer=10, draft_len=8, n_prompt=1024, n_new=128, resid_scale=0.1,
                   sweep_exit_layers=(5, 10, 15), sweep_draft_lens=(4, 8, 12)),
}


def get_workload(name: str) -> Workload:
    return CONFIGS[name.lower()]


def shrink(w: Workload, n_layers: int, exit_layer: int, **kw) -> Workload:
    """Same widths as `w`, fewer layers: a parity case that fits a CPU run."""
    m = replace(w.model, n_layers=n_layers, name=f"{w.model.name}-L{n_layers}")
    return replace(w, model=m, exit_layer=exit_layer, **kw)


# --------------------------------------------------------------------------- tensors

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16, returned as uint16 bit patterns (storage only)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def _tensor_shapes(m: ModelConfig) -> Dict[str, Tuple[int, ...]]:
    return {
        "embed": (m.vocab, m.d_model),
        "lm_head": (m.vocab, m.d_model),
        "final_norm": (m.d_model,),
        "wq": (m.q_dim, m.d_model),
        "wk": (m.kv_dim, m.d_model),
        "wv": (m.kv_dim, m.d_model),
        "wo": (m.d_model, m.q_dim),
        "w_gate": (m.ffn_dim, m.d_model),
        "w_up": (m.ffn_dim, m.d_model),
        "w_down": (m.d_model, m.ffn_dim),
        "attn_norm": (m.d_model,),
        "ffn_norm": (m.d_model,),
    }


def _tensor_id(name: str, layer: int) -> int:
    if layer < 0:
        return _GLOBAL_NAMES.index(name)
    return 16 * (layer + 1) + WEIGHT_NAMES_PER_LAYER.index(name)


_BLOCK_ELEMS = 1 << 22  # tensors are filled in row blocks of about this many elements


def _row_blocks(shape: Tuple[int, ...]) -> List[Tuple[int, int]]:
    rows = shape[0]
    per_row = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    step = max(1, _BLOCK_ELEMS // per_row)
    return [(r, min(rows, r + step)) for r in range(0, rows, step)]


def _fill_block(w: Workload, name: str, layer: int, exit_layer: int, out: np.ndarray,
                blk: int, r0: int, r1: int) -> None:
    """Rows [r0, r1) of one tensor, from the stream keyed by (seed, tensor, block)."""
    shape = (r1 - r0,) + out.shape[1:]
    ss = np.random.SeedSequence([w.weight_seed, _tensor_id(name, layer), blk])
    rng = np.random.Generator(np.random.SFC64(ss))
    if name.endswith("norm"):
        a = np.ones(shape, dtype=np.float32)
        if w.gain_jitter:
            a += np.float32(w.gain_jitter) * rng.standard_normal(shape, dtype=np.float32)
    else:
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(WEIGHT_STD)
        if name in ("wo", "w_down") and layer >= exit_layer:
            a *= np.float32(w.resid_scale)
    out[r0:r1] = f32_to_bf16_bits(a) if out.dtype == np.uint16 else a


def iter_tensor_keys(m: ModelConfig) -> Iterator[Tuple[str, int]]:
    for name in _GLOBAL_NAMES:
        yield name, -1
    for layer in range(m.n_layers):
        for name in WEIGHT_NAMES_PER_LAYER:
            yield name, layer


def make_weights(w: Workload, exit_layer: Optional[int] = None, threads: int = 8) -> dict:
    """All tensors of the synthetic model.

    bf16 models: uint16 arrays of bf16 bit patterns; f32 models: float32 arrays.
    Layout of every matrix is row-major [out_features, in_features].
    `exit_layer` selects which layers get the residual scaling (defaults to the workload's E).
    The values do not depend on `threads`.
    """
    e = w.exit_layer if exit_layer is None else exit_layer
    m = w.model
    shapes = _tensor_shapes(m)
    np_dtype = np.uint16 if m.dtype == "bf16" else np.float32
    out: dict = {"layers": [dict() for _ in range(m.n_layers)]}
    jobs = []
    for name, layer in iter_tensor_keys(m):
        a = np.empty(shapes[name], dtype=np_dtype)
        if layer < 0:
            out[name] = a
        else:
            out["layers"][layer][name] = a
        for blk, (r0, r1) in enumerate(_row_blocks(a.shape)):
            jobs.append((name, layer, a, blk, r0, r1))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(lambda j: _fill_block(w, j[0], j[1], e, j[2], j[3], j[4], j[5]), jobs))
    return out


def make_tensor(w: Workload, name: str, layer: int, exit_layer: Optional[int] = None) -> np.ndarray:
    """One tensor of the model, exactly as make_weights fills it (layer -1 for the global tensors).
    A sweep over exit layers only has to replace wo / w_down of the layers whose scaling changes."""
    e = w.exit_layer if exit_layer is None else exit_layer
    m = w.model
    a = np.empty(_tensor_shapes(m)[name], dtype=np.uint16 if m.dtype == "bf16" else np.float32)
    for blk, (r0, r1) in enumerate(_row_blocks(a.shape)):
        _fill_block(w, name, layer, e, a, blk, r0, r1)
    return a


def make_prompt(w: Workload, n_prompt: Optional[int] = None) -> np.ndarray:
    """Prompt ids, uniform in [0, vocab), int32."""
    n = w.n_prompt if n_prompt is None else n_prompt
    rng = np.random.Generator(np.random.Philox(key=[w.prompt_seed, 0xFFFF]))
    return rng.integers(0, w.model.vocab, size=n, dtype=np.int64).astype(np.int32)
