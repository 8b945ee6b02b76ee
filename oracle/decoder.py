"""CPU oracle: the Llama-style decoder that greedy self-speculative decoding runs on.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package; it
exists so that the tests, the smoke check and the benchmark's CPU-baseline leg have a
plain, slow, independently written statement of what the HIP path must compute.

What it follows (paper sections, restated):
  * Section 4.1: the model is a residual recurrence x_{l+1} = x_l + f_l(x_l) over L
    transformer layers, followed by an LM head g.
  * Section 2.1 ("Exiting Earlier in LLMs"): g is the model's final normalisation
    followed by its final linear layer, and the same g is applied at every exit.
  * Section 4.2: early exit at E runs layers 0..E-1 and outputs g(x_E).
  * Section 4.3.3: one KV cache serves draft and verify, because both walk the same
    layers in the same order.
The inside of f_l (RMSNorm, rotary embedding on half-split pairs, causal softmax
attention with grouped KV heads, SwiGLU feed-forward) is not printed in the paper; it is
the "Llama-style" layer the workloads name, written here in its textbook form.

Precision: `dtype` is float32 by default (the precision the task fixes for this oracle);
float64 is accepted so that the invariant tests can separate algorithmic errors from
rounding.  For bf16 models the stored weights ARE bf16 values (widened exactly); with
`emulate_bf16_act=True` the oracle also rounds, to bf16 with round-to-nearest-even, each
tensor that a bf16 pipeline stores as a matmul input:
  (R2) every RMSNorm output, (R3) q and k after the rotary embedding and v (so the KV
  cache holds bf16 values), (R4) the attention output, (R5) the SwiGLU output.
The residual stream, softmax statistics, rotary sin/cos and the logits stay in `dtype`.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np


# ----------------------------------------------------------------------------- scalars

def bf16_bits_to_float(bits: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16)."""
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(dtype, copy=False)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (ties to even), returned in the input's dtype."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(a.dtype, copy=False)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x_i * gain_i / sqrt(mean_j x_j^2 + eps) along the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * gain


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def softmax_lastaxis(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def rope_angles(positions: Sequence[int], head_dim: int, base: float):
    """cos, sin of t * base^(-2j/head_dim), j < head_dim/2, evaluated in float64."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.power(np.float64(base), -2.0 * j / head_dim)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)


def apply_rope(y: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate the pairs (j, j + hd/2) of y[..., hd] by the angle whose cos/sin are given.

    y: [rows, heads, hd]; cos, sin: [rows, hd/2].
    """
    half = y.shape[-1] // 2
    a, b = y[..., :half], y[..., half:]
    c, s = cos[:, None, :].astype(y.dtype), sin[:, None, :].astype(y.dtype)
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def argmax_lowest(logits: np.ndarray) -> int:
    """Index of the maximum; the lowest index among exact ties."""
    return int(np.argmax(logits))  # numpy returns the first maximal element


def top2_margin(logits: np.ndarray) -> float:
    """Largest minus second-largest value (0 on an exact tie)."""
    if logits.shape[-1] < 2:
        return math.inf
    part = np.partition(logits, -2)[-2:]
    return float(part[1] - part[0])


def runner_up(logits: np.ndarray) -> int:
    """Index of the second-largest value: the lowest index that attains the largest value left once
    the argmax (lowest index on ties) is set aside.  Bookkeeping for the tests' near-tie rule: which
    other token a rounding-sized change of the logits could turn the decision into."""
    best = argmax_lowest(logits)
    rest = np.array(logits, dtype=np.float64, copy=True)
    rest[best] = -np.inf
    return int(np.argmax(rest))


# ------------------------------------------------------------------------------- model

class KVCache:
    """K and V per layer, kv-head and position: the single cache of Section 4.3.3."""

    def __init__(self, n_layers: int, n_kv: int, max_seq: int, head_dim: int, dtype):
        self.k = np.zeros((n_layers, n_kv, max_seq, head_dim), dtype=dtype)
        self.v = np.zeros((n_layers, n_kv, max_seq, head_dim), dtype=dtype)
        self.max_seq = max_seq


class OracleModel:
    def __init__(self, cfg, weights: dict, dtype=np.float32, emulate_bf16_act: bool = False):
        """cfg: a workloads.ModelConfig; weights: the dict workloads.make_weights returns."""
        self.cfg = cfg
        self.dtype = np.dtype(dtype)
        self.emulate = bool(emulate_bf16_act)

        def widen(a):
            if a.dtype == np.uint16:
                return bf16_bits_to_float(a, self.dtype)
            return a.astype(self.dtype, copy=False)

        self.embed = widen(weights["embed"])
        self.lm_head = widen(weights["lm_head"])
        self.final_norm = widen(weights["final_norm"])
        self.layers = [{k: widen(v) for k, v in lw.items()} for lw in weights["layers"]]
        assert len(self.layers) == cfg.n_layers

    # -- helpers
    def _r(self, a: np.ndarray) -> np.ndarray:
        return round_to_bf16(a) if self.emulate else a

    def new_cache(self, max_seq: int) -> KVCache:
        c = self.cfg
        return KVCache(c.n_layers, c.n_kv_heads, max_seq, c.head_dim, self.dtype)

    def embed_tokens(self, tokens: Sequence[int]) -> np.ndarray:
        return self.embed[np.asarray(tokens, dtype=np.int64)].copy()

    # -- one transformer layer f_l applied to a group of rows
    def layer(self, l: int, x: np.ndarray, positions: Sequence[int], cache: KVCache) -> np.ndarray:
        """x: [m, d_model] rows at `positions` (increasing).  Appends their K, V to the cache
        at those positions; row i attends to cache positions 0..positions[i]."""
        c, w = self.cfg, self.layers[l]
        m = x.shape[0]
        hd, nq, nkv = c.head_dim, c.n_q_heads, c.n_kv_heads
        group = nq // nkv
        a = self._r(rmsnorm(x, w["attn_norm"], c.rms_eps))
        q = (a @ w["wq"].T).reshape(m, nq, hd)
        k = (a @ w["wk"].T).reshape(m, nkv, hd)
        v = (a @ w["wv"].T).reshape(m, nkv, hd)
        cos, sin = rope_angles(positions, hd, c.rope_base)
        q = self._r(apply_rope(q, cos, sin))
        k = self._r(apply_rope(k, cos, sin))
        v = self._r(v)
        for i, t in enumerate(positions):
            cache.k[l, :, t, :] = k[i]
            cache.v[l, :, t, :] = v[i]
        o = np.empty((m, nq, hd), dtype=self.dtype)
        scale = self.dtype.type(1.0 / math.sqrt(hd))
        for i, t in enumerate(positions):
            kk = cache.k[l, :, : t + 1, :]                    # [nkv, t+1, hd]
            vv = cache.v[l, :, : t + 1, :]
            qg = q[i].reshape(nkv, group, hd)                 # q-head h uses kv-head h // group
            s = np.matmul(qg, kk.transpose(0, 2, 1)) * scale  # [nkv, group, t+1]
            p = softmax_lastaxis(s)
            o[i] = np.matmul(p, vv).reshape(nq, hd)
        o = self._r(o.reshape(m, nq * hd))
        h = x + o @ w["wo"].T
        b = self._r(rmsnorm(h, w["ffn_norm"], c.rms_eps))
        act = self._r(silu(b @ w["w_gate"].T) * (b @ w["w_up"].T))
        return h + act @ w["w_down"].T

    def run_layers(self, x: np.ndarray, positions: Sequence[int], cache: KVCache,
                   l0: int, l1: int, hidden: Optional[List[np.ndarray]] = None) -> np.ndarray:
        """x_{l0} -> x_{l1}.  If `hidden` is a list, x_{l+1} is appended for each layer run."""
        for l in range(l0, l1):
            x = self.layer(l, x, positions, cache)
            if hidden is not None:
                hidden.append(x.copy())
        return x

    def head(self, x: np.ndarray) -> np.ndarray:
        """g(x): final RMSNorm, then the LM-head linear layer.  x: [m, d_model] -> [m, vocab]."""
        a = self._r(rmsnorm(x, self.final_norm, self.cfg.rms_eps))
        return a @ self.lm_head.T
