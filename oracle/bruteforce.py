"""CPU oracle cross-check: the decoder with NO KV cache, recomputed from scratch.

TEST INFRASTRUCTURE ONLY (see decoder.py).

Every call runs the whole token sequence through every layer with a full causal score
matrix, so nothing is carried between tokens.  It is written head by head with an explicit
mask (not by reusing the cached layer code), and serves as the brute-force reference for
tiny models: greedy decoding with it must give the same ids and hidden states as the
cached decoder.
"""
from __future__ import annotations

import math
from typing import List

import numpy as np

from .decoder import OracleModel


def forward_nocache(model: OracleModel, tokens, n_layers=None):
    """Returns (hidden [n_layers+1, T, dm], logits [T, vocab]) for the whole sequence."""
    c = model.cfg
    L = c.n_layers if n_layers is None else n_layers
    dt = model.dtype
    T = len(tokens)
    hd, half = c.head_dim, c.head_dim // 2
    x = np.stack([model.embed[int(t)] for t in tokens]).astype(dt)
    hidden = [x.copy()]
    theta = np.array([[t * c.rope_base ** (-2.0 * j / hd) for j in range(half)] for t in range(T)])
    cs, sn = np.cos(theta).astype(dt), np.sin(theta).astype(dt)
    mask = np.triu(np.ones((T, T), dtype=bool), k=1)          # True above the diagonal: future keys
    for l in range(L):
        w = model.layers[l]
        rms = np.sqrt((x ** 2).sum(axis=1, keepdims=True) / c.d_model + dt.type(c.rms_eps))
        a = model._r(x / rms * w["attn_norm"][None, :])
        attn = np.zeros((T, c.q_dim), dtype=dt)
        for h in range(c.n_q_heads):
            kvh = h // (c.n_q_heads // c.n_kv_heads)
            qh = a @ w["wq"][h * hd:(h + 1) * hd].T               # [T, hd]
            kh = a @ w["wk"][kvh * hd:(kvh + 1) * hd].T
            vh = model._r(a @ w["wv"][kvh * hd:(kvh + 1) * hd].T)
            qr = np.empty_like(qh)
            kr = np.empty_like(kh)
            for src, dst in ((qh, qr), (kh, kr)):
                dst[:, :half] = src[:, :half] * cs - src[:, half:] * sn
                dst[:, half:] = src[:, half:] * cs + src[:, :half] * sn
            qr, kr = model._r(qr), model._r(kr)
            s = (qr @ kr.T) / dt.type(math.sqrt(hd))
            s = np.where(mask, -np.inf, s)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            attn[:, h * hd:(h + 1) * hd] = p @ vh
        hmid = x + model._r(attn) @ w["wo"].T
        rms = np.sqrt((hmid ** 2).sum(axis=1, keepdims=True) / c.d_model + dt.type(c.rms_eps))
        b = model._r(hmid / rms * w["ffn_norm"][None, :])
        g = b @ w["w_gate"].T
        u = b @ w["w_up"].T
        x = hmid + model._r(g / (1.0 + np.exp(-g)) * u) @ w["w_down"].T
        hidden.append(x.copy())
    rms = np.sqrt((x ** 2).sum(axis=1, keepdims=True) / c.d_model + dt.type(c.rms_eps))
    logits = model._r(x / rms * model.final_norm[None, :]) @ model.lm_head.T
    return np.stack(hidden, axis=0), logits


def greedy_nocache(model: OracleModel, prompt, n_new: int) -> List[int]:
    """Greedy decoding where each new token recomputes the whole sequence."""
    seq = [int(t) for t in prompt]
    out: List[int] = []
    for _ in range(n_new):
        _, logits = forward_nocache(model, seq)
        t = int(np.argmax(logits[-1]))
        out.append(t)
        seq.append(t)
    return out
