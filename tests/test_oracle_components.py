"""Pins for the oracle's building blocks: closed forms, textbook special cases and
library routines (none of them re-uses the oracle's own formula)."""
import math

import numpy as np
import pytest
import scipy.special
import torch
import torch.nn.functional as F

import oracle as O
import workloads as W

rng = np.random.default_rng(1234)


# ------------------------------------------------------------------ bf16 rounding / widening
def test_round_to_bf16_matches_torch_and_ties_to_even():
    a = rng.standard_normal(100000).astype(np.float32) * np.float32(3.0)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(a), want)
    # 1 + 2^-8 lies exactly between 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies between 1+2^-7 (odd) and 1+2^-6 (even): goes up.
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8)], dtype=np.float32)
    np.testing.assert_array_equal(O.round_to_bf16(x),
                                  np.array([1.0, 1.0 + 2.0 ** -6, -1.0], dtype=np.float32))


def test_bf16_bits_widen_exactly_and_generator_roundtrip():
    a = rng.standard_normal(4096).astype(np.float32)
    bits = W.f32_to_bf16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16)
    np.testing.assert_array_equal(bits, want.view(torch.uint16).numpy())
    np.testing.assert_array_equal(O.bf16_bits_to_float(bits), want.to(torch.float32).numpy())


# ------------------------------------------------------------------ RMSNorm, SiLU, softmax
def test_rmsnorm_constant_vector_closed_form_and_library():
    eps = 1e-5
    g = rng.standard_normal(64)
    for cval in (2.5, -0.75):
        x = np.full((1, 64), cval)
        want = math.copysign(1.0, cval) * g / math.sqrt(1.0 + eps / cval ** 2)
        np.testing.assert_allclose(O.rmsnorm(x, g, eps)[0], want, rtol=1e-12)
    x = rng.standard_normal((5, 64))
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, eps), want, rtol=1e-12)


def test_silu_special_values_and_library():
    assert O.silu(np.array([0.0]))[0] == 0.0
    z = rng.standard_normal(1000) * 4
    np.testing.assert_allclose(O.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-12, atol=1e-15)
    assert abs(O.silu(np.array([30.0]))[0] - 30.0) < 1e-9      # silu(z) -> z for large z
    assert abs(O.silu(np.array([-30.0]))[0]) < 1e-9            # and -> 0 for very negative z


def test_softmax_rows_sum_to_one_shift_invariant_library():
    s = rng.standard_normal((7, 33)) * 5
    p = O.softmax_lastaxis(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(O.softmax_lastaxis(s + 1000.0), p, rtol=1e-9)
    np.testing.assert_allclose(p, scipy.special.softmax(s, axis=-1), rtol=1e-12)


# ------------------------------------------------------------------ rotary embedding
def test_rope_is_complex_rotation_of_half_split_pairs():
    hd, base = 16, 10000.0
    pos = [0, 1, 7, 300]
    y = rng.standard_normal((len(pos), 3, hd))
    cos, sin = O.rope_angles(pos, hd, base)
    got = O.apply_rope(y, cos, sin)
    for r, t in enumerate(pos):
        for h in range(3):
            for j in range(hd // 2):
                z = complex(y[r, h, j], y[r, h, j + hd // 2]) * complex(
                    math.cos(t * base ** (-2 * j / hd)), math.sin(t * base ** (-2 * j / hd)))
                assert abs(got[r, h, j] - z.real) < 1e-12
                assert abs(got[r, h, j + hd // 2] - z.imag) < 1e-12
    np.testing.assert_array_equal(got[0], y[0])                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(y, axis=-1), rtol=1e-12)


def test_rope_inner_product_depends_on_relative_position_only():
    hd = 32
    q = rng.standard_normal((1, 1, hd))
    k = rng.standard_normal((1, 1, hd))

    def ip(m, n):
        cq, sq = O.rope_angles([m], hd, 10000.0)
        ck, sk = O.rope_angles([n], hd, 10000.0)
        return float((O.apply_rope(q, cq, sq) * O.apply_rope(k, ck, sk)).sum())

    assert abs(ip(5, 2) - ip(105, 102)) < 1e-10
    assert abs(ip(9, 9) - float((q * k).sum())) < 1e-12
    assert abs(ip(5, 2) - ip(2, 5)) > 1e-3                           # and it is not symmetric


# ------------------------------------------------------------------ argmax / margin
def test_argmax_takes_lowest_index_on_ties_and_margin():
    lg = np.array([0.5, 2.0, -1.0, 2.0, 1.5])
    assert O.argmax_lowest(lg) == 1
    assert O.top2_margin(lg) == 0.0
    assert abs(O.top2_margin(np.array([0.1, 0.9, 0.7])) - 0.2) < 1e-12


def test_runner_up_is_the_second_entry_of_a_stable_sort():
    rng = np.random.default_rng(5)
    for _ in range(50):
        lg = rng.integers(0, 6, size=12).astype(np.float32)      # many exact ties
        order = sorted(range(len(lg)), key=lambda i: (-lg[i], i))  # by value, lowest index first
        assert O.argmax_lowest(lg) == order[0]
        assert O.runner_up(lg) == order[1]
        assert abs(O.top2_margin(lg) - (lg[order[0]] - lg[order[1]])) < 1e-12
    assert O.runner_up(np.array([0.1, 0.9, 0.7])) == 2


# ------------------------------------------------------------------ one layer, special cases
def _tiny_cfg(**kw):
    base = dict(name="t", n_layers=1, d_model=8, n_q_heads=2, n_kv_heads=2, head_dim=4,
                ffn_dim=16, vocab=11, rope_base=10000.0, rms_eps=1e-5, dtype="f32")
    base.update(kw)
    return W.ModelConfig(**base)


def _rand_weights(cfg, scale=0.3, seed=0):
    r = np.random.default_rng(seed)
    dm, qd, kvd, f, v = cfg.d_model, cfg.q_dim, cfg.kv_dim, cfg.ffn_dim, cfg.vocab
    def mk(*s): return (r.standard_normal(s) * scale)
    layers = []
    for _ in range(cfg.n_layers):
        layers.append(dict(wq=mk(qd, dm), wk=mk(kvd, dm), wv=mk(kvd, dm), wo=mk(dm, qd),
                           w_gate=mk(f, dm), w_up=mk(f, dm), w_down=mk(dm, f),
                           attn_norm=1 + 0.1 * r.standard_normal(dm), ffn_norm=1 + 0.1 * r.standard_normal(dm)))
    return dict(embed=mk(v, dm), lm_head=mk(v, dm), final_norm=1 + 0.1 * r.standard_normal(dm), layers=layers)


def test_layer_with_zero_queries_averages_shifted_values_closed_form():
    """wq = 0 makes every visible key equally likely, so the attention output is the running
    mean of v.  With wv a one-step shift (v_i = a_{i+1}), wo the identity and a zero FFN,
    x_1[t] = x_0[t] + mean_{u<=t} shift(rmsnorm(x_0[u])).  A transposed wv shifts the other
    way, a missing causal mask averages over all rows, a dropped residual loses x_0."""
    cfg = _tiny_cfg()
    ws = _rand_weights(cfg)
    lw = ws["layers"][0]
    dm = cfg.d_model
    lw["wq"][:] = 0
    shift = np.zeros((dm, dm))
    for i in range(dm - 1):
        shift[i, i + 1] = 1.0                       # out i <- in i+1
    lw["wv"] = shift.copy()
    lw["wo"] = np.eye(dm)
    lw["w_down"][:] = 0
    lw["attn_norm"] = np.ones(dm)
    m = O.OracleModel(cfg, ws, np.float64)
    toks = [3, 1, 4, 1, 5]
    x0 = ws["embed"][toks]
    cache = m.new_cache(8)
    x1 = m.layer(0, x0.copy(), list(range(5)), cache)
    for t in range(5):
        acc = np.zeros(dm)
        for u in range(t + 1):
            a = x0[u] / math.sqrt(float(np.mean(x0[u] ** 2)) + cfg.rms_eps)
            acc[:-1] += a[1:]
        np.testing.assert_allclose(x1[t], x0[t] + acc / (t + 1), rtol=1e-12, atol=1e-14)


def test_single_key_returns_its_value():
    cfg = _tiny_cfg()
    ws = _rand_weights(cfg, seed=3)
    lw = ws["layers"][0]
    lw["wo"] = np.eye(cfg.d_model)
    lw["w_down"][:] = 0
    m = O.OracleModel(cfg, ws, np.float64)
    x0 = ws["embed"][[7]]
    x1 = m.layer(0, x0.copy(), [0], m.new_cache(4))
    a = O.rmsnorm(x0, lw["attn_norm"], cfg.rms_eps)
    np.testing.assert_allclose(x1[0], x0[0] + lw["wv"] @ a[0], rtol=1e-12)   # position 0: rope is identity


def test_attention_block_matches_library_sdpa_with_grouped_heads():
    """Causal attention with 4 query heads on 2 KV heads against torch's fused routine."""
    cfg = _tiny_cfg(n_q_heads=4, n_kv_heads=2, head_dim=4, d_model=8)
    ws = _rand_weights(cfg, seed=5)
    lw = ws["layers"][0]
    lw["w_down"][:] = 0
    m = O.OracleModel(cfg, ws, np.float64)
    T = 6
    x0 = ws["embed"][[1, 2, 3, 4, 5, 6]]
    x1 = m.layer(0, x0.copy(), list(range(T)), m.new_cache(T))
    a = torch.from_numpy(O.rmsnorm(x0, lw["attn_norm"], cfg.rms_eps))
    q = (a @ torch.from_numpy(lw["wq"]).T).view(T, 4, 4)
    k = (a @ torch.from_numpy(lw["wk"]).T).view(T, 2, 4)
    v = (a @ torch.from_numpy(lw["wv"]).T).view(T, 2, 4)
    cos, sin = O.rope_angles(range(T), 4, cfg.rope_base)
    zq = torch.complex(q[..., :2], q[..., 2:]) * torch.complex(torch.from_numpy(cos), torch.from_numpy(sin))[:, None, :]
    zk = torch.complex(k[..., :2], k[..., 2:]) * torch.complex(torch.from_numpy(cos), torch.from_numpy(sin))[:, None, :]
    q = torch.cat([zq.real, zq.imag], -1)
    k = torch.cat([zk.real, zk.imag], -1)
    o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                       is_causal=True, enable_gqa=True)[0].transpose(0, 1).reshape(T, 16)
    want = x0 + (o @ torch.from_numpy(lw["wo"]).T).numpy()
    np.testing.assert_allclose(x1, want, rtol=1e-10, atol=1e-12)


def test_ffn_closed_form_when_gate_is_large():
    """For a large positive gate pre-activation silu(z) = z (to 1e-9), so the block reduces to
    h + w_down ((w_gate b) * (w_up b)); attention is switched off through wo = 0."""
    cfg = _tiny_cfg(ffn_dim=8)
    ws = _rand_weights(cfg, seed=9)
    lw = ws["layers"][0]
    lw["wo"][:] = 0
    lw["ffn_norm"] = np.ones(cfg.d_model)
    x0 = np.abs(ws["embed"][[2]]) + 1.0
    lw["w_gate"] = np.full((8, 8), 6.0)                      # every gate pre-activation >= 40
    m = O.OracleModel(cfg, ws, np.float64)
    x1 = m.layer(0, x0.copy(), [0], m.new_cache(2))
    b = x0[0] / math.sqrt(float(np.mean(x0[0] ** 2)) + cfg.rms_eps)
    want = x0[0] + lw["w_down"] @ ((lw["w_gate"] @ b) * (lw["w_up"] @ b))
    np.testing.assert_allclose(x1[0], want, rtol=1e-9)


def test_grouped_kv_equals_mha_with_repeated_kv_weights():
    gq = _tiny_cfg(n_q_heads=4, n_kv_heads=2, head_dim=4, d_model=16, n_layers=2)
    ws = _rand_weights(gq, seed=11)
    mh = _tiny_cfg(n_q_heads=4, n_kv_heads=4, head_dim=4, d_model=16, n_layers=2)
    ws2 = dict(ws, layers=[dict(lw) for lw in ws["layers"]])
    for lw in ws2["layers"]:
        for nm in ("wk", "wv"):
            blocks = lw[nm].reshape(2, 4, 16)
            lw[nm] = np.repeat(blocks, 2, axis=0).reshape(16, 16)     # q-head h uses kv-head h // 2
    toks = [1, 5, 2, 9, 3]
    a = O.forward_nocache(O.OracleModel(gq, ws, np.float64), toks)[1]
    b = O.forward_nocache(O.OracleModel(mh, ws2, np.float64), toks)[1]
    np.testing.assert_allclose(a, b, rtol=1e-12)
    ca, cb = O.OracleModel(gq, ws, np.float64), O.OracleModel(mh, ws2, np.float64)
    xa = ca.run_layers(ca.embed_tokens(toks), range(5), ca.new_cache(8), 0, 2)
    xb = cb.run_layers(cb.embed_tokens(toks), range(5), cb.new_cache(8), 0, 2)
    np.testing.assert_allclose(xa, xb, rtol=1e-12)


def test_head_is_final_norm_then_linear():
    cfg = _tiny_cfg()
    ws = _rand_weights(cfg, seed=2)
    m = O.OracleModel(cfg, ws, np.float64)
    x = np.full((1, cfg.d_model), 3.0)                         # constant row: closed-form norm
    want = ws["lm_head"] @ (ws["final_norm"] / math.sqrt(1 + cfg.rms_eps / 9.0))
    np.testing.assert_allclose(m.head(x)[0], want, rtol=1e-12)
