"""Host-side checks of the synthetic workloads (no GPU, no oracle arithmetic)."""
import os

import numpy as np

import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "architectures.txt")


def test_model_shapes_follow_the_papers_architecture_table():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, dim, heads, layers, ctx = line.split()
        w = W.get_workload(name)
        assert w.model.d_model == int(dim) and w.model.n_layers == int(layers)
        if heads != "-":
            assert w.model.n_q_heads == int(heads)
        assert w.n_prompt + w.n_new + w.draft_len + 1 <= int(ctx)


def test_weights_are_seeded_scaled_and_thread_independent():
    w = W.get_workload("c1")
    a, b = W.make_weights(w, threads=1), W.make_weights(w, threads=5)
    for la, lb in zip(a["layers"], b["layers"]):
        for k in la:
            assert np.array_equal(la[k], lb[k])
    assert abs(a["embed"].std() - 0.02) < 5e-4
    E = w.exit_layer
    assert abs(a["layers"][E - 1]["wo"].std() - 0.02) < 1e-3
    assert abs(a["layers"][E]["wo"].std() - 0.02 * w.resid_scale) < 1e-4
    assert abs(a["layers"][E]["w_down"].std() - 0.02 * w.resid_scale) < 1e-4
    assert abs(a["layers"][E]["wq"].std() - 0.02) < 1e-3
    assert np.all(a["final_norm"] == 1.0)
    p = W.make_prompt(w)
    assert p.dtype == np.int32 and p.shape == (32,) and p.min() >= 0 and p.max() < 1024
    assert np.array_equal(p, W.make_prompt(w))


def test_bf16_models_are_stored_as_bit_patterns():
    w = W.shrink(W.get_workload("c2"), 1, 1)
    w = w.with_(model=W.ModelConfig(**{**w.model.__dict__, "vocab": 64, "ffn_dim": 256}))
    ws = W.make_weights(w)
    assert ws["embed"].dtype == np.uint16 and ws["layers"][0]["wq"].shape == (2048, 2048)
    assert ws["final_norm"][0] == 0x3F80                       # bf16 bits of 1.0


def test_byte_model_of_the_paper_shaped_configs():
    m = W.get_workload("c2").model
    assert abs(m.layer_weight_bytes() / 1e6 - 102.77) < 0.01
    assert abs(m.head_weight_bytes() / 1e6 - 131.08) < 0.01
    m = W.get_workload("c4").model
    assert abs(m.layer_weight_bytes() / 1e6 - 436.22) < 0.01 and m.kv_bytes_per_pos_layer() == 4096
