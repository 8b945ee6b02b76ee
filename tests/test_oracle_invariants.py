"""Pins for the oracle's decoding loops: the invariants the method fixes.

* Self-speculative greedy output equals full-model greedy output (Section 4.3.2: the full
  model corrects the drafts, so there is no change in output).
* E = L: the draft already ran every layer, so every draft is accepted (Sections 2.1, 4.2).
* Zero residual scale on layers >= E: x_L = x_E (Section 4.1 recurrence), so acceptance is
  100 % and the number of rounds has a closed form.
* Brute force: recomputing the whole sequence without a cache gives the same ids / states.
* After every crop the cache equals a fresh prefill of prompt + emitted[:-1] (Appendix A.4).
"""
import math

import numpy as np
import pytest

import oracle as O
import workloads as W


def _model(c1, dtype=np.float64, **kw):
    w, ws, p = c1
    return w, O.OracleModel(w.model, ws, dtype, **kw), p


@pytest.mark.parametrize("E,d", [(1, 1), (2, 4), (3, 7), (2, 15), (4, 3), (1, 12)])
def test_self_speculative_equals_full_greedy(c1, E, d):
    w, m, p = _model(c1)
    g = O.greedy_full(m, p, w.n_new)
    s = O.self_speculative(m, p, w.n_new, E, d)
    assert s.tokens == g.tokens
    assert len(s.tokens) == w.n_new
    # accounting (Appendix A.4): every round emits its accepted drafts plus one verified token
    assert 1 + sum(r.n_accept + 1 for r in s.rounds) >= w.n_new
    assert 1 + sum(r.n_accept + 1 for r in s.rounds[:-1]) < w.n_new
    assert s.drafted == d * len(s.rounds) and 0 <= s.accepted <= s.drafted
    for r in s.rounds:
        assert r.draft[:r.n_accept] == r.verify[:r.n_accept]
        assert r.n_accept == d or r.draft[r.n_accept] != r.verify[r.n_accept]


@pytest.mark.parametrize("E,d", [(2, 4), (1, 3), (3, 6)])
def test_verifying_without_cache_reuse_changes_nothing_but_the_work(c1, E, d):
    """Section 4.3.3: reusing the draft stage's cache and exit states is an optimisation only; verifying
    with all L layers over the round's tokens gives the same rounds, drafts and verified tokens."""
    w, m, p = _model(c1)
    a = O.self_speculative(m, p, w.n_new, E, d)
    b = O.self_speculative(m, p, w.n_new, E, d, reuse=False)
    assert b.tokens == a.tokens == O.greedy_full(m, p, w.n_new).tokens
    assert [(r.pos, r.draft, r.verify, r.n_accept) for r in b.rounds] == [(r.pos, r.draft, r.verify, r.n_accept) for r in a.rounds]


@pytest.mark.parametrize("e_low,e_high,d", [(1, 2, 4), (1, 3, 5), (2, 4, 3)])
def test_per_token_exit_layer_is_lossless_and_reduces_to_the_fixed_exits(c1, e_low, e_high, d):
    """The per-token exit layer (the paper's closing section; reading in self_speculative_dynamic):
    whatever the threshold, every row ends up with the states of a fixed exit at e_high, so the
    output is full-model greedy; a threshold nobody reaches is self_speculative(e_high) round for
    round; a threshold everybody reaches drafts like self_speculative(e_low); in between, a draft
    that left early carries the early head's token and margin, a deep one the deep head's."""
    w, m, p = _model(c1)
    g = O.greedy_full(m, p, w.n_new)
    hi = O.self_speculative(m, p, w.n_new, e_high, d)
    lo = O.self_speculative(m, p, w.n_new, e_low, d)
    key = lambda r: [(t.pos, t.draft, t.verify, t.n_accept) for t in r.rounds]
    never = O.self_speculative_dynamic(m, p, w.n_new, e_low, e_high, d, math.inf)
    assert never.tokens == g.tokens and key(never) == key(hi)
    assert all(e == e_high for t in never.rounds for e in t.exit_layers)
    always = O.self_speculative_dynamic(m, p, w.n_new, e_low, e_high, d, 0.0)
    assert always.tokens == g.tokens and key(always) == key(lo)
    assert all(e == e_low for t in always.rounds for e in t.exit_layers)
    margins = sorted(x for t in lo.rounds for x in t.draft_margins)
    tau = margins[len(margins) // 2]                      # about half of the first drafts are confident
    mid = O.self_speculative_dynamic(m, p, w.n_new, e_low, e_high, d, tau)
    assert mid.tokens == g.tokens
    exits = [e for t in mid.rounds for e in t.exit_layers]
    assert e_low in exits and e_high in exits
    for t in mid.rounds:
        for e, mg in zip(t.exit_layers, t.draft_margins):
            assert (mg >= tau) if e == e_low else True    # early leavers met the threshold at e_low
        assert t.draft[:t.n_accept] == t.verify[:t.n_accept]
    # a round of `mid` that starts where a round of `hi` starts verifies to the same tokens as far as
    # the drafts agree: verification does not depend on where the drafts left
    by_pos = {t.pos: t for t in hi.rounds}
    shared = [t for t in mid.rounds if t.pos in by_pos]
    assert shared
    for t in shared:
        h = by_pos[t.pos]
        k = next((i for i in range(d) if t.draft[i] != h.draft[i]), d)
        assert t.verify[:k + 1] == h.verify[:k + 1]


def test_layer_probe_agrees_with_brute_force_and_with_early_exit(c1):
    """The per-layer probe (Section 3) is the head applied to x_1..x_L: row by row it must equal the
    argmax of g over the states of the cache-free recomputation, its last layer is the full model, and
    its layer E at the last prompt row is the first token of early-exit generation (Section 4.2)."""
    w, m, p = _model(c1)
    seq = list(p) + O.greedy_full(m, p, 6).tokens[:5]
    ids, margins = O.layer_probe(m, seq)
    hidden, logits = O.forward_nocache(m, seq)
    L = w.model.n_layers
    for l in range(L):
        lg = m.head(hidden[l + 1])
        assert ids[l] == [O.argmax_lowest(lg[i]) for i in range(len(seq))]
    assert ids[L - 1] == [O.argmax_lowest(logits[i]) for i in range(len(seq))]
    assert all(g >= 0 for row in margins for g in row)
    for E in (1, 2, 3):
        assert ids[E - 1][len(p) - 1] == O.early_exit_greedy(m, p, 1, E).tokens[0]


def test_float32_oracle_is_lossless_too(c1):
    w, m, p = _model(c1, np.float32)
    g = O.greedy_full(m, p, w.n_new)
    s = O.self_speculative(m, p, w.n_new, w.exit_layer, w.draft_len)
    firm = [i for i, mg in enumerate(g.margins) if mg < 1e-4]
    upto = firm[0] if firm else w.n_new
    assert s.tokens[:upto] == g.tokens[:upto]


def test_exit_at_last_layer_accepts_every_draft(c1):
    w, m, p = _model(c1)
    s = O.self_speculative(m, p, 40, w.model.n_layers, 5)
    assert all(r.n_accept == 5 for r in s.rounds)
    assert s.acceptance == 1.0
    assert s.tokens == O.greedy_full(m, p, 40).tokens
    assert O.early_exit_greedy(m, p, 40, w.model.n_layers).tokens == s.tokens


@pytest.mark.parametrize("d", [1, 4, 6])
def test_zero_residual_scale_closed_form(d):
    w = W.get_workload("c1").with_(resid_scale=0.0)
    ws, p = W.make_weights(w), W.make_prompt(w)
    m = O.OracleModel(w.model, ws, np.float64)
    N = 50
    s = O.self_speculative(m, p, N, w.exit_layer, d)
    assert s.acceptance == 1.0
    assert len(s.rounds) == math.ceil((N - 1) / (d + 1))
    assert s.tokens == O.greedy_full(m, p, N).tokens
    assert s.tokens == O.early_exit_greedy(m, p, N, w.exit_layer).tokens


def test_brute_force_without_cache_gives_same_ids_and_states(c1):
    w, m, p = _model(c1)
    N = 12
    g = O.greedy_full(m, p, N, want_hidden=True)
    assert O.greedy_nocache(m, p, N) == g.tokens
    hidden, logits = O.forward_nocache(m, list(p) + g.tokens[:-1])
    assert g.hidden.shape == hidden.shape == (w.model.n_layers + 1, len(p) + N - 1, w.model.d_model)
    np.testing.assert_allclose(g.hidden, hidden, rtol=1e-9, atol=1e-12)
    assert [int(np.argmax(logits[len(p) - 1 + i])) for i in range(N)] == g.tokens


def test_brute_force_matches_with_bf16_emulation():
    w = W.get_workload("c1")
    w = w.with_(model=W.ModelConfig(**{**w.model.__dict__, "dtype": "bf16", "name": "c1-bf16"}))
    ws, p = W.make_weights(w), W.make_prompt(w)
    m = O.OracleModel(w.model, ws, np.float32, emulate_bf16_act=True)
    g = O.greedy_full(m, p, 10)
    firm = [i for i, mg in enumerate(g.margins) if mg < 1e-3]
    upto = firm[0] if firm else 10
    assert O.greedy_nocache(m, p, 10)[:upto] == g.tokens[:upto]
    s = O.self_speculative(m, p, 10, 2, 4)
    assert s.tokens[:upto] == g.tokens[:upto]


def test_cache_after_each_crop_equals_fresh_prefill(c1):
    w, m, p = _model(c1)
    P, L = len(p), w.model.n_layers
    seen = []

    def hook(cache, pos, out):
        if len(out) < 30:                                    # untruncated rounds only
            assert pos == P + len(out) - 1
        fresh = m.new_cache(cache.max_seq)
        seq = list(p) + out[:-1]
        n = min(pos, len(seq))
        O.prefill(m, seq[:n], fresh)
        np.testing.assert_allclose(cache.k[:, :, :n], fresh.k[:, :, :n], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(cache.v[:, :, :n], fresh.v[:, :, :n], rtol=1e-9, atol=1e-12)
        seen.append(pos)

    s = O.self_speculative(m, p, 30, 2, 4, round_hook=hook)
    assert len(seen) == len(s.rounds) and seen == sorted(seen)
    for r0, r1 in zip(s.rounds, s.rounds[1:]):
        assert r1.pos == r0.pos + r0.n_accept + 1 and r1.last == r0.verify[r0.n_accept]


def test_acceptance_does_not_fall_with_deeper_exit(c1):
    """Trend the paper reports (Section 6.2, task-specific finetuning: acceptance grows with E)."""
    w, ws, p = c1
    acc = []
    for E in (1, 2, 3, 4):
        wE = W.make_weights(w, exit_layer=E)
        m = O.OracleModel(w.model, wE, np.float64)
        acc.append(O.self_speculative(m, p, 64, E, 4).acceptance)
    assert acc[-1] == 1.0 and acc[0] <= acc[1] + 0.05 <= acc[-1] + 0.1


# ---------------------------------------------------------------- the pins do catch mistakes
MISTAKES = {
    "rope sign": ("apply_rope", lambda y, c, s: np.concatenate(
        [y[..., :y.shape[-1] // 2] * c[:, None, :] + y[..., y.shape[-1] // 2:] * s[:, None, :],
         y[..., y.shape[-1] // 2:] * c[:, None, :] - y[..., :y.shape[-1] // 2] * s[:, None, :]], -1)),
    "norm drops gain": ("rmsnorm", lambda x, g, eps: x / np.sqrt(np.mean(x * x, -1, keepdims=True) + eps)),
    "norm drops eps": ("rmsnorm", lambda x, g, eps: x / np.sqrt(np.mean(x * x, -1, keepdims=True)) * g),
    "silu is sigmoid": ("silu", lambda z: 1.0 / (1.0 + np.exp(-z))),
    "softmax unnormalised": ("softmax_lastaxis", lambda s: np.exp(s - s.max(-1, keepdims=True))),
}


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistake_in_oracle_is_caught_by_brute_force_or_closed_forms(name, monkeypatch):
    """Plant one mistake in the cached decoder; the no-cache brute force (written separately)
    or the component closed forms must disagree."""
    import oracle.decoder as dec
    fn, bad = MISTAKES[name]
    w = W.get_workload("c1").with_(gain_jitter=0.2)
    ws, p = W.make_weights(w), W.make_prompt(w, 8)
    m = O.OracleModel(w.model, ws, np.float64)
    monkeypatch.setattr(dec, fn, bad)
    cache = m.new_cache(16)
    x = m.run_layers(m.embed_tokens(p), range(8), cache, 0, 2)
    monkeypatch.undo()
    ref = O.forward_nocache(m, p, n_layers=2)[0][-1]
    assert np.max(np.abs(x - ref)) > 1e-6


def test_bf16_rounding_noise_between_summation_orders():
    """With bf16-rounded activations the oracle is not reproducible to fp32 accuracy under a mere
    change of summation order: fp32 sums that differ in their last bits round to different bf16
    values in a few elements per row, and those units (2^-8 relative) reach the residual stream.
    This pins the size of that effect, which is what the bf16 hidden-state tolerance (2e-2 of the row
    maximum) and the near-tie rule for ids have to absorb: the same weights and inputs, with the
    feature axis of every weight matrix and its input permuted alike (the same sums, other order)."""
    cfg = W.ModelConfig(name="noise", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn_dim=1408,
                        vocab=1024, rope_base=10000.0, rms_eps=1e-5, dtype="bf16")
    w = W.Workload(cfg, exit_layer=2, draft_len=2, n_prompt=96, n_new=2, resid_scale=1.0)
    ws, prompt = W.make_weights(w), W.make_prompt(w)
    rng = np.random.default_rng(0)
    perm = {cfg.d_model: rng.permutation(cfg.d_model), cfg.ffn_dim: rng.permutation(cfg.ffn_dim)}

    def states(model):
        hid = []
        cache = model.new_cache(len(prompt) + 1)
        model.run_layers(model.embed_tokens(list(prompt)), list(range(len(prompt))), cache, 0, cfg.n_layers, hid)
        return hid

    a = O.OracleModel(cfg, ws, np.float32, emulate_bf16_act=True)
    b = O.OracleModel(cfg, ws, np.float32, emulate_bf16_act=True)

    class Reordered(np.ndarray):
        """Weight matrix whose products sum over the input features in a permuted order."""
        def __rmatmul__(self, x):                      # x @ W.T arrives here as x @ self
            p = perm[self.shape[0]]
            return np.asarray(x)[..., p] @ np.asarray(self)[p, :]

    for lw in b.layers:
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            wt = np.ascontiguousarray(lw[name].T).view(Reordered)   # [in, out]
            lw[name] = _TransposeProxy(wt)
    ha, hb = states(a), states(b)
    exact = O.OracleModel(cfg, ws, np.float64)
    he = states(exact)
    for l in range(cfg.n_layers):
        num = np.abs(ha[l] - hb[l]).max(axis=1)
        den = np.abs(ha[l]).max(axis=1)
        noise = float((num / den).max())
        vs_exact = float((np.abs(ha[l] - he[l]).max(axis=1) / np.abs(he[l]).max(axis=1)).max())
        assert 1e-4 < noise < 2e-2, (l, noise)         # far above fp32 rounding, inside the bf16 tolerance
        assert noise < 2.0 * vs_exact + 1e-3           # and no larger than bf16's own distance from exact arithmetic


class _TransposeProxy:
    """Stands in for a weight matrix W [out, in]: `x @ proxy.T` multiplies through the reordered copy."""
    def __init__(self, wt):
        self.T = wt
