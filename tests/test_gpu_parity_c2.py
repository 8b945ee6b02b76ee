"""GPU parity at full size: the 1.5B bf16 workload (24 layers, d_model 2048, prompt 512, 256 new
tokens, E=8, d=6) in the launch configuration bench.py times, against the CPU oracle run on the
same seeded weights with bf16-rounded activations.  Ids identical except at flagged near-ties
(oracle margin < 1e-2, or inside the bf16 noise band with the GPU's id equal to the oracle's
runner-up: parity_util.excusable_flip); teacher-forced argmax of every row; hidden states within 2e-2."""
import time

import numpy as np
import pytest

import oracle as O
import workloads as W
from parity_util import same_until_near_tie, check_hidden_full_width, excusable_flip, gpu_decisions, NEAR_TIE, MAX_NOISE_FLIPS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2():
    from paper_2404_16710_amd import LsModel
    w = W.get_workload("c2")
    t0 = time.time()
    ws, prompt = W.make_weights(w, threads=16), W.make_prompt(w)
    om = O.OracleModel(w.model, ws, np.float32, emulate_bf16_act=True)
    gm = LsModel(w.model, ws, max_seq=w.n_prompt + w.n_new + 17)
    print(f"[c2] weights + upload {time.time() - t0:.1f}s", flush=True)
    t0 = time.time()
    ref = O.self_speculative(om, prompt, w.n_new, w.exit_layer, w.draft_len)
    print(f"[c2] oracle self-speculative {time.time() - t0:.1f}s, acceptance {ref.acceptance:.3f}", flush=True)
    yield w, prompt, om, gm, ref
    gm.close()


def test_c2_generate_ids(c2):
    w, prompt, om, gm, ref = c2
    toks, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    ar, _ = gm.generate(prompt, w.n_new, 0, 0)
    stepped, gpu_margins = gpu_decisions(gm, prompt, w.n_new, w.exit_layer, w.draft_len)
    assert stepped == toks
    n = same_until_near_tie(toks, ref.tokens, ref.margins, runner_up=ref.runner_up, gpu_margins=gpu_margins)
    same_until_near_tie(ar, ref.tokens, ref.margins, runner_up=ref.runner_up, gpu_margins=gpu_margins)
    print(f"[c2] {n}/{w.n_new} ids compared before a near-tie; gpu acceptance {st.acceptance:.3f}", flush=True)
    assert toks == ar
    assert len(toks) == w.n_new
    if n == w.n_new:
        assert (st.rounds, st.accepted) == (len(ref.rounds), ref.accepted)


def test_c2_teacher_forced_and_hidden_states(c2):
    w, prompt, om, gm, ref = c2
    P = len(prompt)
    seq = list(prompt) + ref.tokens[:-1]
    cap = gm.debug_capture(True)
    am, mg = gm.score(seq)
    gm.debug_capture(False)
    firm = [i for i in range(w.n_new) if ref.margins[i] >= NEAR_TIE]
    flipped = [i for i in firm if am[P - 1 + i] != ref.tokens[i]]
    bad = [(i, int(am[P - 1 + i]), ref.tokens[i], ref.runner_up[i], float(ref.margins[i]), float(mg[P - 1 + i]))
           for i in flipped
           if not excusable_flip(am[P - 1 + i], ref.margins[i], ref.runner_up[i], mg[P - 1 + i], wide=True)]
    assert not bad, bad   # (position, gpu id, oracle id, oracle runner-up, oracle margin, gpu margin)
    assert len(flipped) <= MAX_NOISE_FLIPS, flipped     # such flips are rare
    print(f"[c2] ids differing at oracle margin in [1e-2, 2.5e-2) where the gpu chose the oracle's runner-up: "
          f"{[(i, round(float(ref.margins[i]), 4)) for i in flipped]}", flush=True)
    assert len(firm) >= int(0.8 * w.n_new)
    # hidden states of every layer at every position, from one oracle pass over the same sequence
    hid = []
    cache = om.new_cache(len(seq) + 1)
    x = om.embed_tokens(seq)
    om.run_layers(x, list(range(len(seq))), cache, 0, w.model.n_layers, hid)
    got = cap.cpu().numpy()
    worst = 0.0
    for l in range(w.model.n_layers):
        worst = max(worst, check_hidden_full_width(got[l, :len(seq)], hid[l], f"c2 layer {l}"))
    print(f"[c2] worst hidden-state error {worst:.2e}", flush=True)


def test_c2_round_replay(c2):
    w, prompt, om, gm, ref = c2
    E, d = w.exit_layer, w.draft_len
    checked = 0
    gpu_side_ties = 0
    for r in ref.rounds[:3] + ref.rounds[-2:]:
        seq = list(prompt) + ref.tokens[: r.pos - len(prompt)]
        gm.prefill(seq)
        pos, last, _ = gm.get_state()
        assert pos == r.pos
        if last != r.last:
            continue
        gm.draft(E, d)
        gm.verify(E, d)
        D, V, dmarg, _, n_acc = gm.peek_round(d)
        kd = next((i for i, g in enumerate(r.draft_margins) if g < NEAR_TIE), d)
        # bf16 rounding noise moves a margin by up to ~1.5e-2 at this width (pinned on the CPU in
        # test_oracle_invariants): a draft may differ where the oracle's margin is inside that band AND
        # the GPU drafted the oracle's runner-up AND the GPU's own margin is a near-tie
        kg = next((i for i in range(kd) if D[i] != r.draft[i]), kd)
        if kg < kd:
            assert excusable_flip(D[kg], r.draft_margins[kg], r.draft_runner_up[kg], dmarg[kg], wide=True), \
                (kg, D, r.draft, r.draft_runner_up, r.draft_margins, dmarg)
            gpu_side_ties += 1
            kd = kg
        assert D[:kd] == r.draft[:kd]
        for i in range(kd + 1 if kd < d else d + 1):
            if r.verify_margins[i] >= NEAR_TIE and D[:i] == r.draft[:i]:
                assert V[i] == r.verify[i]
                checked += 1
        if kd == d and all(g >= NEAR_TIE for g in r.verify_margins):
            assert n_acc == r.n_accept
    assert checked >= 3
    assert gpu_side_ties <= 1
