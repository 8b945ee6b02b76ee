"""GPU parity at the widths of the larger workloads (7B MHA with a 1536-id prompt, 8B grouped-query
with a 128k vocabulary; the 13B shape by properties only), in the launch configuration bench.py
uses for them.  The oracle runs on the same seeded weights with bf16-rounded activations for a
bounded sample: every prompt row's hidden state in every layer, and the first ids of the
self-speculative job.  Properties that need no oracle cover the whole job: the self-speculative ids
equal the GPU's own full greedy ids, and an exit at the last layer accepts every draft."""
import time

import numpy as np
import pytest

import oracle as O
import workloads as W
from parity_util import same_until_near_tie, rel_err_rows, gpu_decisions, NEAR_TIE

pytestmark = pytest.mark.gpu

N_REF = 12     # ids the oracle generates (a 7B oracle step streams 27 GB of fp32 weights on the host)


def _models(name, with_oracle):
    from paper_2404_16710_amd import LsModel
    w = W.get_workload(name)
    t0 = time.time()
    ws, prompt = W.make_weights(w, threads=16), W.make_prompt(w)
    om = O.OracleModel(w.model, ws, np.float32, emulate_bf16_act=True) if with_oracle else None
    gm = LsModel(w.model, ws, max_seq=w.n_prompt + w.n_new + 17)
    print(f"[{name}] weights + upload {time.time() - t0:.1f}s", flush=True)
    return w, prompt, om, gm


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_large_width_prompt_states_and_first_ids(name):
    w, prompt, om, gm = _models(name, True)
    P, L, E, d = len(prompt), w.model.n_layers, w.exit_layer, w.draft_len
    t0 = time.time()
    ref = O.self_speculative(om, prompt, N_REF, E, d)
    hid = []
    om.run_layers(om.embed_tokens(prompt), list(range(P)), om.new_cache(P + 1), 0, L, hid)
    print(f"[{name}] oracle: {N_REF} ids and the prompt's hidden states {time.time() - t0:.1f}s", flush=True)

    cap = gm.debug_capture(True)
    toks, st = gm.generate(prompt, w.n_new, E, d)
    got = cap.cpu().numpy()
    gm.debug_capture(False)
    worst = 0.0
    for l in range(L):
        e = rel_err_rows(got[l, :P], hid[l])
        worst = max(worst, e)
        assert e < 2e-2, (l, e)
    print(f"[{name}] worst prompt hidden-state error {worst:.2e}", flush=True)
    stepped, gpu_margins = gpu_decisions(gm, prompt, N_REF, E, d)
    assert stepped == toks[:N_REF]
    n = same_until_near_tie(toks[:N_REF], ref.tokens, ref.margins, gpu_margins=gpu_margins)
    print(f"[{name}] {n}/{N_REF} ids compared before a near-tie; gpu acceptance {st.acceptance:.3f}", flush=True)
    assert n >= 1
    ar, st_ar = gm.generate(prompt, w.n_new, 0, 0)
    assert toks == ar and len(toks) == w.n_new and st_ar.rounds == 0
    gm.close()


def test_13b_width_is_lossless_against_its_own_full_greedy():
    w, prompt, _, gm = _models("c5", False)
    L, E, d = w.model.n_layers, w.exit_layer, w.draft_len
    n_new = 48
    ar, _ = gm.generate(prompt, n_new, 0, 0)
    toks, st = gm.generate(prompt, n_new, E, d)
    assert toks == ar and st.drafted == st.rounds * d
    full, st_full = gm.generate(prompt, n_new, L, d)
    assert full == ar and st_full.accepted == st_full.drafted
    ablated, st_abl = gm.generate_no_reuse(prompt, n_new, E, d)
    assert ablated == ar and (st_abl.rounds, st_abl.accepted) == (st.rounds, st.accepted)
    gm.close()
