"""ls_generate_static (the entry point that allocates no device memory: its workspace is a fixed array
inside the library) against ls_generate with a caller-owned workspace, through the C ABI: two calls in
a row on the same GPU, the second with a smaller model configuration, prompt and token budget, so that
it runs on top of whatever the first call left in the array.  Token ids and round counters must be
identical (integer results: bit-exact)."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _reference(w, ws, prompt, max_seq, n_new, E, d):
    from paper_2404_16710_amd import LsModel
    m = LsModel(w.model, ws, max_seq=max_seq)
    toks, st = m.generate(prompt, n_new, E, d)
    m.close()
    return toks, st


def test_static_workspace_generation_matches_the_caller_workspace_one():
    import torch
    from paper_2404_16710_amd import DeviceWeights, generate_static, LsError
    w = W.get_workload("c1")
    ws, prompt = W.make_weights(w), W.make_prompt(w)
    dw = DeviceWeights(w.model, ws, torch.device("cuda:0"))
    # first call: the whole tiny workload
    seq1 = w.n_prompt + w.n_new + w.draft_len + 1
    want1, st1 = _reference(w, ws, prompt, seq1, w.n_new, w.exit_layer, w.draft_len)
    got1, gs1 = generate_static(w.model, dw, seq1, prompt, w.n_new, w.exit_layer, w.draft_len)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]     # (the first call made the runtime place the library's array)
    assert got1 == want1 and len(got1) == w.n_new
    assert (gs1.rounds, gs1.drafted, gs1.accepted, gs1.generated) == (st1.rounds, st1.drafted, st1.accepted, st1.generated)
    # second call, smaller: shorter prompt, fewer tokens, shorter drafts and a smaller cache, hence another
    # workspace layout laid over the first call's leftovers
    p2, n2, d2 = prompt[:11], 23, 3
    seq2 = len(p2) + n2 + d2 + 1
    got2, gs2 = generate_static(w.model, dw, seq2, p2, n2, w.exit_layer, d2)
    # full-model greedy through the same entry point (d = 0)
    got3, _ = generate_static(w.model, dw, seq2, p2, n2, 0, 0)
    torch.cuda.synchronize()
    free1 = torch.cuda.mem_get_info()[0]
    # calls after the first take no device memory (the binding's token buffers come from torch's cached pool)
    assert free0 - free1 < (1 << 20), (free0, free1)
    want2, st2 = _reference(w, ws, p2, seq2, n2, w.exit_layer, d2)
    assert got2 == want2 and len(got2) == n2
    assert (gs2.rounds, gs2.drafted, gs2.accepted, gs2.generated) == (st2.rounds, st2.drafted, st2.accepted, st2.generated)
    assert got3 == want2      # the same ids without drafts
    # a model that does not fit the array is refused with the capacity error
    big = W.get_workload("c2")
    with pytest.raises(LsError) as e:
        generate_static(big.model, dw, 785, prompt, 8, 2, 2)
    assert e.value.code == -3
