"""GPU parity on small models: the HIP path through the C ABI against the CPU oracle, element by
element (token ids, per-round drafts / verified tokens / accepted counts, per-layer hidden
states).  Tolerances: ids identical except where the oracle's top-1/top-2 logit margin is below
1e-2 (flagged, excluded); hidden states within 1e-4 (fp32) or 2e-2 (bf16) of max|ref| per row."""
import numpy as np
import pytest

import oracle as O
import workloads as W
from parity_util import same_until_near_tie, rel_err_rows, NEAR_TIE

pytestmark = pytest.mark.gpu


def _tiny(dtype="f32", **kw):
    base = dict(name="tiny", n_layers=4, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=688,
                vocab=1024, rope_base=10000.0, rms_eps=1e-5, dtype=dtype)
    base.update(kw)
    return W.ModelConfig(**base)


def _setup(w, max_seq=None, emulate=None):
    from paper_2404_16710_amd import LsModel
    ws, prompt = W.make_weights(w), W.make_prompt(w)
    emu = (w.model.dtype == "bf16") if emulate is None else emulate
    om = O.OracleModel(w.model, ws, np.float32, emulate_bf16_act=emu)
    gm = LsModel(w.model, ws, max_seq=max_seq or (w.n_prompt + w.n_new + 16 + 1))
    return ws, prompt, om, gm


CASES = {
    "c1": W.get_workload("c1"),
    "c1-gains": W.get_workload("c1").with_(gain_jitter=0.2, weight_seed=3),
    "c1-bf16": W.get_workload("c1").with_(model=_tiny("bf16", name="c1-bf16"), gain_jitter=0.1),
    "gqa-hd128-bf16": W.Workload(_tiny("bf16", name="gqa", n_q_heads=4, n_kv_heads=1, head_dim=128, d_model=384,
                                       ffn_dim=1040, vocab=2064, n_layers=3),
                                 exit_layer=1, draft_len=5, n_prompt=70, n_new=40, resid_scale=0.1, gain_jitter=0.1),
    "gqa2-f32": W.Workload(_tiny("f32", name="gqa2", n_q_heads=8, n_kv_heads=4, head_dim=64, d_model=320,
                                 ffn_dim=848, vocab=1040, n_layers=3, rope_base=500000.0),
                           exit_layer=2, draft_len=3, n_prompt=19, n_new=30, resid_scale=0.05, gain_jitter=0.1),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_generate_matches_oracle_and_full_greedy(name):
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    ref = O.self_speculative(om, prompt, w.n_new, w.exit_layer, w.draft_len)
    toks, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    ar, st_ar = gm.generate(prompt, w.n_new, 0, 0)
    assert len(toks) == len(ar) == w.n_new and st.generated == w.n_new
    n = same_until_near_tie(toks, ref.tokens, ref.margins)
    same_until_near_tie(ar, ref.tokens, ref.margins)
    assert toks == ar                       # the GPU path is lossless against its own full greedy
    assert st_ar.rounds == 0 and st.drafted == st.rounds * w.draft_len
    # no divergence and no near-tie among the oracle's drafts (a draft that flips at a near-tie leaves
    # the tokens alone but changes how many are accepted): the round statistics must agree too
    tight = all(g >= NEAR_TIE for r in ref.rounds for g in r.draft_margins)
    if n == w.n_new and (tight or w.model.dtype == "f32"):
        assert (st.rounds, st.accepted) == (len(ref.rounds), ref.accepted)
    gm.close()


# Shapes whose many-row passes do not fit the LDS input region in one piece, so that the chunked
# forms of the matmul input run: the down projection's input (rows x ffn) goes through two half
# regions with the next chunk requested during the product of the current one; a normalised input
# (rows x d_model) is re-staged chunk by chunk.  d_model 4352 also gives a workgroup two tiles in the
# O / down projections (the form in which two tiles share the staged input).
CHUNKED = {
    "wide-ffn-bf16": W.Workload(_tiny("bf16", name="wide-ffn", n_layers=3, ffn_dim=4240), exit_layer=1, draft_len=15,
                                n_prompt=21, n_new=36, resid_scale=0.1, gain_jitter=0.1),
    "wide-ffn-f32": W.Workload(_tiny("f32", name="wide-ffn32", n_layers=3, ffn_dim=2128), exit_layer=2, draft_len=14,
                               n_prompt=21, n_new=36, resid_scale=0.05, gain_jitter=0.1),
    "wide-dm-bf16": W.Workload(_tiny("bf16", name="wide-dm", n_layers=2, d_model=4352, ffn_dim=528), exit_layer=1,
                               draft_len=15, n_prompt=18, n_new=34, resid_scale=0.1),
    "wide-dm-f32": W.Workload(_tiny("f32", name="wide-dm32", n_layers=2, d_model=2304, ffn_dim=528), exit_layer=1,
                              draft_len=15, n_prompt=18, n_new=34, resid_scale=0.05),
}


@pytest.mark.parametrize("name", sorted(CHUNKED))
def test_inputs_larger_than_the_lds_region_are_chunked_correctly(name):
    """16-row (or 15-row) verification passes whose matmul inputs exceed the LDS region, against the
    oracle: ids, round statistics where no near-tie interferes, hidden states of every position, and
    bit-identical ids from one-row passes (full greedy), where nothing is chunked."""
    w = CHUNKED[name]
    ws, prompt, om, gm = _setup(w)
    ref = O.self_speculative(om, prompt, w.n_new, w.exit_layer, w.draft_len)
    cap = gm.debug_capture(True)
    toks, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    hid = cap.cpu().numpy().copy()
    gm.debug_capture(False)
    ar, _ = gm.generate(prompt, w.n_new, 0, 0)
    n = same_until_near_tie(toks, ref.tokens, ref.margins)
    assert toks == ar and len(toks) == w.n_new
    assert st.drafted == st.rounds * w.draft_len
    full = O.greedy_full(om, prompt, w.n_new, want_hidden=True)
    tol = 2e-2 if w.model.dtype == "bf16" else 1e-4
    P = len(prompt)
    rows = P + min(n, w.n_new - 1)          # positions whose input tokens agree with the oracle's
    for l in range(w.model.n_layers):
        assert rel_err_rows(hid[l, :rows], full.hidden[l + 1][:rows]) < tol, l
    # the ablation runs all layers over 16 rows from the embedding table (the normalised input of the
    # first layer then comes from embedding rows)
    abl, st_abl = gm.generate_no_reuse(prompt, w.n_new, w.exit_layer, w.draft_len)
    assert abl == toks and (st_abl.rounds, st_abl.accepted) == (st.rounds, st.accepted)
    gm.close()


@pytest.mark.parametrize("name", ["c1", "c1-bf16", "gqa-hd128-bf16"])
def test_teacher_forced_scores_match_oracle(name):
    """Full-model argmax of every row of prompt+output, given the oracle's own sequence: covers every
    position regardless of where a free-running comparison would diverge."""
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    ref = O.greedy_full(om, prompt, w.n_new, want_hidden=True)
    seq = list(prompt) + ref.tokens[:-1]
    cap = gm.debug_capture(True)
    am, mg = gm.score(seq)
    P = len(prompt)
    bad = [i for i in range(w.n_new) if am[P - 1 + i] != ref.tokens[i] and ref.margins[i] >= NEAR_TIE]
    assert not bad, bad
    firm = [i for i in range(w.n_new) if ref.margins[i] >= NEAR_TIE]
    assert len(firm) > w.n_new // 2
    np.testing.assert_allclose(mg[P - 1:][firm], np.array(ref.margins)[firm], rtol=0.05, atol=2e-3)
    hid = cap.cpu().numpy()[:, :len(seq), :]                       # x_1..x_L
    tol = 2e-2 if w.model.dtype == "bf16" else 1e-4
    for l in range(w.model.n_layers):
        assert rel_err_rows(hid[l], ref.hidden[l + 1]) < tol, l
    gm.close()


@pytest.mark.parametrize("name,E,d", [("c1", 2, 4), ("c1", 1, 1), ("c1", 4, 15), ("c1", 3, 7),
                                      ("c1-bf16", 2, 6), ("gqa-hd128-bf16", 2, 12)])
def test_rounds_replayed_from_oracle_state(name, E, d):
    """ls_prefill / ls_draft / ls_verify from the oracle's state at each round: drafts, verified
    tokens, accepted count and the new state must be the oracle's (near-ties excluded)."""
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    if E != w.exit_layer:
        ws = W.make_weights(w, exit_layer=E)
        om = O.OracleModel(w.model, ws, np.float32, emulate_bf16_act=(w.model.dtype == "bf16"))
        from paper_2404_16710_amd import LsModel
        gm.close()
        gm = LsModel(w.model, ws, max_seq=w.n_prompt + w.n_new + 17)
    ref = O.self_speculative(om, prompt, min(w.n_new, 40), E, d)
    checked = 0
    for r in ref.rounds[:6]:
        seq = list(prompt) + ref.tokens[: r.pos - len(prompt)]
        gm.prefill(seq)
        pos, last, n_gen = gm.get_state()
        assert pos == r.pos and n_gen == 1
        if last != r.last:
            continue                                              # prefill token sat on a near-tie
        gm.draft(E, d)
        gm.verify(E, d)
        D, V, dmg, vmg, n_acc = gm.peek_round(d)
        # draft i is comparable while every earlier draft margin was firm; verified row i needs the
        # same inputs (last, D_0..D_{i-1}) and a firm margin of its own
        kd = next((i for i, g in enumerate(r.draft_margins) if g < NEAR_TIE), d)
        assert D[:kd] == r.draft[:kd]
        checked += kd
        for i in range(min(kd, d) + 1):
            if r.verify_margins[i] >= NEAR_TIE and D[:i] == r.draft[:i]:
                assert V[i] == r.verify[i], (i, V, r.verify)
                checked += 1
        if kd == d and all(g >= NEAR_TIE for g in r.verify_margins):
            assert V == r.verify and n_acc == r.n_accept
            pos2, last2, n_gen2 = gm.get_state()
            assert (pos2, last2, n_gen2) == (r.pos + r.n_accept + 1, r.verify[r.n_accept], 1 + r.n_accept + 1)
    assert checked >= 1
    gm.close()


@pytest.mark.parametrize("name", ["c1", "c1-bf16", "gqa-hd128-bf16"])
@pytest.mark.parametrize("max_seq", [4096 + 512, 20000])
def test_large_cache_capacity_groups_attention_tiles(name, max_seq):
    """With a large KV capacity one attention work item walks several 64-position tiles with a
    running softmax (16-bit models: in the MFMA accumulators of each wave; the grouped-query case
    has 24 query rows per KV head in its verify pass, i.e. two blocks of 16); the result must not
    change."""
    w = CASES[name].with_(n_prompt=150, n_new=40)
    ws, prompt, om, gm = _setup(w, max_seq=max_seq)
    ref = O.greedy_full(om, prompt, w.n_new, want_hidden=True)
    toks, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    ar, _ = gm.generate(prompt, w.n_new, 0, 0)
    same_until_near_tie(toks, ref.tokens, ref.margins)
    assert toks == ar
    cap = gm.debug_capture(True)
    seq = list(prompt) + ref.tokens[:-1]
    gm.score(seq)
    hid = cap.cpu().numpy()[:, :len(seq), :]
    tol = 2e-2 if w.model.dtype == "bf16" else 1e-4
    for l in range(w.model.n_layers):
        assert rel_err_rows(hid[l], ref.hidden[l + 1]) < tol, l
    gm.debug_capture(False)
    gm.close()


@pytest.mark.parametrize("name", ["c1", "c1-bf16", "gqa-hd128-bf16"])
@pytest.mark.parametrize("max_seq", [256, 4096 + 512])
def test_both_cache_policies_of_the_attention_stage_give_the_same_tokens(name, max_seq):
    """The attention stage exists once per way of reading settled K/V tiles (through the caches, or with
    coherent loads) and per item shape (one tile, or several): the library picks by cache size, the test
    forces each policy on a short and on a long cache.  Same bytes, same arithmetic: identical ids, and
    the self-speculative ids equal the full-greedy ids under either."""
    w = CASES[name].with_(n_prompt=150, n_new=40)
    ws, prompt, om, gm = _setup(w, max_seq=max_seq)
    ref = O.greedy_full(om, prompt, w.n_new)
    outs = []
    for policy in (1, 2, 0):
        gm.debug_kv_policy(policy)
        toks, _ = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
        ar, _ = gm.generate(prompt, w.n_new, 0, 0)
        assert toks == ar, policy
        outs.append(toks)
    assert outs[0] == outs[1] == outs[2]
    same_until_near_tie(outs[0], ref.tokens, ref.margins)
    gm.close()


@pytest.mark.parametrize("name,n_prompt", [("c1", 150), ("c1-bf16", 131), ("gqa-hd128-bf16", 257), ("gqa2-f32", 64),
                                           ("c1", 2100), ("gqa-hd128-bf16", 2085)])   # the last two: more than one chunk of 2048 prompt rows
def test_prefill_hidden_states_and_cache(name, n_prompt):
    """ls_prefill (the GEMM prompt pass for these lengths): per-layer hidden states of every prompt
    row, the first token, and - through one draft/verify round on top of it - the KV cache."""
    w = CASES[name].with_(n_prompt=n_prompt)
    ws, prompt, om, gm = _setup(w, max_seq=n_prompt + 64)
    hid = []
    cache = om.new_cache(n_prompt + 64)
    x = om.embed_tokens(prompt)
    xl = om.run_layers(x, list(range(n_prompt)), cache, 0, w.model.n_layers, hid)
    logits = om.head(xl[-1:])[0]
    cap = gm.debug_capture(True)
    gm.prefill(prompt)
    pos, last, n_gen = gm.get_state()
    assert (pos, n_gen) == (n_prompt, 1)
    if O.top2_margin(logits) >= NEAR_TIE:
        assert last == O.argmax_lowest(logits)
    got = cap.cpu().numpy()[:, :n_prompt, :]
    tol = 2e-2 if w.model.dtype == "bf16" else 1e-4
    for l in range(w.model.n_layers):
        assert rel_err_rows(got[l], hid[l]) < tol, l
    gm.debug_capture(False)
    ref = O.self_speculative(om, prompt, 8, w.exit_layer, w.draft_len)
    if last == ref.tokens[0]:
        r = ref.rounds[0]
        gm.draft(w.exit_layer, w.draft_len)
        gm.verify(w.exit_layer, w.draft_len)
        D, V, _, _, n_acc = gm.peek_round(w.draft_len)
        kd = next((i for i, g in enumerate(r.draft_margins) if g < NEAR_TIE), w.draft_len)
        assert D[:kd] == r.draft[:kd]
        if r.verify_margins[0] >= NEAR_TIE:
            assert V[0] == r.verify[0]
    gm.close()


WIDE160 = W.Workload(_tiny("bf16", name="wide160", n_q_heads=5, n_kv_heads=5, head_dim=128, d_model=640, ffn_dim=1296,
                           vocab=1040, n_layers=3),
                     exit_layer=1, draft_len=4, n_prompt=300, n_new=20, resid_scale=0.1, gain_jitter=0.1)


@pytest.mark.parametrize("name", ["c1", "c1-bf16", "gqa-hd128-bf16", "gqa2-f32", "wide160-bf16"])
def test_every_prompt_pass_shape_matches_oracle(name):
    """ls_set_prompt_tiles: the prompt GEMMs with 128-, 64- and 32-row output tiles, with 64 x 160 tiles
    in the products into the residual rows (d_model 320 and 640 are multiples of 160; elsewhere the
    setting falls back to 64 x 128), and the 16-row passes of the decode kernel, each forced on a prompt
    that spans several tiles of every height with a ragged last one
    (300 = 2 x 128 + 44 = 4 x 64 + 44 = 9 x 32 + 12 = 18 x 16 + 12)."""
    n_prompt = 300
    w = (WIDE160 if name == "wide160-bf16" else CASES[name]).with_(n_prompt=n_prompt)
    ws, prompt, om, gm = _setup(w, max_seq=n_prompt + 64)
    hid = []
    cache = om.new_cache(n_prompt + 64)
    xl = om.run_layers(om.embed_tokens(prompt), list(range(n_prompt)), cache, 0, w.model.n_layers, hid)
    logits = om.head(xl[-1:])[0]
    tol = 2e-2 if w.model.dtype == "bf16" else 1e-4
    ref = O.self_speculative(om, prompt, 12, w.exit_layer, w.draft_len)
    cap = gm.debug_capture(True)
    from paper_2404_16710_amd.binding import LsError
    with pytest.raises(LsError):
        gm.set_prompt_tiles(48)
    for rows in (128, 64, 160, 32, 16, 0):
        print(f"[prompt tiles] {name} rows {rows}", flush=True)
        gm.set_prompt_tiles(rows)
        cap.zero_()
        gm.prefill(prompt)
        pos, last, n_gen = gm.get_state()
        assert (pos, n_gen) == (n_prompt, 1)
        if O.top2_margin(logits) >= NEAR_TIE:
            assert last == O.argmax_lowest(logits), rows
        got = cap.cpu().numpy()[:, :n_prompt, :]
        for l in range(w.model.n_layers):
            assert rel_err_rows(got[l], hid[l]) < tol, (rows, l)
        toks, _ = gm.generate(prompt, 12, w.exit_layer, w.draft_len)      # the same prompt pass, then decoding
        same_until_near_tie(toks, ref.tokens, ref.margins)
    gm.close()


def test_exit_at_last_layer_accepts_everything_on_gpu():
    w = CASES["c1"]
    ws, prompt, om, gm = _setup(w)
    L = w.model.n_layers
    toks, st = gm.generate(prompt, 41, L, 5)
    assert st.accepted == st.drafted and st.rounds == (41 - 1 + 5) // 6
    ar, _ = gm.generate(prompt, 41, 0, 0)
    assert toks == ar
    gm.close()


def test_early_exit_generation_matches_oracle():
    w = CASES["c1"]
    ws, prompt, om, gm = _setup(w)
    ref = O.early_exit_greedy(om, prompt, 32, 2)
    toks, _ = gm.generate_early_exit(prompt, 32, 2)
    same_until_near_tie(toks, ref.tokens, ref.margins)
    gm.close()


@pytest.mark.parametrize("n_prompt", [1, 15, 16, 17, 33])
def test_ragged_prompt_lengths(n_prompt):
    w = CASES["c1"].with_(n_prompt=n_prompt, n_new=12)
    ws, prompt, om, gm = _setup(w)
    ref = O.greedy_full(om, prompt, 12)
    toks, _ = gm.generate(prompt, 12, 2, 4)
    same_until_near_tie(toks, ref.tokens, ref.margins)
    gm.close()


def test_eos_stops_generation_and_output_tail_is_padded():
    w = CASES["c1"]
    ws, prompt, om, gm = _setup(w)
    full, _ = gm.generate(prompt, 30, 0, 0)
    eos = full[7]
    first = full.index(eos)
    toks, st = gm.generate(prompt, 30, 2, 4, eos_id=eos)
    assert toks == full[: first + 1] and st.generated == first + 1
    gm.close()


def test_argument_errors_leave_no_work():
    from paper_2404_16710_amd import LsError
    w = CASES["c1"]
    ws, prompt, om, gm = _setup(w, max_seq=64)
    with pytest.raises(LsError) as e:
        gm.draft(2, 4)
    assert e.value.code == -4                                      # draft before prefill
    gm.prefill(prompt)
    with pytest.raises(LsError) as e:
        gm.verify(2, 4)
    assert e.value.code == -4                                      # verify without draft
    with pytest.raises(LsError) as e:
        gm.draft(0, 4)
    assert e.value.code == -2
    with pytest.raises(LsError) as e:
        gm.draft(5, 4)
    assert e.value.code == -2
    with pytest.raises(LsError) as e:
        gm.generate(prompt, 64, 2, 4)
    assert e.value.code == -3                                      # would not fit max_seq
    gm.draft(2, 4)
    with pytest.raises(LsError) as e:
        gm.verify(2, 3)                                            # d differs from the draft
    assert e.value.code == -4
    gm.verify(2, 4)
    pos, last, n_gen = gm.get_state()
    assert n_gen >= 2 and pos == len(prompt) + n_gen - 1
    gm.close()


def test_read_only_stream_reference_reads_every_byte_once():
    """The measurement aid ls_debug_read folds all it reads into 16 bytes per thread with xor: the
    xor over its sink equals the xor over the source's 16-byte units, for both launch shapes."""
    import ctypes
    import torch
    from paper_2404_16710_amd import binding as B
    lib = B.lib()
    g = torch.Generator().manual_seed(5)
    src_h = torch.randint(-2**31, 2**31 - 1, (1 << 23,), dtype=torch.int32, generator=g)   # 32 MiB
    want = src_h.view(-1, 4).numpy()
    want = np.bitwise_xor.reduce(want, axis=0)
    src = src_h.to("cuda:0")
    for wg in (256, 512):
        sink = torch.zeros(wg * 1024, dtype=torch.int32, device="cuda:0")
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        assert lib.ls_debug_read(ctypes.c_void_p(src.data_ptr()), src.numel() * 4, ctypes.c_void_p(sink.data_ptr()), wg, stream) == 0
        torch.cuda.synchronize()
        got = np.bitwise_xor.reduce(sink.cpu().view(-1, 4).numpy(), axis=0)
        assert (got == want).all(), wg


def test_expired_wait_is_reported_and_the_next_prompt_recovers():
    """Failure handling, forced from the host: with a limit of one poll per wait some workgroup
    gives up at once, every workgroup then leaves (no kernel hangs or faults), the call reports
    LS_E_DEVICE, and after the limit is restored the same context generates the right tokens again."""
    from paper_2404_16710_amd.binding import LsError
    w = CASES["c1"]
    ws, prompt, om, gm = _setup(w)
    want, _ = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    gm.debug_spin_limit(1)
    with pytest.raises(LsError) as ei:
        gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    assert ei.value.code == -6
    gm.debug_spin_limit(0)
    got, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    assert got == want and st.generated == w.n_new
    gm.close()


@pytest.mark.parametrize("name", ["c1", "gqa-hd128-bf16", "gqa2-f32"])
def test_generation_without_cache_reuse_matches(name):
    """ls_generate_no_reuse (ablation of Section 4.3.3): verification recomputes the early layers of the
    round's rows.  The rows of a pass do not influence each other's arithmetic, so tokens and round
    statistics are those of ls_generate exactly; against the oracle's own no-reuse loop up to near-ties."""
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    toks, st = gm.generate(prompt, w.n_new, w.exit_layer, w.draft_len)
    got, sn = gm.generate_no_reuse(prompt, w.n_new, w.exit_layer, w.draft_len)
    assert got == toks
    assert (sn.rounds, sn.drafted, sn.accepted, sn.generated) == (st.rounds, st.drafted, st.accepted, st.generated)
    ref = O.self_speculative(om, prompt, w.n_new, w.exit_layer, w.draft_len, reuse=False)
    same_until_near_tie(got, ref.tokens, ref.margins)
    gm.close()


@pytest.mark.parametrize("name", ["c1", "gqa-hd128-bf16", "gqa2-f32"])
def test_per_token_exit_layer_matches(name):
    """ls_generate_dynamic (a draft leaves at the lower of two exit layers when its margin reaches tau):
    the tokens are those of ls_generate exactly, whatever tau; tau = inf reproduces ls_generate's rounds;
    tau = 0 those of ls_generate at the lower exit; in between, the exit layers agree with the oracle's
    as long as the sequences agree and no margin sits within the near-tie distance of tau."""
    import math
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    L = w.model.n_layers
    e_high = max(2, w.exit_layer)
    e_low = e_high - 1
    d = w.draft_len
    assert e_high < L or e_high == L
    toks, st = gm.generate(prompt, w.n_new, e_high, d)
    t_inf, s_inf, ex_inf, low_inf = gm.generate_dynamic(prompt, w.n_new, e_low, e_high, d, math.inf)
    assert t_inf == toks and (s_inf.rounds, s_inf.accepted) == (st.rounds, st.accepted)
    assert low_inf == 0 and all(e == e_high for r in ex_inf for e in r)
    t_lo, s_lo = gm.generate(prompt, w.n_new, e_low, d)
    t_0, s_0, ex_0, low_0 = gm.generate_dynamic(prompt, w.n_new, e_low, e_high, d, 0.0)
    assert t_0 == toks == t_lo and (s_0.rounds, s_0.accepted) == (s_lo.rounds, s_lo.accepted)
    assert low_0 == s_0.drafted and all(e == e_low for r in ex_0 for e in r)
    ref_lo = O.self_speculative(om, prompt, w.n_new, e_low, d)
    margins = sorted(x for t in ref_lo.rounds for x in t.draft_margins)
    tau = float(margins[len(margins) // 2])
    ref = O.self_speculative_dynamic(om, prompt, w.n_new, e_low, e_high, d, tau)
    got, sg, ex, low = gm.generate_dynamic(prompt, w.n_new, e_low, e_high, d, tau)
    assert got == toks                                   # lossless against the GPU's own greedy path
    same_until_near_tie(got, ref.tokens, ref.margins)
    assert 0 < low < sg.drafted and low == sum(e == e_low for r in ex for e in r)
    # round by round while both sides are in the same state and decide far from the threshold
    # draft by draft while both sides are in the same state and the oracle decides far from the
    # threshold and far from a tie (after the first decision that may differ, nothing is comparable)
    eps = 1e-4 if w.model.dtype == "f32" else NEAR_TIE
    compared, comparable = 0, True
    for k, t in enumerate(ref.rounds):
        if not comparable or k >= len(ex):
            break
        for i in range(d):
            if abs(t.draft_margins[i] - tau) < eps or t.draft_margins[i] < eps:
                comparable = False
                break
            assert ex[k][i] == t.exit_layers[i], (k, i, ex[k], t.exit_layers)
            compared += 1
        comparable = comparable and all(mg >= eps for mg in t.verify_margins)
    assert compared >= 1
    gm.close()


@pytest.mark.parametrize("name", ["c1", "c1-bf16", "gqa2-f32"])
def test_layer_probe_matches_oracle(name):
    """ls_probe_layers: argmax of g(x_l) after every layer for every row of a 40-token sequence (two
    full 16-row passes and a ragged one), against the oracle's probe; near-ties excluded."""
    w = CASES[name]
    ws, prompt, om, gm = _setup(w)
    seq = (list(prompt) * 2)[:40]
    am, mg = gm.probe_layers(seq)
    ids, margins = O.layer_probe(om, seq)
    L = w.model.n_layers
    assert am.shape == (L, len(seq))
    firm = 0
    for l in range(L):
        for i in range(len(seq)):
            if margins[l][i] >= NEAR_TIE:
                firm += 1
                assert am[l][i] == ids[l][i], (l, i, margins[l][i], mg[l][i])
    assert firm > L * len(seq) // 2
    full, _ = gm.score(seq)
    assert list(am[L - 1]) == list(full)          # the last layer's probe is the full model, bit for bit
    gm.close()
