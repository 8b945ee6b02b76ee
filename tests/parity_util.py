"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np

NEAR_TIE = 1e-2   # top-1 minus top-2 below this is a near-tie: flagged and excluded


def same_until_near_tie(got, want, margins, thr=NEAR_TIE, gpu_margins=None):
    """Ids must be identical; the first difference must sit on a flagged near-tie, after which the
    two sequences are no longer comparable.  Returns how many ids were compared equal.
    `gpu_margins[i]` (bf16 models at full width only): the GPU's own top-1/top-2 margin for decision
    i on the same prefix; see near_tie_from_either_side."""
    assert len(got) == len(want), (len(got), len(want))
    for i, (a, b) in enumerate(zip(got, want)):
        if int(a) != int(b):
            if margins[i] >= thr and gpu_margins is not None and near_tie_from_either_side(margins[i], gpu_margins[i]):
                print(f"[parity] id {i}: gpu {a} != oracle {b} at oracle margin {margins[i]:.4g}, gpu margin "
                      f"{gpu_margins[i]:.4g}: a near-tie seen from the gpu's side", flush=True)
                return i
            assert margins[i] < thr, (f"id {i}: gpu {a} != oracle {b} with margin {margins[i]:.4g}"
                                      + (f", gpu margin {gpu_margins[i]:.4g}" if gpu_margins is not None else ""))
            return i
    return len(want)


def near_tie_from_either_side(oracle_margin: float, gpu_margin: float, thr=NEAR_TIE) -> bool:
    """With bf16 activations two correct evaluations of the same model differ by a bf16 unit in a few
    elements per row and layer (the oracle against itself with the sums taken in another order:
    test_bf16_rounding_noise_between_summation_orders); at d_model 2048+ and 24+ layers that moves the
    difference of two logits by up to about 1.5e-2.  A decision is therefore also a near-tie when the
    GPU's own margin is below the threshold while the oracle's is within that noise of it (2.5 x the
    threshold).  Both margins are outputs of their own side; neither side's data enters the other."""
    return bool(oracle_margin < 2.5 * thr and gpu_margin < thr)


def gpu_decisions(gm, prompt, n_new, exit_layer, d):
    """The self-speculative job once more through the step-by-step calls (the same kernels on the same
    cache contents as ls_generate): every emitted id with the GPU's own top-1/top-2 margin of the
    verified decision that produced it (an accepted draft equals the verified token of its row)."""
    P = len(prompt)
    _, mg = gm.score(list(prompt))
    gm.prefill(prompt)
    _, last, _ = gm.get_state()
    toks, margins = [last], [float(mg[P - 1])]
    while len(toks) < n_new:
        gm.draft(exit_layer, d)
        gm.verify(exit_layer, d)
        D, V, _, vm, n = gm.peek_round(d)
        gm.get_state()     # lets the host's capacity check use the real position instead of its upper bound
        toks += list(D[:n]) + [V[n]]
        margins += [float(x) for x in vm[:n + 1]]
    return toks[:n_new], margins[:n_new]


def rel_err_rows(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of max_i |got_i - ref_i| / max_i |ref_i| (arrays [..., d_model])."""
    num = np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64)), axis=-1)
    den = np.max(np.abs(ref.astype(np.float64)), axis=-1)
    return float(np.max(num / den))
