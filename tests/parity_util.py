"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np

NEAR_TIE = 1e-2   # top-1 minus top-2 below this is a near-tie: flagged and excluded


def same_until_near_tie(got, want, margins, thr=NEAR_TIE):
    """Ids must be identical; the first difference must sit on a flagged near-tie, after which the
    two sequences are no longer comparable.  Returns how many ids were compared equal."""
    assert len(got) == len(want), (len(got), len(want))
    for i, (a, b) in enumerate(zip(got, want)):
        if int(a) != int(b):
            assert margins[i] < thr, f"id {i}: gpu {a} != oracle {b} with margin {margins[i]:.4g}"
            return i
    return len(want)


def rel_err_rows(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of max_i |got_i - ref_i| / max_i |ref_i| (arrays [..., d_model])."""
    num = np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64)), axis=-1)
    den = np.max(np.abs(ref.astype(np.float64)), axis=-1)
    return float(np.max(num / den))
