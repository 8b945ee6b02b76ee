"""The rule the GPU parity tests use to decide whether a differing token id is excusable
(tests/parity_util.py), checked on the CPU: which combinations pass and which do not."""
import pytest

from parity_util import excusable_flip, same_until_near_tie, NEAR_TIE, NOISE_BAND


def test_plain_rule_excludes_only_oracle_near_ties():
    assert excusable_flip(7, 0.5 * NEAR_TIE, None)
    assert not excusable_flip(7, 1.01 * NEAR_TIE, None)
    # the wide rule is off unless asked for, whatever else is known
    assert not excusable_flip(7, 1.5 * NEAR_TIE, 7, gpu_margin=0.0)


def test_wide_rule_needs_the_oracles_runner_up_and_the_noise_band():
    m = 1.5 * NEAR_TIE
    assert excusable_flip(7, m, 7, gpu_margin=0.5 * NEAR_TIE, wide=True)
    assert excusable_flip(7, m, 7, wide=True)                                       # gpu margin unknown
    assert not excusable_flip(8, m, 7, gpu_margin=0.0, wide=True)                   # not the runner-up
    assert not excusable_flip(7, NOISE_BAND, 7, gpu_margin=0.0, wide=True)          # outside the band
    assert not excusable_flip(7, m, 7, gpu_margin=2 * NEAR_TIE, wide=True)          # gpu is sure of it
    assert not excusable_flip(7, m, None, gpu_margin=0.0, wide=True)                # no oracle runner-up: plain rule


def test_a_gpu_side_tie_alone_never_excuses_a_flip():
    # the hole the rule used to have: a wrong id that merely sits on a tie of the GPU's own logits
    assert not excusable_flip(123, 2.0 * NEAR_TIE, 7, gpu_margin=0.0, wide=True)
    with pytest.raises(AssertionError):
        same_until_near_tie([1, 2, 123], [1, 2, 3], [1.0, 1.0, 2.0 * NEAR_TIE], runner_up=[0, 0, 7],
                            gpu_margins=[1.0, 1.0, 0.0])


def test_sequences_compare_up_to_the_first_excused_flip():
    assert same_until_near_tie([1, 2, 3], [1, 2, 3], [1.0, 1.0, 1.0]) == 3
    assert same_until_near_tie([1, 9, 3], [1, 2, 3], [1.0, 0.5 * NEAR_TIE, 1.0]) == 1
    assert same_until_near_tie([1, 7, 3], [1, 2, 3], [1.0, 1.5 * NEAR_TIE, 1.0], runner_up=[0, 7, 0],
                               gpu_margins=[1.0, 0.1 * NEAR_TIE, 1.0]) == 1
    with pytest.raises(AssertionError):
        same_until_near_tie([1, 9, 3], [1, 2, 3], [1.0, 1.5 * NEAR_TIE, 1.0])
