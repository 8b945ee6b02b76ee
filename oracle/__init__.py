"""Plain CPU oracle for greedy self-speculative decoding.  TEST INFRASTRUCTURE ONLY:
only tests/, the smoke check and the benchmark's CPU-baseline leg may import it.

Pins (tests/test_oracle_*.py, all run without a GPU): losslessness against full greedy,
E = L accepts every draft, zero residual scale gives the closed-form round count,
brute-force recomputation without a cache, cache contents after every crop, textbook
special cases and library routines for each component, hand-worked tiny models.
Not pinned (needs the paper's trained weights and datasets, which are absent): the
acceptance rates, ROUGE-2 and exact-match numbers of the paper's tables.
"""
from .decoder import (  # noqa: F401
    OracleModel, KVCache, rmsnorm, silu, softmax_lastaxis, rope_angles, apply_rope,
    argmax_lowest, top2_margin, runner_up, round_to_bf16, bf16_bits_to_float,
)
from .selfspec import (  # noqa: F401
    greedy_full, self_speculative, self_speculative_dynamic, early_exit_greedy, layer_probe, prefill,
    DecodeResult, RoundTrace,
)
from .bruteforce import forward_nocache, greedy_nocache  # noqa: F401
