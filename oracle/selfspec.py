"""CPU oracle: full-model greedy decoding and greedy self-speculative decoding.

TEST INFRASTRUCTURE ONLY (see decoder.py).

`greedy_full` is the plain definition of the result: autoregressive greedy decoding with
all L layers (the "Autoregressive" baseline of Section 6.2).

`self_speculative` takes the steps of Section 4.3 in the paper's order and notation:
  self-drafting (4.3.1): d tokens D_0..D_{d-1}, autoregressively, exiting at layer E;
  self-verification (4.3.2): the remaining L-E layers predict the next token for every
    draft position in ONE pass, continuing from the cached exit-layer states (4.3.3) and
    sharing the draft's KV cache; drafts up to the first disagreement are kept, then the
    verified token at the disagreement is appended;
  cache crop (Appendix A.4): the cache keeps (prompt + emitted - 1) positions, i.e. the
    last emitted token has not been through the model yet.
Readings taken where the paper leaves room:
  * verification consumes 1 + d rows (the round's input token and the d drafts): the appendix
    hands the remainder the round's input followed by the drafts; so the last draft needs its
    own early-layer pass (no LM head) and a round emits n+1 tokens, n = accepted drafts;
  * the cached "exit query" is the hidden state x_E of each drafted position;
  * the prompt is prefilled with the full model, whose greedy token is output #1;
  * the output is cut to exactly n_new tokens; acceptance counts the uncut n.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from .decoder import OracleModel, KVCache, argmax_lowest, top2_margin, runner_up


@dataclass
class RoundTrace:
    pos: int                   # cache length at the start of the round
    last: int                  # the round's input token (emitted, not yet in the cache)
    draft: List[int]
    verify: List[int]
    n_accept: int
    draft_margins: List[float]
    verify_margins: List[float]
    exit_layers: Optional[List[int]] = None   # per draft, when the exit layer is chosen per token
    draft_runner_up: Optional[List[int]] = None    # second-best token of each draft decision
    verify_runner_up: Optional[List[int]] = None   # ... of each verified decision


@dataclass
class DecodeResult:
    tokens: List[int]
    margins: List[float]                    # top-1 minus top-2 of the logits that chose each token
    rounds: List[RoundTrace] = field(default_factory=list)
    drafted: int = 0
    accepted: int = 0
    hidden: Optional[np.ndarray] = None     # [L+1, positions, d_model] when requested
    runner_up: List[int] = field(default_factory=list)   # second-best token of the decision behind each token

    @property
    def acceptance(self) -> float:
        return self.accepted / self.drafted if self.drafted else 0.0


def prefill(model: OracleModel, prompt, cache: KVCache, hidden=None):
    """All L layers over the prompt rows; returns the logits of the last row."""
    pos = list(range(len(prompt)))
    x = model.embed_tokens(prompt)
    if hidden is not None:
        hidden.append(x.copy())
    x = model.run_layers(x, pos, cache, 0, model.cfg.n_layers, hidden)
    return model.head(x[-1:])[0]


def greedy_full(model: OracleModel, prompt, n_new: int, max_seq: Optional[int] = None,
                want_hidden: bool = False) -> DecodeResult:
    """t_0 = argmax g(x_L[P-1]); t_k = argmax g(x_L) after feeding t_{k-1} at position P+k-1."""
    L = model.cfg.n_layers
    P = len(prompt)
    cache = model.new_cache(max_seq or (P + n_new + 1))
    hid = [] if want_hidden else None
    logits = prefill(model, prompt, cache, hid)
    per_pos = None
    if want_hidden:
        per_pos = [np.stack(hid, axis=0)]            # [L+1, P, dm]
    tokens, margins, second = [argmax_lowest(logits)], [top2_margin(logits)], [runner_up(logits)]
    while len(tokens) < n_new:
        t = P + len(tokens) - 1
        x = model.embed_tokens([tokens[-1]])
        h = [x.copy()] if want_hidden else None
        x = model.run_layers(x, [t], cache, 0, L, h)
        if want_hidden:
            per_pos.append(np.stack(h, axis=0))
        logits = model.head(x)[0]
        tokens.append(argmax_lowest(logits))
        margins.append(top2_margin(logits))
        second.append(runner_up(logits))
    res = DecodeResult(tokens, margins, runner_up=second)
    if want_hidden:
        res.hidden = np.concatenate(per_pos, axis=1)
    return res


def self_speculative(model: OracleModel, prompt, n_new: int, exit_layer: int, d: int,
                     max_seq: Optional[int] = None, round_hook=None, reuse: bool = True) -> DecodeResult:
    """Greedy self-speculative decoding, Section 4.3 / Appendix A.4.

    round_hook(cache, pos, out) is called after every round (tests use it to inspect the cache).
    reuse=False is the ablation of Section 4.3.3 / the cache-reuse table of the appendix: verification
    does not take the draft stage's exit states and early-layer cache, it runs all L layers over the
    round's 1+d tokens (and the last draft needs no early-layer pass of its own).
    """
    L, E = model.cfg.n_layers, exit_layer
    assert 1 <= E <= L and d >= 1
    P = len(prompt)
    cache = model.new_cache(max_seq or (P + n_new + d + 1))
    logits = prefill(model, prompt, cache)
    out, margins = [argmax_lowest(logits)], [top2_margin(logits)]
    pos, last = P, out[0]
    res = DecodeResult(out, margins, runner_up=[runner_up(logits)])
    while len(out) < n_new:
        # self-drafting: d early-exit steps; X[i] is the exit state x_E of the i-th row
        D, dm_, d2, X = [], [], [], []
        u = last
        for i in range(d):
            x = model.run_layers(model.embed_tokens([u]), [pos + i], cache, 0, E)
            X.append(x[0])
            lg = model.head(x)[0]                       # early exit: g(x_E)
            D.append(argmax_lowest(lg))
            dm_.append(top2_margin(lg))
            d2.append(runner_up(lg))
            u = D[-1]
        if reuse:
            # the last draft has not been an input yet: early layers only, no head
            x = model.run_layers(model.embed_tokens([D[-1]]), [pos + d], cache, 0, E)
            X.append(x[0])
            # self-verification: layers E..L-1 over the 1+d rows in one pass
            rows = np.stack(X, axis=0)
            xl = model.run_layers(rows, list(range(pos, pos + d + 1)), cache, E, L)
        else:
            xl = model.run_layers(model.embed_tokens([last] + D), list(range(pos, pos + d + 1)), cache, 0, L)
        lg = model.head(xl)
        V = [argmax_lowest(lg[i]) for i in range(d + 1)]
        vm = [top2_margin(lg[i]) for i in range(d + 1)]
        v2 = [runner_up(lg[i]) for i in range(d + 1)]
        # acceptance: longest prefix of drafts equal to the verified tokens
        n = 0
        while n < d and D[n] == V[n]:
            n += 1
        emitted = D[:n] + [V[n]]
        emitted_m = vm[:n + 1]
        res.rounds.append(RoundTrace(pos, last, D, V, n, dm_, vm, draft_runner_up=d2, verify_runner_up=v2))
        res.drafted += d
        res.accepted += n
        room = n_new - len(out)
        out.extend(emitted[:room])
        margins.extend(emitted_m[:room])
        res.runner_up.extend(v2[:n + 1][:room])
        pos += n + 1          # crop: positions beyond pos are dead and get overwritten
        last = V[n]
        if round_hook is not None:
            round_hook(cache, pos, list(out))
    return res


def self_speculative_dynamic(model: OracleModel, prompt, n_new: int, e_low: int, e_high: int, d: int,
                             tau: float, max_seq: Optional[int] = None) -> DecodeResult:
    """Self-speculative decoding with a per-token exit layer (the extension the paper's closing section
    names as future work: an exit layer chosen per token by a condition evaluated while decoding).

    The paper gives no algorithm; the reading taken here keeps everything of Section 4.3 and lets a
    draft leave at one of two layers:
      * a draft first exits at layer e_low; if the top-1 / top-2 logit margin of g(x_{e_low}) is at
        least tau, that prediction is the draft token;
      * otherwise the token continues through layers e_low..e_high-1 and g(x_{e_high}) drafts it.
        Layers e_low..e_high-1 need the keys and values of every earlier position, so the rows that
        left early since the last deep draft go through those layers in the same pass (one pass for
        several rows, like verification);
      * before verification the rows still pending (the last draft's row always is) are taken through
        layers e_low..e_high-1 in one pass; verification then is that of Section 4.3.2 from layer e_high.
    Every row ends up with exactly the states and cache entries of a fixed exit at e_high, whatever
    was decided along the way, so the output is full-model greedy as before; tau = +inf is
    `self_speculative(exit_layer=e_high)` and tau <= 0 drafts like `self_speculative(exit_layer=e_low)`.
    `rounds[k].exit_layers` records where each draft left.
    """
    L = model.cfg.n_layers
    assert 1 <= e_low < e_high <= L and d >= 1
    P = len(prompt)
    cache = model.new_cache(max_seq or (P + n_new + d + 1))
    logits = prefill(model, prompt, cache)
    out, margins = [argmax_lowest(logits)], [top2_margin(logits)]
    pos, last = P, out[0]
    res = DecodeResult(out, margins)
    while len(out) < n_new:
        D, dm_, exits = [], [], []
        X = [None] * (d + 1)       # row i: the state of the round's i-th token at the deepest layer it has reached
        j0 = 0                     # rows j0.. have only been through layers 0..e_low-1
        u = last

        def deepen(upto):
            rows = np.stack(X[j0:upto + 1], axis=0)
            y = model.run_layers(rows, list(range(pos + j0, pos + upto + 1)), cache, e_low, e_high)
            for k in range(j0, upto + 1):
                X[k] = y[k - j0]

        for i in range(d):
            X[i] = model.run_layers(model.embed_tokens([u]), [pos + i], cache, 0, e_low)[0]
            lg = model.head(X[i][None, :])[0]
            g = top2_margin(lg)
            if g >= tau:
                exits.append(e_low)
            else:
                deepen(i)
                j0 = i + 1
                lg = model.head(X[i][None, :])[0]
                g = top2_margin(lg)
                exits.append(e_high)
            D.append(argmax_lowest(lg))
            dm_.append(g)
            u = D[-1]
        X[d] = model.run_layers(model.embed_tokens([D[-1]]), [pos + d], cache, 0, e_low)[0]
        deepen(d)
        xl = model.run_layers(np.stack(X, axis=0), list(range(pos, pos + d + 1)), cache, e_high, L)
        lg = model.head(xl)
        V = [argmax_lowest(lg[i]) for i in range(d + 1)]
        vm = [top2_margin(lg[i]) for i in range(d + 1)]
        n = 0
        while n < d and D[n] == V[n]:
            n += 1
        emitted = D[:n] + [V[n]]
        tr = RoundTrace(pos, last, D, V, n, dm_, vm)
        tr.exit_layers = exits
        res.rounds.append(tr)
        res.drafted += d
        res.accepted += n
        room = n_new - len(out)
        out.extend(emitted[:room])
        margins.extend(vm[:n + 1][:room])
        pos += n + 1
        last = V[n]
    return res


def early_exit_greedy(model: OracleModel, prompt, n_new: int, exit_layer: int) -> DecodeResult:
    """Section 4.2 on its own: every token is argmax g(x_E); the late layers never run."""
    E, P = exit_layer, len(prompt)
    cache = model.new_cache(P + n_new + 1)
    x = model.run_layers(model.embed_tokens(prompt), list(range(P)), cache, 0, E)
    logits = model.head(x[-1:])[0]
    tokens, margins = [argmax_lowest(logits)], [top2_margin(logits)]
    while len(tokens) < n_new:
        t = P + len(tokens) - 1
        x = model.run_layers(model.embed_tokens([tokens[-1]]), [t], cache, 0, E)
        logits = model.head(x)[0]
        tokens.append(argmax_lowest(logits))
        margins.append(top2_margin(logits))
    return DecodeResult(tokens, margins)


def layer_probe(model: OracleModel, tokens):
    """The unembedding probe of Section 3: the shared head applied to the output of every layer.
    Returns (ids, margins), each [L][n]: ids[l][i] = argmax g(x_{l+1}) at row i of the causal sequence."""
    n = len(tokens)
    cache = model.new_cache(n + 1)
    hidden = []
    model.run_layers(model.embed_tokens(list(tokens)), list(range(n)), cache, 0, model.cfg.n_layers, hidden)
    ids, margins = [], []
    for x in hidden:
        lg = model.head(x)
        ids.append([argmax_lowest(lg[i]) for i in range(n)])
        margins.append([top2_margin(lg[i]) for i in range(n)])
    return ids, margins
