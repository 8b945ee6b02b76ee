"""Per-stage timeline of the persistent decode kernel, from the events one workgroup records when
`ls_debug_timeline` is armed (a 100 MHz wall-clock reading and a tag per event, kept in LDS while the
kernel runs).  Prints, for one-row passes (draft steps, plain decoding) and for the (d+1)-row
verification pass, the average duration of every stage of a layer split into barrier wait, input
fetch, weight stream + products and epilogue, and the rate of the weight stream.

    python -m paper_2404_16710_amd.stage_timeline --config c2 [--workgroup 100]

Event tags (ls_kernels.inc): stage starts 0x10 QKV, 0x20 attention, 0x30 O projection, 0x40 gate/up,
0x50 down projection, 0x60 head, 0x70 candidate reduction; +1 barrier arrival signalled and first weight
loads issued, +2 barrier passed; 0x80 input rows staged in LDS, 0x81 products of a tile group done;
+4 group done, +5 epilogue stores issued, +6 stores drained; attention: 0x23 K/V and q requested,
0x24 q staged, 0x27 tiles folded, 0x28 partial stored, 0x29 counter known, 0x25 merged;
0x90 / 0x91 a one-row / many-row pass starts.
"""
import argparse
import collections

import numpy as np

import workloads as W
from .binding import LsModel

STAGES = [("QKV + RoPE + cache append", 0x10), ("attention", 0x20), ("O projection + residual", 0x30),
          ("gate/up + SwiGLU", 0x40), ("down projection + residual", 0x50)]


def _events(model, n_events, wg, run, before=None):
    if before is not None:
        before()                                   # work whose events are not wanted
    tl = model.debug_timeline(n_events, wg)
    run()
    ev = tl.cpu().numpy().astype(np.uint64)
    ev = ev[ev != 0]
    t = (ev >> np.uint64(8)).astype(np.int64) * 0.01          # microseconds
    tag = (ev & np.uint64(0xFF)).astype(np.int64)
    brk = np.where(np.diff(t) < 0)[0]
    if len(brk):
        t, tag = t[: brk[0] + 1], tag[: brk[0] + 1]
    return t, tag


def _layers(t, tag, kind):
    """Average event times of whole layers (0x10 ... next 0x10) inside passes of `kind` (0x90 or 0x91), the tag
    sequence they share, and the average layer duration."""
    cur, kinds = 0, []
    for g in tag:
        if g in (0x90, 0x91):
            cur = g
        kinds.append(cur)
    starts = [i for i, g in enumerate(tag) if g == 0x10]
    out = []
    for a, b in zip(starts[:-1], starts[1:]):
        if kinds[a] != kind or any(tag[j] in (0x60, 0x90, 0x91) for j in range(a, b)):
            continue
        out.append((t[a:b] - t[a], tuple(tag[a:b]), t[b] - t[a]))
    if not out:
        return None, None, None
    pattern = collections.Counter(p for _, p, _ in out).most_common(1)[0][0]
    rows = np.array([x for x, p, _ in out if p == pattern])
    return rows.mean(axis=0), pattern, float(np.mean([g for _, _, g in out]))


def _stage_table(times, pattern, weight_bytes, layer_end):
    lines = ["| stage | total µs | barrier | input fetch | weights + products | epilogue | weight MB | GB/s over the stage |",
             "|---|---|---|---|---|---|---|---|"]
    idx = {g: i for i, g in enumerate(pattern)}            # first occurrence
    for k, (name, base) in enumerate(STAGES):
        i0 = idx[base]
        i1 = idx[STAGES[k + 1][1]] if k + 1 < len(STAGES) else len(pattern)
        t0 = times[i0]
        t_end = times[i1] if i1 < len(pattern) else layer_end
        seg = list(zip(pattern[i0:i1], times[i0:i1]))
        at = lambda g: next((x for gg, x in seg if gg == g), None)
        barrier = at(base + 2) - t0
        if base == 0x20 and None in (at(0x24), at(0x27)):
            lines.append(f"| {name} | {t_end - t0:.2f} | {barrier:.2f} | (no attention item on this workgroup) | | | | |")
            continue
        if base == 0x20:
            lines.append(f"| {name} | {t_end - t0:.2f} | {barrier:.2f} | {at(0x24) - at(0x22):.2f} (q, K, V) | "
                         f"{at(0x27) - at(0x24):.2f} (scores, fold) | {t_end - at(0x27):.2f} (partial, counter, merge) | | |")
            continue
        staged = [x for gg, x in seg if gg == 0x80]
        done = [x for gg, x in seg if gg == 0x81]
        fetch = staged[0] - at(base + 2)
        stream = done[-1] - staged[0]          # later groups and chunks restage or reuse the rows in between
        epi = t_end - done[-1]
        lines.append(f"| {name} | {t_end - t0:.2f} | {barrier:.2f} | {fetch:.2f} | {stream:.2f} | {epi:.2f} | "
                     f"{weight_bytes[k] / 1e6:.1f} | {weight_bytes[k] / (t_end - t0) / 1e3:.0f} |")
    return lines


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2")
    ap.add_argument("--workgroup", type=int, default=100)
    a = ap.parse_args()
    w = W.get_workload(a.config)
    m = w.model
    ws, prompt = W.make_weights(w, threads=16), W.make_prompt(w)
    model = LsModel(m, ws, max_seq=w.n_prompt + w.n_new + 17)
    model.generate(prompt, 8, 0, 0)
    B = m.elem_bytes
    wb = [m.d_model * (m.q_dim + 2 * m.kv_dim) * B, 0, m.q_dim * m.d_model * B, 2 * m.d_model * m.ffn_dim * B,
          m.ffn_dim * m.d_model * B]
    print(f"# Stages of one decoder layer inside the persistent decode kernel, workload {a.config} "
          f"({m.name}: L{m.n_layers} d_model {m.d_model} ffn {m.ffn_dim}), workgroup {a.workgroup} of 256\n")
    print("Command (on the MI355X box, from the repository root):\n")
    print(f"    python -m paper_2404_16710_amd.stage_timeline --config {a.config} --workgroup {a.workgroup}\n")
    print("Source: the kernel's own event recording (`ls_debug_timeline`), not a profiler; the kernel-level totals "
          "are in the rocprofv3 summaries beside this file.\n")
    print("Times are averages over the layers one workgroup recorded (100 MHz wall clock); `GB/s over the stage` is the "
          "whole stage's weight matrix over the stage's total time, barrier and hand-over included (all 256 workgroups "
          "stream their shares at the same time; the first register slots of a stage are requested before its barrier, "
          "so the `weights + products` column alone understates the time those bytes had).\n")
    E, d = w.exit_layer, w.draft_len

    def drafted():
        model.debug_timeline(0)
        model.prefill(prompt)
        model.draft(E, d)

    for kind, label, run, before in (
            (0x90, "one-row pass (a draft step / a token of plain decoding), context ≈ prompt length",
             lambda: model.generate(prompt, 3, 0, 0), None),
            (0x91, f"{d + 1}-row verification pass (layers {E}..{m.n_layers - 1} after {d} drafts)",
             lambda: model.verify(E, d), drafted)):
        t, tag = _events(model, 512, a.workgroup, run, before)
        times, pattern, layer_us = _layers(t, tag, kind)
        if times is None:
            print(f"## {label}: no complete layer recorded\n")
            continue
        print(f"## {label}: {layer_us:.1f} µs per layer "
              f"({sum(wb) / 1e6:.1f} MB of weights: {sum(wb) / layer_us / 1e3:.0f} GB/s over the whole layer)\n")
        print("\n".join(_stage_table(times, pattern, wb, layer_us)))
        print()
    # head and candidate reduction from a one-layer early-exit run
    t, tag = _events(model, 512, a.workgroup, lambda: model.generate_early_exit(prompt, 6, 1))
    heads, cands, passes = [], [], []
    i60 = [i for i, g in enumerate(tag) if g == 0x60]
    for i in i60:
        j70 = next((j for j in range(i, len(tag)) if tag[j] == 0x70), None)
        j76 = next((j for j in range(i, len(tag)) if tag[j] == 0x76), None)
        j90 = next((j for j in range(i, len(tag)) if tag[j] == 0x90), None)
        j10 = next((j for j in range(j90 or len(tag), len(tag)) if tag[j] == 0x10), None)
        if None in (j70, j76, j90, j10):
            continue
        heads.append(t[j70] - t[i]); cands.append(t[j76] - t[j70]); passes.append(t[j10] - t[j76])
    if heads:
        hb = m.vocab * m.d_model * B
        print(f"## head and pass overhead (one-row passes)\n")
        print(f"final norm + LM head + argmax candidates: {np.mean(heads):.1f} µs for {hb / 1e6:.1f} MB "
              f"({hb / np.mean(heads) / 1e3:.0f} GB/s); candidate barrier + reduction: {np.mean(cands):.1f} µs; "
              f"from the reduced token to the first stage of the next pass: {np.mean(passes):.1f} µs.")
    model.close()


if __name__ == "__main__":
    main()
