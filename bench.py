#!/usr/bin/env python3
"""Benchmark of the hot path: greedy self-speculative decoding at batch 1 on one MI355X.

One "step" is one whole job of the workload: prefill of the prompt, then draft/verify rounds
until n_new tokens exist (ls_generate), with weights and prompt already resident in HBM.
After the timed steps the same kernels run full-model greedy decoding (d = 0) on the same
weights for the speed-up, and the CPU oracle is timed on a bounded sample of the same job.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def decode_bytes_selfspec(m, P, E, d, rounds, pos_final):
    """Algorithmic bytes of the decode launch: weights read once per pass plus the KV rows each
    pass attends to (positions interpolated linearly over the rounds)."""
    Wl, Wh, kv = m.layer_weight_bytes(), m.head_weight_bytes(), m.kv_bytes_per_pos_layer()
    L = m.n_layers
    total = 0.0
    adv = (pos_final - P) / max(rounds, 1)
    for r in range(rounds):
        pos = P + r * adv
        for i in range(d):
            total += E * Wl + Wh + E * (pos + i + 1) * kv
        total += E * Wl + E * (pos + d + 1) * kv
        total += (L - E) * Wl + Wh + (L - E) * (pos + d + 1) * kv
    return total


def decode_bytes_ar(m, P, n_new):
    Wl, Wh, kv = m.layer_weight_bytes(), m.head_weight_bytes(), m.kv_bytes_per_pos_layer()
    L = m.n_layers
    return sum(L * Wl + Wh + L * (P + k) * kv for k in range(1, n_new))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="c2", help="workload: c1..c5 (default c2, the 1.5B model)")
    ap.add_argument("--exit-layer", type=int, default=None)
    ap.add_argument("--draft", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-new", type=int, default=24)
    ap.add_argument("--sweep", action="store_true",
                    help="also run the workload's (exit layer, draft length) grid and add it to the JSON line")
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run the library's plain copy kernel over this many MiB (byte-counter reference)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as W
    from paper_2404_16710_amd import LsModel

    w = W.get_workload(a.config)
    E = a.exit_layer or w.exit_layer
    d = a.draft if a.draft is not None else w.draft_len
    m = w.model
    t0 = time.time()
    weights = W.make_weights(w, exit_layer=E, threads=min(16, len(os.sched_getaffinity(0))))
    prompt = W.make_prompt(w)
    t_gen = time.time() - t0
    model = LsModel(m, weights, max_seq=w.n_prompt + w.n_new + 16 + 1)
    if a.wg_per_cu:
        model.set_launch(a.wg_per_cu)
    print(f"[bench] {m.name}: weights generated in {t_gen:.1f}s, uploaded; E={E} d={d} "
          f"P={w.n_prompt} N={w.n_new}", file=sys.stderr, flush=True)

    if a.calibration_copy_mib:
        model.debug_copy(a.calibration_copy_mib << 20)
    for _ in range(a.warmup):
        model.generate(prompt, w.n_new, E, d)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    runs = []
    for _ in range(a.steps):
        toks, st = model.generate(prompt, w.n_new, E, d)
        runs.append(st)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = t1 - t0
    value = a.steps * w.n_new / sec
    ms_dec = float(np.mean([r.ms_decode for r in runs]))
    ms_pre = float(np.mean([r.ms_prefill for r in runs]))
    st = runs[-1]
    pos_final, _, _ = model.get_state()

    # full-model greedy on the same kernels and weights (the "Autoregressive" baseline)
    model.generate(prompt, w.n_new, 0, 0)
    ar_runs = [model.generate(prompt, w.n_new, 0, 0) for _ in range(max(1, min(a.steps, 3)))]
    ar_toks = ar_runs[-1][0]
    ar_ms_dec = float(np.mean([r[1].ms_decode for r in ar_runs]))
    ar_ms_pre = float(np.mean([r[1].ms_prefill for r in ar_runs]))

    # the two other curves of the paper's tables on the same weights: verification without reuse of the
    # draft stage's cache and exit states (its ablation), and early exit on its own (lossy: other tokens)
    model.generate_no_reuse(prompt, w.n_new, E, d)
    nr_toks, nr = model.generate_no_reuse(prompt, w.n_new, E, d)
    model.generate_early_exit(prompt, w.n_new, E)
    _, ee = model.generate_early_exit(prompt, w.n_new, E)
    # NEXT row of the scope table: per-token exit layer (a draft leaves at E/2 when its margin reaches tau)
    dyn = None
    if E >= 2:
        e_low, tau = max(1, E // 2), 0.05
        dy_toks, dy, _, dy_low = model.generate_dynamic(prompt, w.n_new, e_low, E, d, tau)
        dyn = {"exit_low": e_low, "exit_high": E, "tau": tau,
               "decode_tokens_per_s": round((w.n_new - 1) / (dy.ms_decode * 1e-3), 2),
               "ms_decode": round(dy.ms_decode, 3), "acceptance": round(dy.acceptance, 4), "rounds": dy.rounds,
               "drafts_leaving_at_exit_low": round(dy_low / max(dy.drafted, 1), 4), "same_ids": bool(dy_toks == toks)}

    # the stages on their own, through the step-by-step calls (one launch each, timed with events on
    # the launch stream): ls_draft = d draft steps + the early-layer pass of the last draft, ls_verify =
    # the (d+1)-row pass over layers [E, L) + head + acceptance; a draft step alone = an early-exit token
    Wl, Wh, kvb = m.layer_weight_bytes(), m.head_weight_bytes(), m.kv_bytes_per_pos_layer()
    model.prefill(prompt)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_draft, t_verify, b_draft, b_verify = [], [], [], []
    for _ in range(8):
        pos_r, _, _ = model.get_state()
        ev[0].record(); model.draft(E, d); ev[1].record(); model.verify(E, d); ev[2].record()
        torch.cuda.synchronize()
        t_draft.append(ev[0].elapsed_time(ev[1])); t_verify.append(ev[1].elapsed_time(ev[2]))
        b_draft.append(sum(E * Wl + Wh + E * (pos_r + i + 1) * kvb for i in range(d)) + E * Wl + E * (pos_r + d + 1) * kvb)
        b_verify.append((m.n_layers - E) * (Wl + (pos_r + d + 1) * kvb) + Wh)
    t_draft, t_verify = t_draft[1:], t_verify[1:]            # the first round warms the caches
    b_draft, b_verify = b_draft[1:], b_verify[1:]
    gb = lambda by, ms_: float(np.sum(by) / (np.sum(ms_) * 1e-3) / 1e9)
    ee_bytes = sum(E * Wl + Wh + E * (w.n_prompt + k) * kvb for k in range(1, w.n_new))
    # streaming reference: the library's plain copy kernel over 1 GiB (read + write)
    import ctypes
    c_src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
    c_dst = torch.empty_like(c_src)
    copy = lambda: model.lib.ls_debug_copy(ctypes.c_void_p(c_dst.data_ptr()), ctypes.c_void_p(c_src.data_ptr()),
                                           1 << 30, model._stream())
    copy()
    ev[0].record()
    for _ in range(4):
        copy()
    ev[1].record()
    torch.cuda.synchronize()
    stream_gbs = 4 * 2 * (1 << 30) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    del c_src, c_dst

    b_ss = decode_bytes_selfspec(m, w.n_prompt, E, d, st.rounds, pos_final)
    b_ar = decode_bytes_ar(m, w.n_prompt, w.n_new)
    ach = b_ss / (ms_dec * 1e-3) / 1e9
    ach_ar = b_ar / (ar_ms_dec * 1e-3) / 1e9

    # HBM bytes per decode launch from the committed counter profile of this very workload
    # (FETCH_SIZE + WRITE_SIZE scaled by the copy-kernel reference); null for other workloads
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "decode_kernel_c2_hbm_traffic.txt")
    if a.config == "c2" and E == w.exit_layer and d == w.draft_len and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
    out = {
        "metric": "generated tokens/s at batch 1, greedy self-speculative decoding (whole job: prefill + decode)",
        "value": round(value, 2), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec / a.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{a.config}: {m.name} L{m.n_layers} dm{m.d_model} ffn{m.ffn_dim} V{m.vocab}, "
                               f"prompt {w.n_prompt}, {w.n_new} new tokens, E={E}, d={d}, batch 1",
                   "exit_layer": E, "draft_len": d, "n_prompt": w.n_prompt, "n_new": w.n_new},
        "selfspec": {"decode_tokens_per_s": round((w.n_new - 1) / (ms_dec * 1e-3), 2),
                     "ms_prefill": round(ms_pre, 3), "ms_decode": round(ms_dec, 3),
                     "acceptance": round(st.acceptance, 4), "rounds": st.rounds,
                     "tokens_per_round": round((w.n_new - 1) / max(st.rounds, 1), 3)},
        "full_greedy": {"tokens_per_s": round(w.n_new / ((ar_ms_pre + ar_ms_dec) * 1e-3), 2),
                        "decode_tokens_per_s": round((w.n_new - 1) / (ar_ms_dec * 1e-3), 2),
                        "ms_prefill": round(ar_ms_pre, 3), "ms_decode": round(ar_ms_dec, 3),
                        "hbm_gbs": round(ach_ar, 1), "hbm_frac": round(ach_ar / HBM_PEAK_GBS, 4)},
        "no_cache_reuse": {"decode_tokens_per_s": round((w.n_new - 1) / (nr.ms_decode * 1e-3), 2),
                           "ms_decode": round(nr.ms_decode, 3), "same_ids": bool(nr_toks == toks),
                           "reuse_saves_ms_per_token": round((nr.ms_decode - ms_dec) / (w.n_new - 1), 4)},
        "early_exit_only": {"decode_tokens_per_s": round((w.n_new - 1) / (ee.ms_decode * 1e-3), 2),
                            "ms_decode": round(ee.ms_decode, 3), "exit_layer": E},
        "per_token_exit_layer": dyn,
        "stages": {"draft_launch": {"ms": round(float(np.mean(t_draft)), 3), "hbm_gbs": round(gb(b_draft, t_draft), 1),
                                    "hbm_frac": round(gb(b_draft, t_draft) / HBM_PEAK_GBS, 4),
                                    "what": f"{d} draft steps + early layers of the last draft (ls_draft)"},
                   "verify_launch": {"ms": round(float(np.mean(t_verify)), 3), "hbm_gbs": round(gb(b_verify, t_verify), 1),
                                     "hbm_frac": round(gb(b_verify, t_verify) / HBM_PEAK_GBS, 4),
                                     "what": f"{d + 1} rows through layers [{E}, {m.n_layers}) + head (ls_verify)"},
                   "draft_step": {"hbm_gbs": round(ee_bytes / (ee.ms_decode * 1e-3) / 1e9, 1),
                                  "hbm_frac": round(ee_bytes / (ee.ms_decode * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                  "what": f"layers [0, {E}) + head per token (the early-exit job)"}},
        "speedup_vs_full_greedy": round(ar_ms_dec / ms_dec, 3),
        "same_ids_as_full_greedy": bool(toks == ar_toks),
        "roofline": {"bound": "hbm", "kernel": "ls_decode_kernel<bf16> (one launch = all draft + tail + verify passes of a job)",
                     "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "stream_copy_gbs": round(stream_gbs, 1), "frac_of_stream_copy": round(ach / stream_gbs, 4),
                     "bytes_per_launch": int(b_ss), "ms_per_launch": round(ms_dec, 3)},
    }

    if not a.no_cpu_baseline:
        import oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        om = O.OracleModel(m, weights, np.float32, emulate_bf16_act=(m.dtype == "bf16"))
        n_s = min(a.cpu_sample_new, w.n_new)
        c0 = time.perf_counter()
        cache = om.new_cache(w.n_prompt + 2)
        O.prefill(om, prompt, cache)
        c_pre = time.perf_counter() - c0
        del cache
        c0 = time.perf_counter()
        ref = O.self_speculative(om, prompt, n_s, E, d)
        c_all = time.perf_counter() - c0
        c0 = time.perf_counter()
        O.greedy_full(om, prompt, max(2, n_s // 2))
        c_ar = time.perf_counter() - c0
        out["cpu_baseline"] = {
            "value": round(n_s / c_all, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"same weights and {w.n_prompt}-id prompt, first {n_s} of {w.n_new} new tokens "
                      f"(prefill included, {c_pre:.1f}s of {c_all:.1f}s), E={E} d={d}, numpy float32",
            "decode_tokens_per_s": round((n_s - 1) / max(c_all - c_pre, 1e-9), 3),
            "full_greedy_decode_tokens_per_s": round((max(2, n_s // 2) - 1) / max(c_ar - c_pre, 1e-9), 3),
            "acceptance": round(ref.acceptance, 4),
            "ids_match_gpu_until_near_tie": int(next((i for i, (x, y) in enumerate(zip(toks, ref.tokens)) if x != y), n_s)),
        }
    model.close()
    if a.sweep and w.sweep_exit_layers:
        # the (E, d) grid of the workload: weights are regenerated per E (the scaled layers follow E);
        # full-model greedy is timed once per E on those weights
        del model, weights
        out["sweep"] = []
        for Es in w.sweep_exit_layers:
            ws = W.make_weights(w, exit_layer=Es, threads=min(16, len(os.sched_getaffinity(0))))
            mod = LsModel(m, ws, max_seq=w.n_prompt + w.n_new + 16 + 1)
            mod.generate(prompt, w.n_new, 0, 0)
            ar_t, ar_s = mod.generate(prompt, w.n_new, 0, 0)
            for ds in w.sweep_draft_lens:
                mod.generate(prompt, w.n_new, Es, ds)
                tk, s_ = mod.generate(prompt, w.n_new, Es, ds)
                row = {"exit_layer": Es, "draft_len": ds, "acceptance": round(s_.acceptance, 4), "rounds": s_.rounds,
                       "decode_tokens_per_s": round((w.n_new - 1) / (s_.ms_decode * 1e-3), 2),
                       "full_greedy_decode_tokens_per_s": round((w.n_new - 1) / (ar_s.ms_decode * 1e-3), 2),
                       "speedup_vs_full_greedy": round(ar_s.ms_decode / s_.ms_decode, 3),
                       "same_ids_as_full_greedy": bool(tk == ar_t)}
                out["sweep"].append(row)
                print(f"[bench] sweep {row}", file=sys.stderr, flush=True)
            mod.close()
            del mod, ws
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
