#!/usr/bin/env python3
"""Benchmark of the hot path: greedy self-speculative decoding at batch 1 on one MI355X.

One "step" is one whole job of a workload: prefill of the prompt, then draft/verify rounds until
n_new tokens exist (ls_generate), with weights and prompt already resident in HBM.

The headline (`value`, `roofline`, `cpu_baseline`) is the largest workload that fits one GPU: the
13B shape at its stated exit layer and draft length.  `per_config` then holds, for every one of the
five workloads, tokens/s, acceptance, the speed-up over full-model greedy decoding on the same
kernels and weights, the speed-up a pure bandwidth model predicts for that acceptance, and the
achieved fraction of the HBM roofline for the whole decode launch, the draft launch and the verify
launch; `sweep` is the 13B grid of exit layers and draft lengths.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
HEADLINE = "c5"
ALL_CONFIGS = ("c1", "c2", "c3", "c4", "c5")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


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


def committed_traffic(name, E, d, rounds):
    """HBM bytes per decode launch from the committed counter profile of this workload (FETCH_SIZE +
    WRITE_SIZE scaled by the copy-kernel reference).  The profile belongs to a job with a certain
    number of rounds; a run with another count gets null."""
    path = os.path.join(ROOT, "profiles", f"decode_kernel_{name}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    vals = {}
    for line in open(path):
        if ":" in line and line.split(":")[0] in ("traffic_bytes_per_launch", "rounds", "exit_layer", "draft_len"):
            vals[line.split(":")[0]] = int(line.split(":")[1])
    if vals.get("rounds") != rounds or vals.get("exit_layer", E) != E or vals.get("draft_len", d) != d:
        return None, vals.get("rounds")
    return vals.get("traffic_bytes_per_launch"), vals.get("rounds")


def time_jobs(model, prompt, n_new, E, d, steps, warmup):
    """W untimed jobs, then exactly K timed ones between device synchronisations."""
    import torch
    for _ in range(warmup):
        model.generate(prompt, n_new, E, d)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    runs = []
    toks = None
    for _ in range(steps):
        toks, st = model.generate(prompt, n_new, E, d)
        runs.append(st)
    torch.cuda.synchronize()
    return time.perf_counter() - t0, runs, toks


def stage_launches(model, m, prompt, E, d):
    """The stages on their own through the step-by-step calls (one launch each, timed with events on
    the launch stream): ls_draft = d draft steps + the early-layer pass of the last draft, ls_verify =
    the (d+1)-row pass over layers [E, L) + head + acceptance."""
    import numpy as np
    import torch
    Wl, Wh, kvb = m.layer_weight_bytes(), m.head_weight_bytes(), m.kv_bytes_per_pos_layer()
    model.prefill(prompt)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_draft, t_verify, b_draft, b_verify = [], [], [], []
    for _ in range(6):
        pos_r, _, _ = model.get_state()
        ev[0].record(); model.draft(E, d); ev[1].record(); model.verify(E, d); ev[2].record()
        torch.cuda.synchronize()
        t_draft.append(ev[0].elapsed_time(ev[1])); t_verify.append(ev[1].elapsed_time(ev[2]))
        b_draft.append(sum(E * Wl + Wh + E * (pos_r + i + 1) * kvb for i in range(d)) + E * Wl + E * (pos_r + d + 1) * kvb)
        b_verify.append((m.n_layers - E) * (Wl + (pos_r + d + 1) * kvb) + Wh)
    t_draft, t_verify, b_draft, b_verify = t_draft[1:], t_verify[1:], b_draft[1:], b_verify[1:]   # first round warms up
    gb = lambda by, ms_: float(np.sum(by) / (np.sum(ms_) * 1e-3) / 1e9)
    return {
        "draft_launch": {"ms": round(float(np.mean(t_draft)), 3), "hbm_gbs": round(gb(b_draft, t_draft), 1),
                         "hbm_frac": round(gb(b_draft, t_draft) / HBM_PEAK_GBS, 4),
                         "what": f"{d} draft steps + early layers of the last draft (ls_draft)"},
        "verify_launch": {"ms": round(float(np.mean(t_verify)), 3), "hbm_gbs": round(gb(b_verify, t_verify), 1),
                          "hbm_frac": round(gb(b_verify, t_verify) / HBM_PEAK_GBS, 4),
                          "what": f"{d + 1} rows through layers [{E}, {m.n_layers}) + head (ls_verify)"},
    }


def measure(model, name, w, prompt, E, d, steps, warmup, ar=None):
    """Self-speculative jobs, then full-model greedy on the same kernels and weights (unless `ar`
    already holds it for these weights), and what follows from both."""
    import numpy as np
    m = w.model
    sec, runs, toks = time_jobs(model, prompt, w.n_new, E, d, steps, warmup)
    st = runs[-1]
    pos_final, _, _ = model.get_state()
    ms_dec = float(np.mean([r.ms_decode for r in runs]))
    ms_pre = float(np.mean([r.ms_prefill for r in runs]))
    if ar is None:
        model.generate(prompt, w.n_new, 0, 0)
        ar_runs = [model.generate(prompt, w.n_new, 0, 0) for _ in range(max(1, min(steps, 3)))]
        ar = {"toks": ar_runs[-1][0], "ms_decode": float(np.mean([r[1].ms_decode for r in ar_runs])),
              "ms_prefill": float(np.mean([r[1].ms_prefill for r in ar_runs]))}
    b_ss = decode_bytes_selfspec(m, w.n_prompt, E, d, st.rounds, pos_final)
    b_ar = decode_bytes_ar(m, w.n_prompt, w.n_new)
    ach, ach_ar = b_ss / (ms_dec * 1e-3) / 1e9, b_ar / (ar["ms_decode"] * 1e-3) / 1e9
    row = {
        "workload": f"{name}: {m.name} L{m.n_layers} dm{m.d_model} ffn{m.ffn_dim} V{m.vocab}, prompt {w.n_prompt}, "
                    f"{w.n_new} new tokens, batch 1",
        "exit_layer": E, "draft_len": d, "dtype": "bf16" if m.dtype == "bf16" else "f32",
        "tokens_per_s": round(steps * w.n_new / sec, 2), "steps": steps,
        "decode_tokens_per_s": round((w.n_new - 1) / (ms_dec * 1e-3), 2),
        "ms_prefill": round(ms_pre, 3), "ms_decode": round(ms_dec, 3),
        "acceptance": round(st.acceptance, 4), "rounds": st.rounds,
        "tokens_per_round": round((w.n_new - 1) / max(st.rounds, 1), 3),
        "full_greedy_decode_tokens_per_s": round((w.n_new - 1) / (ar["ms_decode"] * 1e-3), 2),
        "full_greedy_ms_decode": round(ar["ms_decode"], 3),
        "speedup_vs_full_greedy": round(ar["ms_decode"] / ms_dec, 3),
        # what a pure bandwidth model gives at this acceptance: bytes of the greedy job over bytes of the
        # self-speculative job, (n + 1) * AR / (d * draft + tail + verify) summed over the rounds
        "bandwidth_model_speedup": round(b_ar / b_ss, 3),
        "same_ids_as_full_greedy": bool(toks == ar["toks"]),
        "roofline": {"bytes_per_launch": int(b_ss), "ms_per_launch": round(ms_dec, 3), "hbm_gbs": round(ach, 1),
                     "frac": round(ach / HBM_PEAK_GBS, 4)},
        "full_greedy_roofline": {"bytes_per_launch": int(b_ar), "ms_per_launch": round(ar["ms_decode"], 3),
                                 "hbm_gbs": round(ach_ar, 1), "frac": round(ach_ar / HBM_PEAK_GBS, 4)},
    }
    return row, sec, toks, ar


def stream_copy_gbs(model):
    """Streaming reference: the library's plain copy kernel over 1 GiB (read + write)."""
    import torch
    src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    copy = lambda: model.lib.ls_debug_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()),
                                           1 << 30, model._stream())
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    copy()
    ev[0].record()
    for _ in range(4):
        copy()
    ev[1].record()
    torch.cuda.synchronize()
    return 4 * 2 * (1 << 30) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def stream_read_gbs(model, workgroups):
    """Read-only streaming reference: 2 GiB walked once per launch in the decode kernels' launch shape
    (`workgroups` x 256 threads, 64 KB per workgroup in flight), ls_read_kernel."""
    import torch
    n = 2 << 30
    src = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    sink = torch.empty(workgroups * 4096, dtype=torch.uint8, device="cuda:0")
    def read():
        rc = model.lib.ls_debug_read(ctypes.c_void_p(src.data_ptr()), n, ctypes.c_void_p(sink.data_ptr()), workgroups,
                                     model._stream())
        if rc != 0:
            raise RuntimeError(f"ls_debug_read: {rc}")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    read()
    ev[0].record()
    for _ in range(4):
        read()
    ev[1].record()
    torch.cuda.synchronize()
    return 4 * n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def cpu_oracle_baseline(w, weights, prompt, E, d, n_sample, gpu_toks):
    """The oracle as it stands, on the host cores, for a bounded sample of the same job."""
    import numpy as np
    import oracle as O
    m = w.model
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    om = O.OracleModel(m, weights, np.float32, emulate_bf16_act=(m.dtype == "bf16"))
    n_s = min(n_sample, w.n_new)
    c0 = time.perf_counter()
    cache = om.new_cache(w.n_prompt + 2)
    O.prefill(om, prompt, cache)
    c_pre = time.perf_counter() - c0
    del cache
    c0 = time.perf_counter()
    ref = O.self_speculative(om, prompt, n_s, E, d)
    c_all = time.perf_counter() - c0
    first_diff = next((i for i, (x, y) in enumerate(zip(gpu_toks, ref.tokens)) if x != y), None)
    out = {
        "value": round(n_s / c_all, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"same weights and {w.n_prompt}-id prompt, first {n_s} of {w.n_new} new tokens in {c_all:.1f}s, prompt pass "
                  f"included (a prompt pass timed on its own: {c_pre:.1f}s), E={E} d={d}, numpy float32",
        # decode-only rate by subtraction of the separately timed prompt pass: only where the rounds are a
        # sizeable part of the sample (on the 13B workload the prompt pass is nearly all of it)
        "decode_tokens_per_s": round((n_s - 1) / (c_all - c_pre), 3) if c_all - c_pre > 0.2 * c_all else None,
        "acceptance": round(ref.acceptance, 4),
        "first_differing_id_vs_gpu": first_diff,
        "oracle_margin_there": None if first_diff is None else round(float(ref.margins[first_diff]), 5),
    }
    del om
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default=HEADLINE, help="headline workload: c1..c5 (default c5, the 13B model)")
    ap.add_argument("--only", action="store_true", help="the headline workload only: no per_config list, no sweep")
    ap.add_argument("--exit-layer", type=int, default=None)
    ap.add_argument("--draft", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-new", type=int, default=0, help="tokens of the oracle sample (0: by workload)")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the ablation / early-exit / per-token-exit jobs")
    ap.add_argument("--other-steps", type=int, default=3, help="timed jobs per non-headline workload")
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

    threads = min(16, len(os.sched_getaffinity(0)))
    name = a.config
    w = W.get_workload(name)
    E = a.exit_layer or w.exit_layer
    d = a.draft if a.draft is not None else w.draft_len
    m = w.model
    t0 = time.time()
    weights = W.make_weights(w, exit_layer=E, threads=threads)
    prompt = W.make_prompt(w)
    model = LsModel(m, weights, max_seq=w.n_prompt + w.n_new + 16 + 1)
    if a.wg_per_cu:
        model.set_launch(a.wg_per_cu)
    log(f"{m.name}: weights generated and uploaded in {time.time() - t0:.1f}s; E={E} d={d} P={w.n_prompt} N={w.n_new}")
    if a.calibration_copy_mib:
        model.debug_copy(a.calibration_copy_mib << 20)

    head, sec, toks, ar = measure(model, name, w, prompt, E, d, a.steps, a.warmup)
    head["stages"] = stage_launches(model, m, prompt, E, d)
    log(f"{name}: {head['tokens_per_s']} tok/s, acceptance {head['acceptance']}, speed-up {head['speedup_vs_full_greedy']} "
        f"(bandwidth model {head['bandwidth_model_speedup']}), hbm {head['roofline']['frac']}")
    extras = {}
    if not a.no_extras:
        # the other curves of the paper's tables on the same weights: verification without reuse of the
        # draft stage's cache and exit states (its ablation), early exit on its own (lossy: other tokens),
        # and the per-token exit layer (a draft leaves at E/2 when its margin reaches tau)
        model.generate_no_reuse(prompt, w.n_new, E, d)
        nr_toks, nr = model.generate_no_reuse(prompt, w.n_new, E, d)
        model.generate_early_exit(prompt, w.n_new, E)
        _, ee = model.generate_early_exit(prompt, w.n_new, E)
        Wl, Wh, kvb = m.layer_weight_bytes(), m.head_weight_bytes(), m.kv_bytes_per_pos_layer()
        ee_bytes = sum(E * Wl + Wh + E * (w.n_prompt + k) * kvb for k in range(1, w.n_new))
        extras["no_cache_reuse"] = {"decode_tokens_per_s": round((w.n_new - 1) / (nr.ms_decode * 1e-3), 2),
                                    "ms_decode": round(nr.ms_decode, 3), "same_ids": bool(nr_toks == toks),
                                    "reuse_saves_ms_per_token": round((nr.ms_decode - head["ms_decode"]) / (w.n_new - 1), 4)}
        extras["early_exit_only"] = {"decode_tokens_per_s": round((w.n_new - 1) / (ee.ms_decode * 1e-3), 2),
                                     "ms_decode": round(ee.ms_decode, 3), "exit_layer": E,
                                     "hbm_frac": round(ee_bytes / (ee.ms_decode * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if E >= 2:
            e_low, tau = max(1, E // 2), 0.05
            dy_toks, dy, _, dy_low = model.generate_dynamic(prompt, w.n_new, e_low, E, d, tau)
            extras["per_token_exit_layer"] = {
                "exit_low": e_low, "exit_high": E, "tau": tau,
                "decode_tokens_per_s": round((w.n_new - 1) / (dy.ms_decode * 1e-3), 2),
                "ms_decode": round(dy.ms_decode, 3), "acceptance": round(dy.acceptance, 4), "rounds": dy.rounds,
                "drafts_leaving_at_exit_low": round(dy_low / max(dy.drafted, 1), 4), "same_ids": bool(dy_toks == toks)}
    stream_gbs = stream_copy_gbs(model)
    read_gbs = {wg: stream_read_gbs(model, wg) for wg in (256, 2048)}
    traffic, traffic_rounds = committed_traffic(name, E, d, head["rounds"])
    out = {
        "metric": "generated tokens/s at batch 1, greedy self-speculative decoding (whole job: prefill + decode)",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec / a.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"] + f", E={E}, d={d}", "exit_layer": E, "draft_len": d,
                   "n_prompt": w.n_prompt, "n_new": w.n_new},
        "selfspec": {k: head[k] for k in ("decode_tokens_per_s", "ms_prefill", "ms_decode", "acceptance", "rounds",
                                          "tokens_per_round")},
        "full_greedy": {"decode_tokens_per_s": head["full_greedy_decode_tokens_per_s"],
                        "ms_decode": head["full_greedy_ms_decode"], "hbm_gbs": head["full_greedy_roofline"]["hbm_gbs"],
                        "hbm_frac": head["full_greedy_roofline"]["frac"]},
        "speedup_vs_full_greedy": head["speedup_vs_full_greedy"],
        "bandwidth_model_speedup": head["bandwidth_model_speedup"],
        "same_ids_as_full_greedy": head["same_ids_as_full_greedy"],
        "stages": head["stages"],
        **extras,
        "roofline": {"bound": "hbm",
                     "kernel": f"ls_decode_kernel_{'bf16' if m.dtype == 'bf16' else 'f32'}_hd{m.head_dim} "
                               "(one launch = all draft + tail + verify passes of a job)",
                     "achieved": head["roofline"]["hbm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["roofline"]["frac"], "traffic": traffic, "traffic_profile_rounds": traffic_rounds,
                     "rounds": head["rounds"],
                     "stream_copy_gbs": round(stream_gbs, 1),
                     "stream_read_gbs": {"decode_launch_shape_256_workgroups": round(read_gbs[256], 1),
                                         "2048_workgroups": round(read_gbs[2048], 1)},
                     "frac_of_stream_read": round(head["roofline"]["hbm_gbs"] / max(read_gbs.values()), 4),
                     "bytes_per_launch": head["roofline"]["bytes_per_launch"],
                     "ms_per_launch": head["roofline"]["ms_per_launch"]},
    }

    per_config = {name: head}
    if a.only or a.no_sweep or not w.sweep_exit_layers or a.exit_layer or a.draft is not None:
        pass
    else:
        # the (E, d) grid of the workload: the layers whose residual scaling follows E are replaced in
        # place per E; full-model greedy is timed once per E on those weights
        out["sweep"] = []
        cur_E = E
        for Es in w.sweep_exit_layers:
            for l in range(min(cur_E, Es), max(cur_E, Es)):
                for tn in ("wo", "w_down"):
                    model.replace_tensor(tn, l, W.make_tensor(w, tn, l, Es))
            cur_E = Es
            ar_s = ar if Es == E else None
            for ds in w.sweep_draft_lens:
                row, _, _, ar_s = measure(model, name, w, prompt, Es, ds, 1, 1, ar=ar_s)
                out["sweep"].append({k: row[k] for k in (
                    "exit_layer", "draft_len", "acceptance", "rounds", "decode_tokens_per_s",
                    "full_greedy_decode_tokens_per_s", "speedup_vs_full_greedy", "bandwidth_model_speedup",
                    "same_ids_as_full_greedy")} | {"hbm_frac": row["roofline"]["frac"]})
                log(f"sweep {out['sweep'][-1]}")
        # (the host copy of the weights still holds the headline's E: the oracle below uses that one)
    model.close()
    del model
    gc.collect()
    torch.cuda.empty_cache()

    if not a.no_cpu_baseline:
        n_s = a.cpu_sample_new or {"c1": 64, "c2": 24, "c3": 8, "c4": 12, "c5": 6}[name]
        out["cpu_baseline"] = cpu_oracle_baseline(w, weights, prompt, E, d, n_s, toks)
        log(f"cpu oracle: {out['cpu_baseline']}")
    del weights
    gc.collect()

    if not a.only:
        for other in ALL_CONFIGS:
            if other == name:
                continue
            wo = W.get_workload(other)
            t0 = time.time()
            ws = W.make_weights(wo, threads=threads)
            pr = W.make_prompt(wo)
            mod = LsModel(wo.model, ws, max_seq=wo.n_prompt + wo.n_new + 16 + 1)
            del ws
            row, _, _, _ = measure(mod, other, wo, pr, wo.exit_layer, wo.draft_len, max(1, a.other_steps), 1)
            row["stages"] = stage_launches(mod, wo.model, pr, wo.exit_layer, wo.draft_len)
            per_config[other] = row
            log(f"{other} ({time.time() - t0:.0f}s): {row['tokens_per_s']} tok/s, acceptance {row['acceptance']}, speed-up "
                f"{row['speedup_vs_full_greedy']} (bandwidth model {row['bandwidth_model_speedup']}), hbm {row['roofline']['frac']}")
            mod.close()
            del mod
            gc.collect()
            torch.cuda.empty_cache()
        out["per_config"] = [per_config[c] for c in ALL_CONFIGS if c in per_config]
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
