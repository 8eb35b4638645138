#!/usr/bin/env python3
"""Benchmark of the sequence-scheduled decode path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic group: plan -> every micro-batch
(prompt forward + decode forwards) -> failure collection -> recomputation pass, through the C ABI
(ss_run_group).  Inputs and weights are resident in HBM (weights) / host-side int arrays of a few KB
(prompts) when the timed region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 3]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
PAPER_CONTEXT = ("paper, Table 4: 1.22 -> 2.27 samples/s (+86%) on one A100-80GB, Vicuna-7B, T=0.5 sampling, "
                 "10k alpaca-subset prompts, group 256; other hardware and data: context, not a target")


T_START = time.time()


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def decode_step_bytes(shape, B: int, ctx: int) -> int:
    """Algorithmic HBM bytes of one decode forward: every weight once, each live row's key/value history
    read once, one new key/value slot and one embedding row per live row."""
    kv = shape.kv_bytes_per_token()
    return shape.weight_bytes_per_step() + B * (ctx + 1) * kv + B * kv + B * shape.d_model * 2


TRAFFIC_PROFILE = os.path.join("profiles", "decode_step_7b_hbm_traffic.txt")


def profile_traffic(shape_name: str, rows: int, ctx: int, gemm_mode: int):
    """HBM bytes per decode step from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE runs of
    `bench.py --roofline-only`); a figure from that file, not a live one: (None, reason) when the file is absent
    or was taken at another shape."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    if not os.path.exists(path):
        return None, f"{TRAFFIC_PROFILE} absent"
    kv = {}
    for line in open(path):
        if line.startswith("@") and "=" in line:
            k, v = line[1:].split("=", 1)
            kv[k.strip()] = v.strip()
    want = dict(shape=shape_name, rows=str(rows), ctx=str(ctx), gemm_mode=str(gemm_mode))
    if any(kv.get(k) != v for k, v in want.items()) or "decode_step_hbm_bytes" not in kv:
        return None, f"{TRAFFIC_PROFILE} was taken at another shape or launch configuration"
    return float(kv["decode_step_hbm_bytes"]), f"{TRAFFIC_PROFILE} (rocprofv3 counters of an earlier run, not live)"


def ablation(a, ss, gw, wl, shape) -> int:
    """Table 5 of the paper on the synthetic group: which component buys what on this hardware.
    Every row is one pass over the same queries with the same predictions (multiplicative lognormal noise,
    sigma 0.3); 'perfect' uses the true length as the prediction (the paper's upper-bound row of Table 4); 'biased
    upward' imitates the paper's training target, the maximum over several generations (Sec. 4.2); 'power-of-two
    batch sizes' is the rule Sec. 4.2 states for its own runs (16 from length 300 on, else 256*50/L rounded to a
    power of two) in place of the configured clamp(floor(16*L_max/L), 16, 256)."""
    rows = [("vanilla", (), False), ("sort", ("SORT",), False), ("sort+FCR", ("SORT", "FCR"), False),
            ("sort+FCR+VBS", ("SORT", "FCR", "VBS"), False), ("binning", ("SORT", "BIN"), False),
            ("binning+FCR", ("SORT", "BIN", "FCR"), False), ("binning+FCR+VBS", ("SORT", "BIN", "FCR", "VBS"), False),
            ("binning+FCR+VBS+compaction", ("SORT", "BIN", "FCR", "VBS", "COMPACT"), False),
            ("binning+FCR+VBS, perfect predictor", ("SORT", "BIN", "FCR", "VBS"), True),
            ("binning+FCR+VBS, predictor biased upward (max of 4 draws)", ("SORT", "BIN", "FCR", "VBS"), "max4"),
            ("binning+FCR+VBS+compaction, predictor biased upward (max of 4 draws)",
             ("SORT", "BIN", "FCR", "VBS", "COMPACT"), "max4"),
            ("binning+FCR+VBS, paper's power-of-two batch sizes", ("SORT", "BIN", "FCR", "VBS"), "pow2"),
            ("binning+FCR+VBS+compaction, paper's power-of-two batch sizes",
             ("SORT", "BIN", "FCR", "VBS", "COMPACT"), "pow2")]
    if a.ablation_only:
        rows = [r for r in rows if r[0] == "vanilla" or a.ablation_only in r[0]]
    pred = wl.pred_lens
    if pred is None:   # config 2 carries no predictions: draw config 3's (same group)
        from paper_2305_13144_amd import synth
        pred = synth.make_workload(3).pred_lens
    binw = wl.bin_width or 50
    useful = int(wl.target_lens.sum())
    from paper_2305_13144_amd import synth as _synth
    pred_max4 = _synth.make_predictions_max_of(wl.target_lens, 0.3, 4, seed=20230513 + a.cfg)
    wt, wo = _synth.gather_prompts(wl, range(min(wl.n, wl.max_batch)))                  # warm-up: workspace growth
    ss.ss_decode_microbatch(gw, wt, wo, 4, np.full(len(wo) - 1, 4, np.int32), 0)
    base = None
    for name, flags, perfect in rows:
        pol = ss.make_policy(flags, wl.base_batch, wl.l_max, wl.max_batch,
                             ss.SS_VBS_PAPER_POW2 if perfect == "pow2" else ss.SS_VBS_CLAMP_FLOOR)
        p = None if not flags else (pred_max4 if perfect == "max4" else wl.target_lens if perfect is True else pred)
        r = ss.ss_run_group(gw, wl.prompt_tokens, wl.prompt_offsets, wl.target_lens, p, binw if "BIN" in flags else 0, pol)
        assert np.array_equal(r["lens"], wl.target_lens)
        st = r["stats"]
        tps = useful / (st["wall_ms"] / 1e3)
        base = base or tps
        log(f"ablation row '{name}': {st['wall_ms'] / 1e3:.1f} s, {tps:.0f} tok/s")
        print(json.dumps(dict(ablation=name, group=wl.n, model=shape.name, useful_tokens_per_s=tps,
                              samples_per_s=wl.n / (st["wall_ms"] / 1e3), vs_vanilla=tps / base, ms=st["wall_ms"],
                              steps=st["steps"], micro_batches=[st["n_mb_first"], st["n_mb_failure"]],
                              n_failed=st["n_failed"], padded_row_steps=st["padded_row_steps"],
                              computed_row_steps=st["computed_row_steps"],
                              avg_len=st["padded_row_steps"] / (wl.n + st["n_failed"]))), flush=True)
    gw.close()
    return 0


def sweeps(a, ss, gw, wl, shape) -> int:
    """Analogues of the paper's Fig. 3 on the synthetic workload, one JSON line per point.
    batch: throughput against micro-batch size, (a) every row generates a fixed 64 tokens, (b) vanilla batches
           run until their longest row finishes (a 64-query subset of the group keeps batch 1 affordable).
    group: throughput against group size for the full policy and for vanilla batching on the same queries."""
    from paper_2305_13144_amd import synth
    if a.sweep == "step":
        # One decode forward (ss_bench_decode_step: the kernels and launch shapes of a real step) against the number
        # of live rows at a fixed context, and against the context at 16 rows (the paper's App. D: time per token
        # grows linearly with the position).
        rng = np.random.default_rng(7)
        points = [("rows", B, 100) for B in (1, 2, 4, 8, 16, 24, 32, 48, 64, 65, 81, 96, 128, 129, 163, 200, 256)]
        points += [("context", 16, c) for c in (25, 50, 100, 200, 400, 800, 1600, 3200, 4000)]
        for what, B, ctx in points:
            ptoks = rng.integers(0, shape.vocab, size=B * ctx).astype(np.int32)
            ms = ss.ss_bench_decode_step(gw, ptoks, B, ctx, 11)[3:]
            nbytes = decode_step_bytes(shape, B, ctx)
            row = dict(sweep="step", vary=what, rows=B, ctx=ctx, ms=float(ms.mean()), ms_min=float(ms.min()),
                       algorithmic_bytes=nbytes, achieved_GBs=nbytes / (ms.mean() * 1e-3) / 1e9,
                       frac_of_hbm_peak=nbytes / (ms.mean() * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       mfma_TFLOPs=2.0 * B * (shape.weight_bytes_per_step() / 2) / (ms.mean() * 1e-3) / 1e12)
            log(f"sweep step {row}")
            print(json.dumps(row), flush=True)
        gw.close()
        return 0
    if a.sweep == "sync":
        # The configured group with ends the host does not know: the device applies the same lengths and the host
        # polls every `sync` decode forwards.  T = 0 emits the tokens of the known-length run, so the difference to
        # it is the polling protocol alone (reads + forwards run after the last row ended); T = 0.5 adds the sampler.
        pol = ss.make_policy(wl.flags, wl.base_batch, wl.l_max, wl.max_batch)
        useful = int(wl.target_lens.sum())
        ss.ss_run_group(gw, wl.prompt_tokens, wl.prompt_offsets, wl.target_lens, wl.pred_lens, wl.bin_width, pol)   # warm
        k = ss.ss_run_group(gw, wl.prompt_tokens, wl.prompt_offsets, wl.target_lens, wl.pred_lens, wl.bin_width, pol)
        print(json.dumps(dict(sweep="sync", mode="lengths known to the host", sync_every=None, temperature=0.0,
                              useful_tokens_per_s=useful / (k["stats"]["wall_ms"] / 1e3), ms=k["stats"]["wall_ms"],
                              steps=k["stats"]["steps"])), flush=True)
        draws = synth.make_draws(wl.n, wl.l_max, seed=20230513)
        for T in (0.0, 0.5):
            for sync in (1, 2, 4, 8, 16, 32, 64):
                g = ss.ss_run_group_generate(gw, wl.prompt_tokens, wl.prompt_offsets, wl.pred_lens, wl.bin_width, pol,
                                             eos_id=-1, temperature=T, draws=draws, target_lens=wl.target_lens,
                                             sync_every=sync)
                assert np.array_equal(g["lens"], wl.target_lens)
                if T == 0.0 and "COMPACT" not in wl.flags:
                    assert np.array_equal(g["tokens"], k["tokens"])
                st = g["stats"]
                row = dict(sweep="sync", mode="ends polled", sync_every=sync, temperature=T,
                           useful_tokens_per_s=useful / (st["wall_ms"] / 1e3), ms=st["wall_ms"], steps=st["steps"],
                           polls=st["polls"], idle_steps=st["idle_steps"], vs_known=k["stats"]["wall_ms"] / st["wall_ms"])
                log(f"sweep sync {row}")
                print(json.dumps(row), flush=True)
        gw.close()
        return 0
    full = synth.make_workload(4, shape=shape)                      # 1024 queries, with predictions
    if a.sweep == "batch":
        sub = list(range(64))
        for B in (1, 2, 4, 8, 16, 32, 64, 128, 256):
            idx = list(range(B))
            toks, offs = synth.gather_prompts(full, idx)
            ss.ss_decode_microbatch(gw, toks, offs, 2, np.full(B, 2, np.int32), 0)          # workspace growth
            r = ss.ss_decode_microbatch(gw, toks, offs, 64, np.full(B, 64, np.int32), 0)
            ms = r["stats"]["prefill_ms"] + r["stats"]["decode_ms"]
            row = dict(sweep="batch", batch=B, fixed_len_tokens_per_s=B * 64 / (ms / 1e3), fixed_len_ms=ms)
            if B <= 64:
                toks, offs = synth.gather_prompts(full, sub)
                pol = ss.make_policy((), B, full.l_max, max(B, 256))
                g = ss.ss_run_group(gw, toks, offs, full.target_lens[sub], None, 0, pol)
                row.update(until_finished_tokens_per_s=int(full.target_lens[sub].sum()) / (g["stats"]["wall_ms"] / 1e3),
                           until_finished_ms=g["stats"]["wall_ms"], until_finished_steps=g["stats"]["steps"])
            log(f"sweep batch {B}: {row}")
            print(json.dumps(row), flush=True)
    else:
        for n in (32, 64, 128, 256, 512, 1024):
            idx = list(range(n))
            toks, offs = synth.gather_prompts(full, idx)
            t, pr = full.target_lens[idx], full.pred_lens[idx]
            useful = int(t.sum())
            pol = ss.make_policy(full.flags, full.base_batch, full.l_max, full.max_batch)
            g = ss.ss_run_group(gw, toks, offs, t, pr, full.bin_width, pol)
            v = ss.ss_run_group(gw, toks, offs, t, None, 0, ss.make_policy((), full.base_batch, full.l_max, full.max_batch))
            row = dict(sweep="group", group=n, scheduled_tokens_per_s=useful / (g["stats"]["wall_ms"] / 1e3),
                       vanilla_tokens_per_s=useful / (v["stats"]["wall_ms"] / 1e3),
                       ratio=v["stats"]["wall_ms"] / g["stats"]["wall_ms"], scheduled_steps=g["stats"]["steps"],
                       vanilla_steps=v["stats"]["steps"], n_failed=g["stats"]["n_failed"])
            log(f"sweep group {n}: {row}")
            print(json.dumps(row), flush=True)
    gw.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=3, choices=[2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=0, help="development only: reduced depth (reported in config)")
    ap.add_argument("--no-vanilla", action="store_true", help="skip the vanilla-batching comparison run")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--step-iters", type=int, default=20, help="decode-step timing iterations")
    ap.add_argument("--step-rows", type=int, default=16, help="rows of the timed decode step (roofline legs)")
    ap.add_argument("--step-ctx", type=int, default=200, help="context length of the timed decode step")
    ap.add_argument("--gemm-mode", type=int, default=0, choices=[0, 1, 2, 4, 5, 6, 8],
                    help="small-batch projection kernel: 0 chosen per shape, 1 always k_gemm_skinny, 2 always k_gemm_sweep "
                         "(for A/B profiles; anything but 0 is reported in config)")
    ap.add_argument("--ablation", action="store_true",
                    help="instead of the headline run: the paper's Table 5 ablation (Binning x FCR x VBS), a perfect "
                         "predictor and compaction on the same group, one pass each; prints one JSON line per row")
    ap.add_argument("--ablation-only", default=None,
                    help="with --ablation: run vanilla plus the rows whose name contains this text")
    ap.add_argument("--sweep", choices=["batch", "group", "sync", "step"], default=None,
                    help="instead of the headline run: throughput against micro-batch size or against group size "
                         "(the paper's Fig. 3a / 3b on the synthetic workload), ('sync') the group run with ends "
                         "that the host must poll for, against the poll period, greedy and sampled at T=0.5, or ('step') "
                         "the time of one decode forward against live rows and against context length (App. D)")
    ap.add_argument("--in-flight", type=int, default=4, choices=[1, 2, 3, 4],
                    help="micro-batches of a group pass generated at the same time (SS_OPT_IN_FLIGHT; reported in config)")
    ap.add_argument("--no-cfg4", action="store_true", help="skip the configuration-4 leg of the default run")
    ap.add_argument("--time-budget-s", type=float, default=560.0,
                    help="seconds the whole program should stay within: the optional legs after the timed passes (the "
                         "configuration-4 comparison, then the sampled rerun) shrink or are left out, and say so in the JSON, "
                         "when the passes asked for have already used most of it")
    ap.add_argument("--no-generate", action="store_true",
                    help="skip the leg that reruns the group with sampled tokens and ends discovered by polling")
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the roofline legs (weight-stream kernels and one decode step); the command profiled "
                         "under rocprofv3 for profiles/")
    ap.add_argument("--in-flight-only", action="store_true",
                    help="only the leg that runs --in-flight decode steps at the same time, one per lane (the command "
                         "profiled under rocprofv3 for profiles/decode_steps_in_flight_7b_kernel_trace.txt)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (micro-batches would be dealt to GPUs "
              "host-side, no collective exists to time)", file=sys.stderr)
        return 2

    from paper_2305_13144_amd import binding as ss
    from paper_2305_13144_amd import synth

    ss.lib()  # fail loudly if the HIP library is missing
    ss.ss_set_gemm_mode(a.gemm_mode)
    ss.ss_set_verbose(1 if (a.cfg >= 4 or a.ablation or a.sweep) else 0)   # long groups: a progress line per micro-batch
    wl = synth.make_workload(a.cfg)
    shape = wl.shape if a.layers <= 0 else wl.shape.with_layers(a.layers)
    t0 = time.time()
    W = synth.make_weights(shape, seed=wl.weight_seed, threads=min(16, os.cpu_count() or 8))
    log(f"weights {shape.name}: {sum(t.nbytes for t in W) / 1e9:.2f} GB generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    gw = ss.Weights(shape, W)
    log(f"uploaded + packed in {time.time() - t0:.1f}s")
    gw.set_option(ss.SS_OPT_IN_FLIGHT, a.in_flight)

    pol = ss.make_policy(wl.flags, wl.base_batch, wl.l_max, wl.max_batch)
    vpol = ss.make_policy((), wl.base_batch, wl.l_max, wl.max_batch)

    def run(policy, pred, binw):
        return ss.ss_run_group(gw, wl.prompt_tokens, wl.prompt_offsets, wl.target_lens, pred, binw, policy)

    if a.in_flight_only:
        B0, ctx = a.step_rows, a.step_ctx
        ptoks = np.random.default_rng(7).integers(0, shape.vocab, size=B0 * ctx).astype(np.int32)
        ms_l = ss.ss_bench_decode_steps_in_flight(gw, ptoks, B0, ctx, a.step_iters + 6, a.in_flight)[:, 3:-3]
        ach_l = a.in_flight * decode_step_bytes(shape, B0, ctx) / (ms_l.mean() * 1e-3) / 1e9
        log(f"{a.in_flight} decode steps in flight, B={B0} ctx={ctx}: {ms_l.mean():.3f} ms each -> {ach_l:.0f} GB/s = "
            f"{ach_l / HBM_PEAK_GBS:.3f} of peak for the bytes of all")
        print(json.dumps(dict(lanes=a.in_flight, rows=B0, ctx=ctx, iters_per_lane=int(ms_l.shape[1]), ms=float(ms_l.mean()),
                              achieved=ach_l, unit="GB/s", frac=ach_l / HBM_PEAK_GBS)), flush=True)
        gw.close()
        return 0
    if a.ablation:
        return ablation(a, ss, gw, wl, shape)
    if a.sweep:
        return sweeps(a, ss, gw, wl, shape)

    # ---- timed region: W warmup passes, then exactly K passes over the group ----------------------
    if a.roofline_only:
        a.warmup, a.steps, a.no_vanilla, a.no_cpu, a.no_cfg4 = 0, 0, True, True, True
    for i in range(a.warmup):
        r = run(pol, wl.pred_lens, wl.bin_width)
        log(f"warmup {i}: {r['stats']['wall_ms']:.0f} ms")
    # device-wide synchronize on both sides of the timed region, through the HIP runtime the library
    # itself is linked against (a second HIP runtime in this process, e.g. a framework's own copy, would
    # not see the device once this one has initialised it)
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    assert hip.hipDeviceSynchronize() == 0
    t0 = time.perf_counter()
    for i in range(a.steps):
        r = run(pol, wl.pred_lens, wl.bin_width)
        if a.steps > 1:
            log(f"pass {i + 1}/{a.steps}: {r['stats']['wall_ms']:.0f} ms")     # a long run must not look hung
    assert hip.hipDeviceSynchronize() == 0
    dt = time.perf_counter() - t0
    useful = int(wl.target_lens.sum())
    if a.steps > 0:
        st = r["stats"]
        assert np.array_equal(r["lens"], wl.target_lens)
        value = useful * a.steps / dt
        log(f"cfg{a.cfg}: {useful} useful tokens in {dt / a.steps * 1e3:.0f} ms/pass -> {value:.0f} tok/s; stats {st}")
    else:
        st = dict(steps=0, padded_row_steps=0, computed_row_steps=0, n_failed=0, n_mb_first=0, n_mb_failure=0,
                  prefill_ms=0.0, decode_ms=0.0, plan_ms=0.0, wall_ms=0.0)
        value, dt = 0.0, 0.0

    extras = {}
    if not a.no_vanilla:
        rv = run(vpol, None, 0)
        sv = rv["stats"]
        # vanilla batching by its definition: chunks of base_batch in arrival order, each run to its longest response,
        # every row computed at every step, nothing capped, every query emitted once and in full
        t_ = wl.target_lens
        v_steps = sum(int(t_[c:c + wl.base_batch].max()) for c in range(0, wl.n, wl.base_batch))
        v_padded = sum(int(t_[c:c + wl.base_batch].max()) * len(t_[c:c + wl.base_batch]) for c in range(0, wl.n, wl.base_batch))
        assert np.array_equal(rv["lens"], t_) and sv["n_failed"] == 0 and sv["n_mb_failure"] == 0
        assert sv["steps"] == v_steps and sv["padded_row_steps"] == v_padded == sv["computed_row_steps"]
        assert all((rv["tokens"][i, :t_[i]] >= 0).all() and (rv["tokens"][i, t_[i]:] == -1).all() for i in range(wl.n))
        extras["vanilla_batching"] = dict(
            workload=f"same group, arrival order, batch {wl.base_batch}, no cap (config 2 policy)",
            useful_tokens_per_s=useful / (sv["wall_ms"] / 1e3), ms=sv["wall_ms"], steps=sv["steps"],
            padded_row_steps=sv["padded_row_steps"])
        extras["scheduled_over_vanilla"] = (useful / (st["wall_ms"] / 1e3)) / extras["vanilla_batching"]["useful_tokens_per_s"]
        log(f"vanilla: {sv['wall_ms']:.0f} ms -> ratio {extras['scheduled_over_vanilla']:.3f}")

    pass_s = dt / a.steps if a.steps else 0.0
    reserve_s = 25.0                                     # the perception leg, the roofline legs, cpu_baseline
    skipped = {}

    def budget_left() -> float:
        return a.time_budget_s - (time.time() - T_START) - reserve_s

    if a.in_flight > 1 and a.steps > 0 and not a.roofline_only:
        # the same pass with one micro-batch at a time: what generating several at once is worth on this group
        if 1.3 * pass_s > budget_left():
            skipped["one_microbatch_at_a_time"] = f"left out: {budget_left():.0f} s of the {a.time_budget_s:.0f} s budget remained"
        else:
            gw.set_option(ss.SS_OPT_IN_FLIGHT, 1)
            r1 = run(pol, wl.pred_lens, wl.bin_width)
            gw.set_option(ss.SS_OPT_IN_FLIGHT, a.in_flight)
            assert np.array_equal(r1["tokens"], r["tokens"]) and np.array_equal(r1["lens"], r["lens"])
            assert all(r1["stats"][k] == st[k] for k in ("steps", "padded_row_steps", "computed_row_steps", "n_failed"))
            extras["one_microbatch_at_a_time"] = dict(
                what="the same pass with SS_OPT_IN_FLIGHT = 1: identical tokens and counters, micro-batches one after another",
                in_flight=a.in_flight,
                useful_tokens_per_s=useful / (r1["stats"]["wall_ms"] / 1e3), ms=r1["stats"]["wall_ms"],
                in_flight_over_it=r1["stats"]["wall_ms"] / st["wall_ms"])
            log(f"one micro-batch at a time: {r1['stats']['wall_ms']:.0f} ms -> {a.in_flight} in flight are "
                f"{extras['one_microbatch_at_a_time']['in_flight_over_it']:.3f}x")

    # The configuration-4 leg: one scheduled pass over a group 4x as large with micro-batches of up to 256 rows costs
    # about 2.15 timed passes, the vanilla pass over that group about 4.85 more.  What is left of the time budget after
    # the passes asked for decides its form: both passes on the whole group; or the scheduled pass alone, compared with
    # the vanilla rate just measured on the 256-query group (the same length laws and batch 16: 1,991 against 1,996
    # tokens/s when both are measured); or that on a power-of-two prefix of the group; or nothing.  The JSON says which.
    run_cfg4 = not a.roofline_only and a.cfg == 3 and not a.no_cfg4 and a.layers <= 0 and a.steps > 0
    n4, cfg4_own_vanilla = 1024, True
    if run_cfg4:
        if 7.0 * pass_s > budget_left():
            cfg4_own_vanilla = False
            while n4 > 256 and 2.15 * pass_s * n4 / 1024 > budget_left():
                n4 //= 2
            if 2.15 * pass_s * n4 / 1024 > budget_left() or a.no_vanilla:
                skipped["config4"] = f"left out: {budget_left():.0f} s of the {a.time_budget_s:.0f} s budget remained"
                run_cfg4 = False
    cfg4_cost = (7.0 if cfg4_own_vanilla else 2.15) * pass_s * n4 / 1024 if run_cfg4 else 0.0
    if not a.roofline_only and not a.no_generate and a.steps > 0 and 1.05 * pass_s + cfg4_cost > budget_left():
        skipped["sampled_polled_generation"] = (f"left out: {budget_left():.0f} s of the {a.time_budget_s:.0f} s budget remained; "
                                                "profiles/polled_generation_sync_sweep_7b.md has this leg's figures")
        a.no_generate = True
    if not a.roofline_only and not a.no_generate and a.steps > 0:
        # The same group when the host does not know the lengths (Sec. 4.2, Experimental Setting, of the paper samples at T = 0.5 and rows
        # end by themselves): tokens drawn by the sampling kernel, the same lengths applied on the device as
        # simulated ends, the host polling the unfinished-row count after every decode forward (the period that
        # profiles/polled_generation_sync_sweep_7b.md shows to be the cheapest).
        draws = synth.make_draws(wl.n, wl.l_max, seed=20230513)
        rg = ss.ss_run_group_generate(gw, wl.prompt_tokens, wl.prompt_offsets, wl.pred_lens, wl.bin_width, pol,
                                      eos_id=-1, temperature=0.5, draws=draws, target_lens=wl.target_lens, sync_every=1)
        assert np.array_equal(rg["lens"], wl.target_lens)
        sg = rg["stats"]
        extras["sampled_polled_generation"] = dict(
            what="same group and policy; tokens sampled at T=0.5 on the device, ends applied on the device and "
                 "discovered by the host polling after every decode forward",
            useful_tokens_per_s=useful / (sg["wall_ms"] / 1e3), ms=sg["wall_ms"], steps=sg["steps"], polls=sg["polls"],
            idle_steps=sg["idle_steps"], n_failed=sg["n_failed"],
            over_known_lengths=(useful / (sg["wall_ms"] / 1e3)) / (useful / (st["wall_ms"] / 1e3)))
        log(f"sampled + polled: {sg['wall_ms']:.0f} ms ({sg['steps']} forwards, {sg['polls']} polls, "
            f"{sg['idle_steps']} idle) -> {extras['sampled_polled_generation']['over_known_lengths']:.3f} of the "
            f"known-length pass")

    if not a.roofline_only and wl.pred_lens is not None:
        # Length-perception overhead, simulated (Sec. 4.1, "Overhead of Length Prediction": one prompt forward plus
        # 2-3 generated tokens per query before anything can be scheduled).  No predictor is built; this only puts
        # its cost next to the gain: every query gets a prompt forward + 3 tokens, 64 queries per micro-batch.
        t_p = 0.0
        for lo in range(0, wl.n, 64):
            idx = list(range(lo, min(wl.n, lo + 64)))
            ptk, pof = synth.gather_prompts(wl, idx)
            rp = ss.ss_decode_microbatch(gw, ptk, pof, 3, np.full(len(idx), 3, np.int32), 0)
            t_p += rp["stats"]["prefill_ms"] + rp["stats"]["decode_ms"]
        extras["simulated_length_perception"] = dict(
            what="prompt forward + 3 generated tokens for every query, 64 per micro-batch, before scheduling",
            ms=t_p, useful_tokens_per_s_including_it=useful / ((st["wall_ms"] + t_p) / 1e3))
        log(f"simulated perception overhead: {t_p:.0f} ms on top of {st['wall_ms']:.0f} ms")

    if run_cfg4:
        # The case the method gains most on this hardware, beside the headline's fixed batch of 16: configuration 4
        # (same weights, group 1024, variable batch size up to 256 rows, compaction) against vanilla batching on
        # its own group.  When the run has already taken long (many timed passes), a prefix of that group stands in
        # for it; the JSON says which.
        w4 = synth.make_workload(4)
        idx4 = list(range(n4))
        tk4, of4 = synth.gather_prompts(w4, idx4)
        t4, p4 = w4.target_lens[idx4], w4.pred_lens[idx4]
        pol4 = ss.make_policy(w4.flags, w4.base_batch, w4.l_max, w4.max_batch)
        ss.ss_set_verbose(0)
        r4 = ss.ss_run_group(gw, tk4, of4, t4, p4, w4.bin_width, pol4)
        assert np.array_equal(r4["lens"], t4)
        u4 = int(t4.sum())
        s4 = r4["stats"]
        tps4 = u4 / (s4["wall_ms"] / 1e3)
        extras["config4"] = dict(
            workload=f"config 4: {shape.name}, group {n4}" + ("" if n4 == w4.n else f" (first {n4} of {w4.n} queries)")
                     + f", policy {'+'.join(w4.flags)} bin {w4.bin_width}, batch {w4.base_batch}..{w4.max_batch}",
            useful_tokens_per_s=tps4, ms=s4["wall_ms"], steps=s4["steps"], n_failed=s4["n_failed"],
            micro_batches=[s4["n_mb_first"], s4["n_mb_failure"]], computed_row_steps=s4["computed_row_steps"])
        if cfg4_own_vanilla:
            v4 = ss.ss_run_group(gw, tk4, of4, t4, None, 0, ss.make_policy((), w4.base_batch, w4.l_max, w4.max_batch))
            assert np.array_equal(v4["lens"], t4)
            sv4 = v4["stats"]
            extras["config4"].update(vanilla="batch 16 in arrival order on this same group, measured in this run",
                                     vanilla_useful_tokens_per_s=u4 / (sv4["wall_ms"] / 1e3), vanilla_ms=sv4["wall_ms"],
                                     vanilla_steps=sv4["steps"], scheduled_over_vanilla=sv4["wall_ms"] / s4["wall_ms"])
        else:
            vt = extras["vanilla_batching"]["useful_tokens_per_s"]
            extras["config4"].update(vanilla="the time budget left no room for a vanilla pass over this group: the rate is the one "
                                             "measured in this run on the 256-query group (same length laws, batch 16)",
                                     vanilla_useful_tokens_per_s=vt, scheduled_over_vanilla=tps4 / vt)
        log(f"config 4 (group {n4}): {s4['wall_ms']:.0f} ms scheduled, {tps4:.0f} tok/s -> "
            f"{extras['config4']['scheduled_over_vanilla']:.2f}x vanilla ({'own' if cfg4_own_vanilla else 'config-2'} vanilla pass)")

    # ---- roofline: one whole decode step, timed live with HIP events; its projection launches and a plain read
    # ---- stream over the same matrices as sub-entries -------------------------------------------------------------
    B0, ctx = a.step_rows, a.step_ctx
    ms_w, launches = ss.ss_bench_weight_stream(gw, B0, a.step_iters + 3)
    log("weight stream iterations (ms): " + " ".join(f"{x:.2f}" for x in ms_w))
    ms_w = ms_w[3:]
    wbytes = shape.weight_bytes_per_step() - (2 * shape.n_layers + 1) * shape.d_model * 2   # matrices only
    ach_w = wbytes / (ms_w.mean() * 1e-3) / 1e9
    # the ceiling for those launches: the same matrices read by a plain stream kernel, launch by launch
    ms_r, rbytes = ss.ss_bench_read_stream(gw, a.step_iters + 3)
    ms_r = ms_r[3:]
    rng = np.random.default_rng(7)
    ptoks = rng.integers(0, shape.vocab, size=B0 * ctx).astype(np.int32)
    ms_s = ss.ss_bench_decode_step(gw, ptoks, B0, ctx, a.step_iters + 3)[3:]
    sbytes = decode_step_bytes(shape, B0, ctx)
    ach = sbytes / (ms_s.mean() * 1e-3) / 1e9
    # several such steps at once, one per lane, as a group pass runs its micro-batches: each streams the whole model
    # (not under --roofline-only: the profiles taken from that command keep every kernel's launches undisturbed)
    two = None
    if not a.roofline_only and a.in_flight > 1:
        per_lanes = {}
        for lanes in sorted({2, a.in_flight}):
            ms_l = ss.ss_bench_decode_steps_in_flight(gw, ptoks, B0, ctx, a.step_iters + 6, lanes)[:, 3:-3]
            ach_l = lanes * sbytes / (ms_l.mean() * 1e-3) / 1e9
            per_lanes[lanes] = dict(ms=float(ms_l.mean()), achieved=ach_l, frac=ach_l / HBM_PEAK_GBS)
        two = dict(what=f"{a.in_flight} such steps running at the same time on {a.in_flight} streams (as many micro-batches of a "
                        "group pass): bytes of all / the time one of them takes then",
                   lanes=a.in_flight, unit="GB/s", **per_lanes[a.in_flight],
                   **({"with_two_lanes": per_lanes[2]} if a.in_flight != 2 else {}))
    step_launches = launches + 3 * shape.n_layers + 3     # + attention and two norms per layer, embedding, final norm, token choice
    traffic, traffic_source = profile_traffic(shape.name, B0, ctx, a.gemm_mode)
    roofline = dict(bound="hbm",
                    kernel=f"one whole decode step of {B0} rows at context {ctx}: all {step_launches} launches (projections, "
                           f"decode attention, RMSNorm, embedding, token choice)",
                    achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS, traffic=traffic,
                    traffic_source=traffic_source, ms=float(ms_s.mean()), ms_min=float(ms_s.min()),
                    algorithmic_bytes=sbytes, launches_per_step=step_launches,
                    steps_in_flight=two,
                    projection_launches=dict(
                        what="the projection kernels of that step alone (k_gemm_sweep + k_gemm_skinny), back to back",
                        ms=float(ms_w.mean()), achieved=ach_w, unit="GB/s", frac=ach_w / HBM_PEAK_GBS, launches=launches,
                        avg_launch_us=ms_w.mean() * 1e3 / launches, bytes_per_launch=wbytes / launches),
                    plain_read_stream=dict(
                        what="one plain non-temporal read kernel per weight matrix, same bytes and launch sizes, nothing computed",
                        ms=float(ms_r.mean()), achieved=rbytes / (ms_r.mean() * 1e-3) / 1e9, unit="GB/s",
                        projections_over_stream=float(ms_r.mean() / ms_w.mean()) * wbytes / rbytes))
    extras["decode_step"] = dict(rows=B0, ctx=ctx, ms=float(ms_s.mean()), ms_min=float(ms_s.min()),
                                 algorithmic_bytes=sbytes, achieved_GBs=ach, frac_of_hbm_peak=ach / HBM_PEAK_GBS)
    log(f"plain read stream over the same matrices: {ms_r.mean():.3f} ms/iter -> {roofline['plain_read_stream']['achieved']:.0f} GB/s")
    log(f"weight stream: {ms_w.mean():.3f} ms/iter -> {ach_w:.0f} GB/s; decode step B={B0} ctx={ctx}: "
        f"{ms_s.mean():.3f} ms -> {ach:.0f} GB/s = {ach / HBM_PEAK_GBS:.3f} of peak"
        + (f"; {two['lanes']} in flight: {two['ms']:.3f} ms each -> {two['achieved']:.0f} GB/s = {two['frac']:.3f}" if two else ""))
    if a.roofline_only:
        # calibration for the HBM byte counters: a plain device-to-device copy of known size (1 GiB read,
        # 1 GiB written) shows up in the same trace as a copyBuffer dispatch.  It runs after the timed legs:
        # allocating and freeing 2 GiB before the library's first workspace allocation changes where that
        # workspace lands and was measured to slow the projection kernels down by 6 %.
        size = 1 << 30
        src, dst = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipMalloc(ctypes.byref(src), ctypes.c_size_t(size)) == 0
        assert hip.hipMalloc(ctypes.byref(dst), ctypes.c_size_t(size)) == 0
        assert hip.hipMemset(src, 1, ctypes.c_size_t(size)) == 0
        assert hip.hipMemcpy(dst, src, ctypes.c_size_t(size), 3) == 0     # hipMemcpyDeviceToDevice
        assert hip.hipDeviceSynchronize() == 0
        hip.hipFree(src)
        hip.hipFree(dst)

    gw.close()

    # ---- cpu_baseline: the oracle as it stands, on a bounded sample of the same workload -----------
    cpu = None
    if not a.no_cpu:
        from oracle.model_oracle import OracleModel
        om = OracleModel(shape, W, "f32")
        rows, cap = [0, 1, 2, 3, 4, 5], 48
        toks, offs = synth.gather_prompts(wl, rows)
        tl = np.minimum(wl.target_lens[rows], cap)
        t0 = time.perf_counter()
        ro = om.greedy_microbatch(toks, offs, cap, tl, margins=False)
        dtc = time.perf_counter() - t0
        cpu = dict(value=float(ro["lens"].sum() / dtc), unit="tokens/s", cores=int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                   kind="oracle",
                   sample=f"fp32 build of the oracle; queries 0-{len(rows) - 1} of the group as one micro-batch, cap {cap}: "
                          f"{int(offs[-1])} prompt token-rows + {int(ro['lens'].sum())} generated tokens in {dtc:.1f}s")
        log(f"cpu oracle: {cpu}")

    out = dict(metric="useful_generated_tokens_per_s", value=value, unit="tokens/s", n_gpus=1, steps=a.steps,
               warmup=a.warmup, ms_per_step=(dt / a.steps * 1e3 if a.steps else 0.0), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16", data="synthetic",
               config=dict(workload=f"config {a.cfg}: {shape.name}, group {wl.n}, policy {'+'.join(wl.flags) or 'vanilla'}"
                                    f" bin {wl.bin_width} base batch {wl.base_batch} L_max {wl.l_max}"
                                    + (f", {a.in_flight} micro-batches in flight" if a.in_flight > 1 else ""),
                           group=wl.n, useful_tokens=useful, steps_per_pass=st["steps"],
                           padded_row_steps=st["padded_row_steps"], computed_row_steps=st["computed_row_steps"],
                           n_failed=st["n_failed"], micro_batches=[st["n_mb_first"], st["n_mb_failure"]],
                           samples_per_s=(wl.n * a.steps / dt if a.steps else 0.0), prefill_ms=st["prefill_ms"], decode_ms=st["decode_ms"],
                           plan_ms=st["plan_ms"], microbatches_in_flight=a.in_flight,
                           precision="weights: bf16 values, held as IEEE half (exact); projection inputs and key/value slots: "
                                     "IEEE half; MFMA f16 x f16 with fp32 accumulation; softmax, norms, residual stream fp32", **({"reduced_layers": a.layers} if a.layers > 0 else {}),
                           **({"gemm_mode": a.gemm_mode} if a.gemm_mode else {})),
               roofline=roofline, cpu_baseline=cpu, paper_context=PAPER_CONTEXT,
               **({"legs_left_out": skipped} if skipped else {}), **extras)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
