#!/usr/bin/env python3
"""Benchmark of the early-exit head evaluation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Default workload (the one the headline metric is quoted on): batch-1 decode,
Pythia-410M-shaped heads (d=1024, V=50304, 23 exit heads + final, bf16 weights,
fp32 accumulation).  One "step" is one pass of the whole hot path over one
batch of synthetic input: 2048 seeded decode steps, each a dynamic-exit cascade
(LayerNorm -> projection -> streaming entropy/argmax -> threshold test) that
stops at the first head with H < tau.  All inputs are resident in HBM before
the timed region starts.

Prints ONE JSON line:  value = (row, head) evaluations per second over the
timed steps; "roofline" = algorithmic bytes of the dominant kernel per launch
over its average launch duration (HIP events on the launch stream) against
the 8 TB/s HBM peak; "cpu_baseline" = the fp64 CPU oracle timed on a bounded
sample of the same workload on this machine's host cores (all BLAS threads, and
one thread as "value_1core").

Without --workload the line is the decode workload's and carries two more
objects, timed in the same run: "batched" = the batched configurations
(calibration pass on 512 tokens against the matrix-core peak; 64-row dynamic
exit and 144-position verification against the HBM peak), each with its own
evaluations/s, time per head and roofline object, and "read_ceiling" = what a
plain read of the same weight buffers reaches on this chip.  With --workload
NAME only that workload runs and the line is its own.
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

HBM_PEAK_GBS = 8000.0
# HBM traffic of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs scaled
# by what the same counters read for a plain 1 GiB elementwise kernel (factors 2.0 and 1.0):
# measured bytes per launch / algorithmic bytes per launch of the same launches
# (profiles/c1_decode_persistent_kernel.md).  Reported as that ratio times this run's
# algorithmic bytes per launch.
TRAFFIC_RATIO_C1 = (1.9298e9 + 1.43e6) / 1.7635e9
# The same for the batched projection kernel (profiles/c2_calib_gemm32_kernel.md,
# profiles/c3_dynexit_c4_verify_kernels.md): measured HBM bytes per head.
TRAFFIC_BYTES_C2 = 271.4e6 + 1.31e6        # 206 MB of weights, read 1.3 times by the two token groups
TRAFFIC_RATIO_C3 = (264.9e6 + 0.70e6) / 257.75e6
TRAFFIC_RATIO_C4 = (272.4e6 + 2.32e6) / 258.29e6
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=None,
                    choices=["c1_decode", "c2_calib", "c3_dynexit", "c4_verify", "f1_calibrate", "f3_draft", "f4_losses",
                             "read_ceiling", "mfma_ceiling"])
    ap.add_argument("--batched-steps", type=int, default=100,
                    help="timed steps of each batched configuration in the default run (their steps are milliseconds)")
    ap.add_argument("--batched-warmup", type=int, default=20)
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per bench step (c1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of known size (1 GiB read + 1 GiB written each), "
                         "to scale rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--metrics", action="store_true",
                    help="c2_calib only: also produce the maximum probability and the top-2 probability "
                         "difference of every (head, token) (eh_eval_heads_metrics)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def event_ms(fn, torch):
    """Run fn() between two HIP events on the current (launch) stream."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1)


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return os.cpu_count() or 1


def cpu_head_evals(args, G, heads, chunks, what):
    """Time the oracle's head evaluation on (head, rows) chunks until the CPU budget is used.
    Widening a head's weights to fp64 is input marshalling and is not timed."""
    from oracle import eh_oracle as O
    f64 = G.to_f64_numpy
    done, spent, n_chunks = 0, 0.0, 0
    cached = (None, None)
    for l, rows in chunks:
        if cached[0] != l:
            cached = (l, (f64(heads.W[l]), f64(heads.gamma[l]), f64(heads.beta[l])))
        W64, g64, b64 = cached[1]
        h64 = f64(rows)
        c0 = time.perf_counter()
        O.head_eval(h64, g64, b64, W64, 1e-5, True)
        spent += time.perf_counter() - c0
        done += h64.shape[0]
        n_chunks += 1
        if spent > args.cpu_seconds:
            break
    return {"value": done / spent, "unit": "evals/s", "cores": oracle_threads(), "kind": "oracle",
            "sample": f"{what}: {n_chunks} chunks, {done} evaluations, {spent:.1f} s (fp64 numpy, weights pre-widened)"}


def bench_calibrate(args, torch, B, G, dev):
    """Threshold calibration of one head (the step after config 2 in the paper's pipeline):
    M = 2^24 calibration tokens, the paper's sweep of 11 confidence levels in one call."""
    import numpy as np
    M = 1 << 24
    eps = [0.5 + 0.05 * i for i in range(11)]
    t_setup = time.time()
    w = G.Workload("calib", d=64, V=64, n_heads=1, rows=4, dtype="bf16", seed=1)
    heads = G.make_heads(w, dev)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=4)
    sets = [G.make_calibration_case(M, dev, seed=s, ties=False) for s in range(2)]
    tau = torch.zeros(len(eps), device=dev)
    n_exit = torch.zeros(len(eps), dtype=torch.int64, device=dev)

    def step(i):
        H, pred, ref = sets[i % len(sets)]
        B.eh_calibrate(ctx, H, pred, ref, eps, tau, n_exit)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev_s = ev0.elapsed_time(ev1) * 1e-3
    value = args.steps * M / dt
    # algorithmic bytes: each token's entropy and two predictions are read once (12 B); the
    # 11 thresholds and counts written are negligible.  The call as a whole is timed (every
    # kernel of it, and the read-back of one word that ends it).
    sorted_calls = B.eh_probe_calibrate_sorted(ctx)
    bytes_per_launch = 12.0 * M
    avg_s = ev_s / args.steps
    roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": None,
            "kernel": "eh_calibrate (one pass that packs correctness and finds the key range, three passes "
                      "that count entropies into bins, three small kernels that keep bins per level)",
            "avg_launch_us": avg_s * 1e6, "bytes_per_launch": bytes_per_launch, "launches": args.steps,
            "calls_served_by_full_sort": sorted_calls}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import eh_oracle as O
        m = 12000                                  # the oracle is quadratic: a bounded sample
        H, pred, ref = G.make_calibration_case(m, "cpu", seed=0)
        Hc = H.numpy().astype(np.float64)
        t = O.correctness(pred.numpy(), ref.numpy())
        c0 = time.perf_counter()
        n_lv = 0
        for e in eps:
            O.calibrate_threshold(Hc, t, e)
            n_lv += 1
            if time.perf_counter() - c0 > args.cpu_seconds:
                break
        cdt = time.perf_counter() - c0
        cpu = {"value": m * n_lv / len(eps) / cdt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
               "sample": f"{m} tokens, {n_lv} of {len(eps)} levels ({cdt:.1f} s); the oracle is the literal "
                         "quadratic definition, so its rate falls with the size of the set"}
    B.eh_destroy(ctx)
    line = {"metric": "calibration_tokens_per_sec", "value": value, "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
            "data": "synthetic",
            "config": {"workload": f"f1_calibrate: one head, M = {M} calibration tokens, {len(eps)} confidence "
                                   "levels 0.5 ... 1.0 per call", "tau": [float(x) for x in tau.cpu()]},
            "roofline": roof, "cpu_baseline": cpu, "setup_s": round(time.time() - t_setup, 1)}
    print(json.dumps(line), flush=True)


def bench_draft(args, torch, B, G, dev):
    """DSSD drafting phase on the device (the controller around config 1's cascade): the decode
    workload's positions in windows of `limit` = 32, one dssd_draft call per window."""
    import numpy as np
    w = G.CONFIGS["c1_decode"]
    limit = 32
    n_dec = args.decode_steps or w.steps
    n_win = n_dec // limit
    t_setup = time.time()
    heads = G.make_heads(w, dev)
    hid = G.make_hidden(w, heads, dev, rows=n_dec)               # [n_heads, n_dec, d]
    tau = G.tau_linear(w)
    # Two regimes per bench step, over the same windows: the workload's own thresholds, under
    # which a window soon meets a position no exit head is confident about (the drafter falls
    # back to the full model), and thresholds whose deepest exit head always exits, under which
    # every window drafts until the buffer is full.
    tau_full = list(tau)
    tau_full[w.n_heads - 2] = float("inf")
    regimes = [("calibrated", tau), ("deepest_exit_head_always_confident", tau_full)]
    ctxs = [B.eh_create(heads.W, heads.gamma, heads.beta, t, max_rows=1) for _, t in regimes]
    hp = hid.h.permute(1, 0, 2)                                  # [position, head, d]
    wins = [hp[i * limit:(i + 1) * limit] for i in range(n_win)]
    nr = len(regimes)
    draft = torch.zeros((nr, n_win, limit), dtype=torch.int32, device=dev)
    layers = torch.zeros((nr, n_win, limit), dtype=torch.int32, device=dev)
    ln = torch.zeros((nr, n_win), dtype=torch.int32, device=dev)
    reason = torch.zeros((nr, n_win), dtype=torch.int32, device=dev)
    fb = torch.zeros((nr, n_win), dtype=torch.int32, device=dev)
    nev = torch.zeros((nr, 1), dtype=torch.int64, device=dev)

    def step():
        for r, ctx in enumerate(ctxs):
            for i in range(n_win):
                B.dssd_draft(ctx, wins[i], limit, -1, draft[r, i], ln[r, i:i + 1], layers[r, i], reason[r, i:i + 1],
                             fb[r, i:i + 1], nev[r])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    nev.zero_()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev_s = ev0.elapsed_time(ev1) * 1e-3
    for ctx in ctxs:
        B.eh_check(ctx)
    evals = int(nev.sum().item())
    drafted = int(ln.sum().item())
    fallbacks = int((reason == 2).sum().item())
    live = (drafted + fallbacks) * args.steps                   # cascades that did work
    per_regime = {}
    for r, (name, _) in enumerate(regimes):
        stops = torch.bincount(reason[r].long(), minlength=4).tolist()
        per_regime[name] = {"drafted_tokens_per_step": int(ln[r].sum().item()),
                            "evals_per_step": int(nev[r].item()) // args.steps,
                            "windows_by_stop_reason": {"limit": stops[0], "eos": stops[1], "fallback": stops[2],
                                                       "exhausted": stops[3]}}
    esz = 2
    bytes_per_eval = w.d * w.V * esz + w.d * esz + 12
    # the cascades that run are the dominant kernel; the launches behind a stop return at once.
    # The whole timed region (controllers and empty launches included) is charged to them.
    bytes_per_launch = bytes_per_eval * evals / live
    avg_s = ev_s / live
    roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": TRAFFIC_RATIO_C1 * bytes_per_launch,
            "kernel": "eh::decode_kernel<DtBf16> (one live launch = one drafted position's cascade)",
            "avg_launch_us": avg_s * 1e6, "bytes_per_launch": bytes_per_launch, "launches": live}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import eh_oracle as O
        f64 = G.to_f64_numpy
        W64 = [f64(Wl) for Wl in heads.W]
        g64 = [f64(g) for g in heads.gamma]
        b64 = [f64(b) for b in heads.beta]
        c_evals, c_wins = 0, 0
        c0 = time.perf_counter()
        for i in range(n_win):
            Ht, At = [], []
            for t in range(i * limit, (i + 1) * limit):
                hl = [f64(hid.h[l, t:t + 1]) for l in range(w.n_heads)]
                r = O.cascade(hl, g64, b64, W64, tau, w.ln_eps, True)
                e = int(r["exit_layer"][0])
                # heads behind the exit are never consulted by the drafting rule: NaN = never confident
                Ht.append([float(r["H"][l][0]) if l <= e else float("nan") for l in range(w.n_heads)])
                At.append([int(r["token"][0]) if l == e else -1 for l in range(w.n_heads)])
                if e == w.n_heads - 1:
                    break
            res = O.dssd_draft(Ht, At, tau, limit, -1)
            c_evals += res["n_evals"]
            c_wins += 1
            if time.perf_counter() - c0 > args.cpu_seconds:
                break
        cdt = time.perf_counter() - c0
        cpu = {"value": c_evals / cdt, "unit": "evals/s", "cores": oracle_threads(), "kind": "oracle",
               "sample": f"first {c_wins} windows of the same workload ({c_evals} evaluations, {cdt:.1f} s; "
                         "fp64 numpy cascade per position, then the drafting rule)"}
    for ctx in ctxs:
        B.eh_destroy(ctx)
    line = {"metric": "exit_head_evals_per_sec", "value": evals / dt, "unit": "evals/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"f3_draft: d=1024 V=50304 24 heads batch-1 bf16, {n_win} drafting windows of "
                                   f"{limit} positions per bench step under each of two sets of thresholds, draft "
                                   "until the buffer is full or no exit head is confident",
                       "windows": n_win, "limit": limit, "regimes": per_regime,
                       "drafted_tokens_per_sec": drafted * args.steps / dt,
                       "mean_evals_per_live_position": evals / live},
            "roofline": roof, "cpu_baseline": cpu, "setup_s": round(time.time() - t_setup, 1)}
    print(json.dumps(line), flush=True)


def bench_losses(args, torch, B, G, dev):
    """The training objectives of Section 3.3, forward only, on config 2's shape: one step = the
    KL / cross-entropy / hybrid objectives of each of the 23 exit heads against the model's head
    on 512 tokens (one eh_head_losses call per exit head)."""
    import numpy as np
    w = G.CONFIGS["c2_calib"]
    t_setup = time.time()
    heads = G.make_heads(w, dev)
    hid = G.make_hidden(w, heads, dev)
    R, fin = w.rows, w.n_heads - 1
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    labels = torch.randint(0, w.V, (R,), generator=gen, device=dev, dtype=torch.int32)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    loss = torch.zeros((fin, 3), device=dev)

    def step():
        for l in range(fin):
            B.eh_head_losses(ctx, l, hid.h[l], hid.h[fin], labels, R, 0.5, None, None, loss[l])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev_s = ev0.elapsed_time(ev1) * 1e-3
    launches = args.steps * fin
    flops_per_launch = 2 * 2.0 * w.d * w.V * R          # two projections per call
    avg_s = ev_s / launches
    roof = {"bound": "mfma", "achieved": flops_per_launch / avg_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": flops_per_launch / avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
            "kernel": "eh::gemm32_kl_kernel<2> (one launch = one exit head and the model's head on 512 tokens; the "
                      "time per launch includes the two LayerNorm launches and the two reductions of the call)",
            "avg_launch_us": avg_s * 1e6, "flops_per_launch": flops_per_launch, "launches": launches}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import eh_oracle as O
        f64 = G.to_f64_numpy
        Wt, gt, bt = f64(heads.W[fin]), f64(heads.gamma[fin]), f64(heads.beta[fin])
        lab = labels.cpu().numpy()
        done, spent, n_heads_done = 0, 0.0, 0
        for l in range(fin):
            Wl, gl, bl = f64(heads.W[l]), f64(heads.gamma[l]), f64(heads.beta[l])
            hs, ht = f64(hid.h[l][:128]), f64(hid.h[fin][:128])
            c0 = time.perf_counter()
            O.head_losses(hs, ht, gl, bl, Wl, gt, bt, Wt, lab[:128], 0.5, 1e-5, True)
            spent += time.perf_counter() - c0
            done += 128
            n_heads_done += 1
            if spent > args.cpu_seconds:
                break
        cpu = {"value": done / spent, "unit": "token-head losses/s", "cores": oracle_threads(), "kind": "oracle",
               "sample": f"the first 128 tokens of {n_heads_done} exit heads ({done} loss terms, {spent:.1f} s; "
                         "fp64 numpy, weights pre-widened)"}
    B.eh_destroy(ctx)
    line = {"metric": "head_loss_terms_per_sec", "value": launches * R / dt, "unit": "token-head losses/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"f4_losses: d=2048 V=50304, {fin} exit heads x 512 tokens bf16 against the model's "
                                   "head: KL, cross-entropy and hybrid objective per head",
                       "L_kl_head0": float(loss[0, 1].item()), "L_ce_head0": float(loss[0, 0].item())},
            "roofline": roof, "cpu_baseline": cpu, "setup_s": round(time.time() - t_setup, 1)}
    print(json.dumps(line), flush=True)


def timed(torch, step, steps, warmup):
    """warmup untimed steps, then `steps` timed ones between HIP events on the launch stream
    (and the host clock around the same region).  Returns (host seconds, event seconds); the
    median, minimum and maximum time of a step, from an event behind every step, are left in
    timed.step_ms."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    host_s = time.perf_counter() - t0
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))
    timed.step_ms = {"median": per[len(per) // 2], "min": per[0], "max": per[-1]}
    return host_s, evs[0].elapsed_time(evs[-1]) * 1e-3


timed.step_ms = None


def oracle_rate(run_some, seconds):
    """Times the oracle twice on the same sample recipe: with one BLAS thread for about a
    third of the budget, then with all of them.  run_some(deadline_seconds) -> (units, spent)."""
    out = {}
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1, user_api="blas"):
            n1, t1 = run_some(max(2.0, seconds / 3.0))
        out["value_1core"] = n1 / t1
        out["sample_1core"] = f"{n1} units in {t1:.1f} s with one BLAS thread"
    except Exception as e:        # threadpoolctl missing: the all-thread figure alone
        out["value_1core"] = None
        out["sample_1core"] = f"not measured ({type(e).__name__})"
    n, t = run_some(seconds)
    out["value"] = n / t
    return out, n, t


def run_c1(args, torch, B, G, dev, steps, warmup, cpu_leg, ceiling):
    import numpy as np
    w = G.CONFIGS["c1_decode"]
    heads = G.make_heads(w, dev)
    esz = 2
    n_dec = args.decode_steps or w.steps
    hid = G.make_hidden(w, heads, dev, rows=n_dec)           # [n_heads, n_dec, d]
    tau = G.tau_linear(w)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=16)
    ex = torch.full((n_dec,), -1, dtype=torch.int32, device=dev)
    tok = torch.full((n_dec,), -1, dtype=torch.int32, device=dev)
    nev = torch.zeros(1, dtype=torch.int64, device=dev)
    views = [hid.h[:, t:t + 1] for t in range(n_dec)]

    def step():
        for t in range(n_dec):
            B.eh_cascade(ctx, views[t], 1, ex[t:t + 1], tok[t:t + 1], None, nev)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    nev.zero_()
    dt, ev_s = timed(torch, step, steps, 0)
    B.eh_check(ctx)                       # raises if the kernel reported a device-side failure
    evals = int(nev.item())
    # Dominant kernel: the persistent decode kernel, one launch per decode step (LayerNorm,
    # projection, entropy/argmax, exchange and exit test of every head up to the exit head).
    # Algorithmic bytes per launch = evaluations in that launch x (weights of one head + one
    # hidden row + 12 bytes of results); average launch duration from HIP events around the
    # timed region, on the stream the launches went to (launches are back to back).
    launches = steps * n_dec
    bytes_per_eval = w.d * w.V * esz + w.d * esz + 12
    bytes_per_launch = bytes_per_eval * evals / launches
    avg_s = ev_s / launches
    roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS,
            "traffic": TRAFFIC_RATIO_C1 * bytes_per_launch,
            "kernel": "eh::decode_kernel<DtBf16> (one launch = one decode step's cascade)",
            "avg_launch_us": avg_s * 1e6, "bytes_per_launch": bytes_per_launch, "launches": launches}
    cfg = {"workload": "c1_decode: d=1024 V=50304 24 heads batch-1 bf16, "
                       f"{n_dec} decode steps per bench step, exit at first H<tau",
           "decode_steps": n_dec, "mean_evals_per_decode_step": evals / launches,
           "mean_exit_layer": float(ex.float().mean().item())}
    res = {"value": evals / dt, "ms_per_step": dt / steps * 1e3, "step_ms": timed.step_ms, "roofline": roof, "config": cfg, "dtype": w.dtype,
           "cpu_baseline": None}
    if ceiling:
        res["read_ceiling"] = read_ceiling(torch, B, ctx, w, dev)
    if cpu_leg:
        from oracle import eh_oracle as O
        f64 = G.to_f64_numpy
        W64 = [f64(Wl) for Wl in heads.W]                      # input marshalling, not timed
        g64 = [f64(g) for g in heads.gamma]
        b64 = [f64(b) for b in heads.beta]

        def run_some(seconds):
            done_evals, t0 = 0, time.perf_counter()
            for t in range(0, n_dec):
                hl = [f64(hid.h[l, t:t + 1]) for l in range(w.n_heads)]
                r = O.cascade(hl, g64, b64, W64, tau, w.ln_eps, True)
                done_evals += int(r["exit_layer"][0]) + 1
                if time.perf_counter() - t0 > seconds:
                    break
            return done_evals, time.perf_counter() - t0

        rates, n, t = oracle_rate(run_some, args.cpu_seconds)
        res["cpu_baseline"] = {"value": rates["value"], "unit": "evals/s", "cores": oracle_threads(), "kind": "oracle",
                               "value_1core": rates["value_1core"],
                               "sample": f"the first decode steps of the same workload ({n} evaluations, {t:.1f} s; fp64 "
                                         f"numpy, weights pre-widened); one core: {rates['sample_1core']}"}
    B.eh_destroy(ctx)
    return res


def read_ceiling(torch, B, ctx, w, dev, reps=5):
    """A plain read of the context's weight buffers: what the chip delivers to the simplest
    streaming kernel, as one launch over all heads and as one launch per head, with loads into
    registers (the decode kernel's way) and straight into LDS (the batched kernel's way)."""
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)
    out = {"unit": "GB/s", "peak": HBM_PEAK_GBS, "heads": w.n_heads}
    for how, hname in ((B.PROBE_READ_REGISTERS, "registers"), (B.PROBE_READ_LDS, "lds")):
        for per_head, lname in ((False, "one_launch"), (True, "launch_per_head")):
            nbytes = B.eh_probe_read_weights(ctx, how, per_head, 0, w.n_heads, sink)     # warm-up
            torch.cuda.synchronize()
            ms = event_ms(lambda: [B.eh_probe_read_weights(ctx, how, per_head, 0, w.n_heads, sink) for _ in range(reps)],
                          torch)
            out[f"{hname}_{lname}"] = nbytes * reps / (ms * 1e-3) / 1e9
    out["bytes_per_sweep"] = nbytes
    return out


def run_c2(args, torch, B, G, dev, steps, warmup, cpu_leg):
    # every head on every token; one step = all 24 heads on 512 tokens (eh_eval_heads)
    w = G.CONFIGS["c2_calib"]
    heads = G.make_heads(w, dev)
    hid = G.make_hidden(w, heads, dev)
    R = w.rows
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    Hb = torch.zeros((w.n_heads, R), device=dev)
    Lb = torch.zeros((w.n_heads, R), device=dev)
    Ab = torch.zeros((w.n_heads, R), dtype=torch.int32, device=dev)
    Pb = torch.zeros((w.n_heads, R), device=dev)
    Mb = torch.zeros((w.n_heads, R), device=dev)

    def step():
        # all heads in one call: one LayerNorm launch, one projection launch, one launch for the final merges
        if args.metrics:
            B.eh_eval_heads_metrics(ctx, 0, w.n_heads, hid.h, R, Hb, Lb, Ab, Pb, Mb)
        else:
            B.eh_eval_heads(ctx, 0, w.n_heads, hid.h, R, Hb, Lb, Ab)

    dt, ev_s = timed(torch, step, steps, warmup)
    evals = steps * w.n_heads * R
    launches = steps * w.n_heads
    flops_per_launch = 2.0 * w.d * w.V * R
    avg_s = ev_s / launches
    roof = {"bound": "mfma", "achieved": flops_per_launch / avg_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": flops_per_launch / avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "traffic": TRAFFIC_BYTES_C2,
            "kernel": "eh::gemm32_stats_kernel<2,false,false> (one head on 512 rows = 1/24 of the launch; the time "
                      "per head includes its share of the LayerNorm and final-merge launches)",
            "avg_launch_us": avg_s * 1e6,
            "flops_per_launch": flops_per_launch, "launches": launches}
    cfg = {"workload": "c2_calib: d=2048 V=50304 24 heads x 512 tokens bf16, all heads on all tokens"
                       + (", with max-probability and top-2 difference" if args.metrics else "")}
    res = {"value": evals / dt, "ms_per_step": dt / steps * 1e3, "step_ms": timed.step_ms, "roofline": roof, "config": cfg, "dtype": w.dtype,
           "cpu_baseline": None, "us_per_head": avg_s * 1e6}
    if cpu_leg:
        res["cpu_baseline"] = cpu_head_evals(args, G, heads, ((l, hid.h[l][:128]) for l in range(w.n_heads)),
                                             "the first 128 tokens of each head in turn")
    B.eh_destroy(ctx)
    return res


def run_c3(args, torch, B, G, dev, steps, warmup, cpu_leg, keep=None):
    # 64 decode rows through 32 heads; a row leaves at its first H < tau and the
    # survivors are compacted between heads.  Thresholds: the 10/40/70 % exit schedule,
    # set from this library's own entropies of every head on every row (a bench input,
    # not a parity reference).
    w = G.CONFIGS["c3_dynexit"]
    heads = G.make_heads(w, dev)
    esz = 2
    hid = G.make_hidden(w, heads, dev)
    R = w.rows
    ctx0 = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")] * w.n_heads, max_rows=R)
    Hall = torch.zeros((w.n_heads, R), device=dev)
    for l in range(w.n_heads):
        B.eh_eval(ctx0, l, hid.h[l], R, Hall[l], None, None)
    torch.cuda.synchronize()
    B.eh_destroy(ctx0)
    tau = G.tau_for_schedule(Hall.cpu().numpy(), w.n_heads)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=R)
    ex = torch.full((R,), -1, dtype=torch.int32, device=dev)
    tok = torch.full((R,), -1, dtype=torch.int32, device=dev)
    nev = torch.zeros(1, dtype=torch.int64, device=dev)

    def step():
        B.eh_cascade(ctx, hid.h, R, ex, tok, None, nev)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    nev.zero_()
    dt, ev_s = timed(torch, step, steps, 0)
    B.eh_check(ctx)
    evals = int(nev.item())
    exl = ex.cpu().numpy()
    heads_run = int(exl.max()) + 1                       # heads that still had a live row
    launches = steps * heads_run
    # dominant kernel: the projection of one head on the live rows; it streams the head's
    # weights once whatever the number of live rows (HBM-bound: <= 64 flop per byte)
    bytes_per_launch = w.d * w.V * esz + (evals / launches) * (w.d * esz + 12)
    avg_s = ev_s / launches
    roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": TRAFFIC_RATIO_C3 * bytes_per_launch,
            "kernel": "eh::gemm32_stats_kernel_rows<false> (one launch = a whole cascade; one head on the live rows = "
                      "cascade time / heads run)",
            "avg_launch_us": avg_s * 1e6, "bytes_per_launch": bytes_per_launch, "launches": launches}
    cfg = {"workload": "c3_dynexit: d=2560 V=50304 32 heads x 64 rows bf16, rows exit at first H<tau, "
                       "compaction between heads",
           "mean_evals_per_cascade": evals / steps,
           "exited_by_layer_8_16_24": [float((exl < l).mean()) for l in (8, 16, 24)]}
    res = {"value": evals / dt, "ms_per_step": dt / steps * 1e3, "step_ms": timed.step_ms, "roofline": roof, "config": cfg, "dtype": w.dtype,
           "cpu_baseline": None, "us_per_head": avg_s * 1e6}
    if cpu_leg:
        # head by head on the rows this run's cascade kept alive up to that head
        exd = ex.to(dev)
        res["cpu_baseline"] = cpu_head_evals(args, G, heads, ((l, hid.h[l][exd >= l]) for l in range(heads_run)),
                                             "each head in turn on the rows still alive at it")
    B.eh_destroy(ctx)
    if keep is not None:
        keep["heads"] = heads
    return res


def run_c4(args, torch, B, G, dev, steps, warmup, cpu_leg, heads=None):
    # 16 rows x (8 drafts + 1): argmax of the final head at 144 positions and the accepted
    # prefix per row.  Four copies of the final head are used in turn so that the 257.6 MB
    # weight stream comes from HBM, not from the last-level cache.
    w = G.CONFIGS["c4_verify"]
    esz = 2
    fin = w.n_heads - 1
    if heads is None:
        heads = G.make_heads(w, dev)
    Bsz, k = 16, 8
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    draft = torch.randint(0, w.V, (Bsz, k), generator=gen, device=dev)
    case = G.make_verify_case(w, heads, draft, dev)
    n_copies = 4
    ctxs = []
    for c in range(n_copies):
        Wc = heads.W[fin].clone()
        ctxs.append(B.eh_create([Wc], [heads.gamma[fin]], [heads.beta[fin]], [float("inf")],
                                max_rows=Bsz * (k + 1)))
        del Wc
    acc = torch.full((Bsz,), -1, dtype=torch.int32, device=dev)
    nxt = torch.full((Bsz,), -1, dtype=torch.int32, device=dev)
    d32 = draft.to(torch.int32).contiguous()
    calls_per_step = 8

    def step():
        for i in range(calls_per_step):
            B.dssd_verify(ctxs[i % n_copies], case.f_final, d32, None, acc, nxt, None)

    dt, ev_s = timed(torch, step, steps, warmup)
    launches = steps * calls_per_step
    evals = launches * Bsz * (k + 1)
    bytes_per_launch = w.d * w.V * esz + Bsz * (k + 1) * (w.d * esz + 4)
    avg_s = ev_s / launches
    roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": TRAFFIC_RATIO_C4 * bytes_per_launch,
            "kernel": "eh::gemm32_stats_kernel_rows<true> (one launch = one verification: LayerNorm, argmax-only "
                      "projection of 144 positions, prefix comparison; the time also holds the preset launch)",
            "avg_launch_us": avg_s * 1e6, "bytes_per_launch": bytes_per_launch, "launches": launches}
    cfg = {"workload": "c4_verify: d=2560 V=50304 final head, 16 rows x (8 drafts + 1) bf16, "
                       f"{calls_per_step} verifications per bench step over {n_copies} weight copies",
           "mean_accepted": float(acc.float().mean().item())}
    # the bookkeeping of Section 4.3.2 on this batch's outcome (outside the timed region)
    counters = torch.zeros(5, dtype=torch.int64, device=dev)
    B.dssd_tally(ctxs[0], None, acc, Bsz, k, None, counters)
    cnt = counters.tolist()
    cfg.update(drafted=cnt[1], accepted=cnt[2], wasted=cnt[3], acceptance_rate=cnt[2] / max(cnt[1], 1))
    res = {"value": evals / dt, "ms_per_step": dt / steps * 1e3, "step_ms": timed.step_ms, "roofline": roof, "config": cfg, "dtype": w.dtype,
           "cpu_baseline": None, "us_per_head": avg_s * 1e6}
    if cpu_leg:
        from oracle import eh_oracle as O
        f64 = G.to_f64_numpy
        W64, g64, b64 = f64(heads.W[fin]), f64(heads.gamma[fin]), f64(heads.beta[fin])
        done, spent = 0, 0.0
        for b0 in range(0, Bsz, 2):
            f2, d2 = f64(case.f_final[b0:b0 + 2]), draft[b0:b0 + 2].cpu().numpy()
            c0 = time.perf_counter()
            O.dssd_verify(f2, d2, g64, b64, W64, None, 1e-5, True)
            spent += time.perf_counter() - c0
            done += 2 * (k + 1)
            if spent > args.cpu_seconds:
                break
        res["cpu_baseline"] = {"value": done / spent, "unit": "evals/s", "cores": oracle_threads(), "kind": "oracle",
                               "sample": f"{done // (k + 1)} of the {Bsz} rows, two at a time ({done} evaluations, "
                                         f"{spent:.1f} s; fp64 numpy, weights pre-widened)"}
    for c in ctxs:
        B.eh_destroy(c)
    return res


def run_ceiling(args, torch, B, G, dev):
    """--workload read_ceiling / mfma_ceiling: the practical ceilings alone, as their own line."""
    t_setup = time.time()
    if args.workload == "read_ceiling":
        out = {}
        for name in ("c1_decode", "c3_dynexit"):
            w = G.CONFIGS[name]
            heads = G.make_heads(w, dev)
            ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")] * w.n_heads, max_rows=16)
            del heads
            out[name] = read_ceiling(torch, B, ctx, w, dev, reps=max(1, args.steps))
            B.eh_destroy(ctx)
            torch.cuda.empty_cache()
        best = out["c1_decode"]["registers_one_launch"]
        line = {"metric": "weight_read_GBps", "value": best, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                "warmup": 1, "ms_per_step": out["c1_decode"]["bytes_per_sweep"] / best / 1e6, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
                "config": {"workload": "read_ceiling: a plain read of every head's re-tiled weights (2.47 GB for the decode "
                                       "workload, 8.24 GB for the 64-row one), four variants each", "variants": out},
                "roofline": {"bound": "hbm", "achieved": best, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": best / HBM_PEAK_GBS, "traffic": None, "kernel": "eh probe_read_reg_kernel, one launch"},
                "cpu_baseline": None, "setup_s": round(time.time() - t_setup, 1)}
    else:
        w = G.Workload("probe", d=64, V=64, n_heads=1, rows=4, dtype="bf16", seed=1)
        heads = G.make_heads(w, dev)
        ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=4)
        sink = torch.zeros(1024 * 256, device=dev)
        out = {}
        for name, iters, rnd in (("zeros_4000", 4000, False), ("random_4000", 4000, True), ("random_130", 130, True)):
            flops = B.eh_probe_mfma(ctx, iters, rnd, sink)
            torch.cuda.synchronize()
            reps = max(3, args.steps)
            ms = event_ms(lambda: [B.eh_probe_mfma(ctx, iters, rnd, sink) for _ in range(reps)], torch)
            out[name] = flops * reps / (ms * 1e-3) / 1e12
            if name == "random_4000":
                ms_step = ms / reps
        B.eh_destroy(ctx)
        best = out["random_4000"]
        line = {"metric": "mfma_bf16_TFLOPs", "value": best, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
                "warmup": 1, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "mfma_ceiling: the batched kernel's 28 matrix instructions per k-step from registers "
                                       "only, one workgroup of 4 waves per compute unit; iterations and operands vary",
                           "variants_TFLOPs": out},
                "roofline": {"bound": "mfma", "achieved": best, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": best / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": "eh probe_mfma_kernel"},
                "cpu_baseline": None, "setup_s": round(time.time() - t_setup, 1)}
    print(json.dumps(line), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build is single-GPU by construction; --gpus {args.gpus} is not "
              "supported (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2407_21082_amd import binding as B     # raises if libeh.so is missing
    from workloads import generators as G

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(7)
        dst = torch.empty(n, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        for _ in range(10):
            torch.add(src, 1, out=dst)      # an elementwise kernel: reads n bytes, writes n bytes
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"kernel": "torch.add(uint8, 1) elementwise",
                                               "bytes_read": n, "bytes_written": n, "copies": 10}}))
        return
    if args.workload == "f1_calibrate":
        return bench_calibrate(args, torch, B, G, dev)
    if args.workload == "f3_draft":
        return bench_draft(args, torch, B, G, dev)
    if args.workload == "f4_losses":
        return bench_losses(args, torch, B, G, dev)
    if args.workload in ("read_ceiling", "mfma_ceiling"):
        return run_ceiling(args, torch, B, G, dev)
    t_setup = time.time()
    cpu_leg = not args.no_cpu_baseline
    extra = {}
    if args.workload is None:
        # the headline line (decode) plus the batched configurations, all timed in this run
        res = run_c1(args, torch, B, G, dev, args.steps, args.warmup, cpu_leg, ceiling=True)
        extra["read_ceiling"] = res.pop("read_ceiling")
        torch.cuda.empty_cache()
        bs, bw = args.batched_steps, args.batched_warmup
        batched = {}

        def brief(r):
            return {"value": r["value"], "unit": "evals/s", "us_per_head": r["us_per_head"], "steps": bs, "warmup": bw,
                    "step_ms": r.get("step_ms"), "workload": r["config"]["workload"], "roofline": r["roofline"]}

        batched["c2_calib"] = brief(run_c2(args, torch, B, G, dev, bs, bw, False))
        torch.cuda.empty_cache()
        keep = {}
        batched["c3_dynexit"] = brief(run_c3(args, torch, B, G, dev, bs, bw, False, keep))
        batched["c4_verify"] = brief(run_c4(args, torch, B, G, dev, bs, bw, False, keep.get("heads")))
        extra["batched"] = batched
    elif args.workload == "c1_decode":
        res = run_c1(args, torch, B, G, dev, args.steps, args.warmup, cpu_leg, ceiling=False)
    elif args.workload == "c2_calib":
        res = run_c2(args, torch, B, G, dev, args.steps, args.warmup, cpu_leg)
    elif args.workload == "c3_dynexit":
        res = run_c3(args, torch, B, G, dev, args.steps, args.warmup, cpu_leg)
    elif args.workload == "c4_verify":
        res = run_c4(args, torch, B, G, dev, args.steps, args.warmup, cpu_leg)
    else:
        raise SystemExit("unknown workload: " + str(args.workload))

    line = {"metric": "exit_head_evals_per_sec", "value": res["value"], "unit": "evals/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
            "step_ms": res.get("step_ms"),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": res["dtype"],
            "data": "synthetic", "config": res["config"], "roofline": res["roofline"], "cpu_baseline": res["cpu_baseline"]}
    line.update(extra)
    line["setup_s"] = round(time.time() - t_setup, 1)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
