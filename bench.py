#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A *step* is one pass of every stage over one batch of synthetic gradients:
all W simulated workers accumulate all layers, the leader of each layer scores,
selects and compacts its pairs (compress_segmented), every worker's residual is
gathered at the index set and summed (gather_sum_at_indices), and the weights are
updated and the sent residuals cleared (apply_sparse_update).  The default route
runs the step through iwp_step_segmented, which produces the same bytes as the
three separate calls with the exchange folded into the streaming pass.  Inputs
are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload alexnet|resnet50|many_small|tiny|flat]

Prints ONE JSON line: metric / value / unit, ms_per_step, the roofline of the
dominant kernel, stand-alone part timings and the oracle timed on the host
(cpu_baseline).  The default workload is the
AlexNet-shaped set the headline metric is quoted on.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published peak HBM3E bandwidth
WORKLOADS = {"tiny": 1, "alexnet": 2, "resnet50": 3, "many_small": 4, "flat": 5}
DOMINANT_KERNEL = {"whole_step": "k_follow_gather", "three_calls": "k_accumulate_rest", "threshold": "k_follow_mask",
                   "layerwise": "k_follow_mask"}


def step_bytes(ps, W_acc, W_list):
    """Algorithmic bytes of one step: W_acc workers accumulate (12 B/elem), the
    leader also reads w (4 B/elem), 8 B per pair out, and the exchange floor
    (12 + 8 W) B per pair (index, W gathers, weight read-modify-write, W clears)."""
    return (12 * W_acc + 4) * ps.P + (8 + 12 + 8 * W_list) * ps.K


def dominant_kernel_bytes(ps, W_acc, W_list, route):
    """Algorithmic bytes one launch of the dominant streaming kernel moves.
    three_calls: the W_acc - 1 non-leading workers accumulate (12 B/elem).
    whole_step: the W_acc - 1 non-leading workers accumulate (12 B/elem) and all
    W_list - 1 non-leaders hand over their value at the K pairs and clear it:
    index read (4 B) once per worker tile is counted once, + 4 B gathered out per worker."""
    if W_acc == 1:                                    # k_leader_pass: r, g, w in, r out
        return 16 * ps.P
    if route == "three_calls":
        return 12 * (W_acc - 1) * ps.P
    return 12 * (W_acc - 1) * ps.P + (4 + 4 * (W_list - 1)) * ps.K


def layerwise_extra_bytes(ps, n_lead):
    """Layer-wise thresholds: the statistics need the chosen nodes' importance before the
    threshold exists, so the mask pass reads their residual and the weights again (8 B/elem)."""
    return 8 * n_lead * ps.P


def threshold_step_bytes(ps, W_acc, W_list, n_lead, pairs):
    """Threshold mode: W_acc workers accumulate (12 B/elem), each chosen node also reads
    w (4 B/elem), the encoded mask goes out once (1 bit/elem), and per sent pair the
    same exchange floor as above (index out and in, sum out, weight read-modify-write,
    W gathers and clears)."""
    return (12 * W_acc + 4 * n_lead) * ps.P + ps.P / 8 + (8 + 12 + 8 * W_list) * pairs


def threshold_dominant_bytes(ps, W_acc, W_list, n_lead, pairs):
    """k_follow_mask: the W_acc - n_lead workers that are not chosen accumulate
    (12 B/elem), read the mask once (1 bit/elem) and hand over 4 B per pair each."""
    return 12 * (W_acc - n_lead) * ps.P + ps.P / 8 + 4 * (W_acc - n_lead) * pairs


def traffic_from_profiles(workload, kernel):
    """HBM bytes per launch of the dominant kernel from the committed counter runs
    (profiles/traffic.json), or None if no such measurement exists."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="alexnet", choices=sorted(WORKLOADS))
    ap.add_argument("--route", default="whole_step", choices=["whole_step", "three_calls", "threshold", "layerwise"],
                    help="whole_step: iwp_step_segmented; three_calls: compress_segmented + gather_sum_at_indices "
                         "+ apply_sparse_update (same results); threshold: iwp_step_threshold_segmented with fixed "
                         "per-layer thresholds (calibrated by a few top-k steps to the same keep ratio); layerwise: "
                         "iwp_step_layerwise_segmented, thresholds from each layer's importance mean / variance")
    ap.add_argument("--n-lead", type=int, default=1, help="threshold route: chosen nodes per layer")
    ap.add_argument("--random-selection", action="store_true",
                    help="threshold route: also send sub-threshold elements with probability importance / threshold")
    ap.add_argument("--no-hint", action="store_true",
                    help="top-k routes: do not pass the previous step's thresholds as a hint (results are "
                         "identical either way; the hint saves the second pass over the leaders' layers)")
    ap.add_argument("--no-parts", action="store_true", help="skip the stand-alone compress / exchange timings")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--scale-down", type=int, default=1, help="shrink the many_small / flat workloads (debug)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU; --gpus N with N > 1 is not supported "
              "(the path would shard by worker: one GPU per data-parallel worker)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1901_01544_amd import iwp, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    iwp.load()
    dev = torch.device("cuda:0")
    cfg = WORKLOADS[args.workload]
    ps = wl.make_config(cfg, scale_down=args.scale_down)
    flat_cfg = cfg == 5
    W_list = ps.W + 1 if flat_cfg else ps.W            # config 5: local worker + 8 static peers
    W_acc = 1 if flat_cfg else ps.W
    pool = 2 if flat_cfg else ps.W

    t0 = time.time()
    if flat_cfg:
        # 1e9-element buffers are drawn on the device (seeded); same laws as the host generator
        w = wl.gen_weights_device(ps, dev)
        grads = [wl.gen_laplace_device(ps, 1 + s, dev) for s in range(pool)]
        r = [torch.zeros(ps.flat, device=dev)] + [wl.gen_laplace_device(ps, 100 + p, dev) for p in range(8)]
        w_np = grads_np = None
    else:
        w_np = wl.gen_weights(ps)
        grads_np = [wl.gen_gradient(ps, s) for s in range(pool)]
        w = torch.from_numpy(w_np).to(dev)
        grads = [torch.from_numpy(g).to(dev) for g in grads_np]
        r = [torch.zeros(ps.flat, device=dev) for _ in range(ps.W)]
    gen_s = time.time() - t0

    plan = iwp.Plan(ps.rows())
    fused = args.route in ("whole_step", "threshold", "layerwise")   # threshold routes: top-k steps calibrate
    thr_mode = args.route in ("threshold", "layerwise")
    lw_mode = args.route == "layerwise"
    assert not (thr_mode and flat_cfg), "the threshold route is measured on the multi-worker workloads"
    n_lead = args.n_lead
    dominant = DOMINANT_KERNEL[args.route]
    if flat_cfg and args.route in ("whole_step", "three_calls"):
        dominant = "k_leader_pass"                    # one accumulating worker: nothing follows, the leader's look dominates
    ws_bytes = plan.step_workspace_bytes(W_list) if fused else plan.workspace_bytes
    ws = torch.empty(max(1, ws_bytes), dtype=torch.uint8, device=dev)
    idx = torch.empty(ps.K, dtype=torch.int32, device=dev)
    val = torch.empty(ps.K, dtype=torch.float32, device=dev)
    sm = torch.empty(ps.K, dtype=torch.float32, device=dev)
    thr2 = [torch.zeros(3 * len(ps.layers), dtype=torch.int32, device=dev) for _ in range(2)]   # ping-pong: the
    thr = thr2[0]                                     # records of step t-1 are the hint of step t
    use_hint = not thr_mode and not args.no_hint
    CAL = 8                                           # threshold route: top-k steps that settle the thresholds
    total = args.warmup + args.steps + (CAL if thr_mode else 0)
    spare = 1                                         # the layerwise route spends one more step on calibration
    if flat_cfg:
        lead_np = np.zeros((total, 1), np.int32)
    else:
        lead_np = np.stack([wl.leaders(ps, t).astype(np.int32) for t in range(total)])
    leaders = torch.from_numpy(lead_np).to(dev)
    eps, scale = float(ps.eps), float(ps.scale)
    stream = torch.cuda.current_stream()

    def step(t):
        if flat_cfg:
            g = [grads[t % pool]] + [None] * 8
        else:
            g = [grads[wl.gradient_set_of(ps, p, t, pool)] for p in range(ps.W)]
        if fused:
            hint = thr2[(t + 1) % 2] if (use_hint and t > 0) else None
            iwp.step_segmented(plan, w, g, r, leaders[t], eps, scale, idx, val, sm, thr2[t % 2], ws, stream,
                               thr_hint=hint)
        else:
            hint = thr2[(t + 1) % 2] if (use_hint and t > 0) else None
            iwp.compress_segmented(plan, w, g, r, leaders[t], eps, idx, val, thr2[t % 2], ws, stream, thr_hint=hint)
            iwp.gather_sum_at_indices(r, idx, ps.K, sm, stream)
            iwp.apply_sparse_update(w, idx, sm, ps.K, scale, r, stream)

    # plain-copy ceiling of this machine (read 1 : write 1), quoted beside the result
    a = torch.empty(1 << 28, device=dev)
    b = torch.empty(1 << 28, device=dev)
    for _ in range(3):
        iwp.copy_f32(b, a, stream)
    iwp.timing_enable("k_copy", 16)
    for _ in range(10):
        iwp.copy_f32(b, a, stream)
    torch.cuda.synchronize()
    ms, cnt = iwp.timing_collect()
    copy_gbps = 2 * 4 * a.numel() * cnt / (ms * 1e-3) / 1e9
    del a, b

    first = 0
    pairs_per_step = ps.K
    if thr_mode:
        # fixed thresholds: the k-th largest importance of each layer after CAL top-k steps,
        # so the mask keeps about the same share of every layer as the top-k route
        for t in range(CAL):
            step(t)
        torch.cuda.synchronize()
        first = CAL
        fixed_thr = thr2[(CAL - 1) % 2].view(-1, 3)[:, 0].contiguous().view(torch.float32).clone()
        max_pairs = min(ps.P, (16 if args.random_selection else 8) * ps.K)
        del ws
        ws = torch.empty(plan.threshold_workspace_bytes(W_list, n_lead, max_pairs), dtype=torch.uint8, device=dev)
        mask = torch.empty(plan.mask_bytes, dtype=torch.uint8, device=dev)
        counts = torch.zeros(total + spare, len(ps.layers) + 2, dtype=torch.int32, device=dev)
        idx = torch.empty(max_pairs, dtype=torch.int32, device=dev)
        sm = torch.empty(max_pairs, dtype=torch.float32, device=dev)
        chosen = torch.from_numpy(np.stack([wl.chosen_nodes(ps, t, n_lead).astype(np.int32).ravel()
                                            for t in range(total + spare)])).to(dev)

        stats = torch.zeros(len(ps.layers), n_lead, 2, dtype=torch.float64, device=dev)
        thr_slots = torch.zeros(len(ps.layers), n_lead, dtype=torch.float32, device=dev)
        rule = None
        if lw_mode:
            # one rule for all layers: alpha = the median calibrated threshold; one step with beta = 0
            # gives the layers' var/mean ratios; C = their median, beta = a 10 % correction at C
            alpha = float(fixed_thr.median())
            g0 = [grads[wl.gradient_set_of(ps, p, CAL, pool)] for p in range(ps.W)]
            iwp.step_layerwise_segmented(plan, w, g0, r, chosen[CAL], n_lead, alpha, 0.0, 0.0, eps, scale, stats,
                                         thr_slots, mask, counts[CAL], idx, sm, max_pairs, ws, stream)
            torch.cuda.synchronize()
            ratio = (stats[:, :, 1] / stats[:, :, 0]).flatten()
            c_rule = float(ratio[torch.isfinite(ratio)].median())
            rule = (alpha, 0.1 * alpha / c_rule, c_rule)
            first = CAL + 1
            total += 1

        def step(t):                                  # noqa: F811 -- the timed step of this route
            g = [grads[wl.gradient_set_of(ps, p, t, pool)] for p in range(ps.W)]
            if lw_mode:
                iwp.step_layerwise_segmented(plan, w, g, r, chosen[t], n_lead, rule[0], rule[1], rule[2], eps, scale,
                                             stats, thr_slots, mask, counts[t], idx, sm, max_pairs, ws, stream)
            elif args.random_selection:
                iwp.step_threshold_random_segmented(plan, w, g, r, chosen[t], n_lead, fixed_thr, ps.seed, t, eps, scale,
                                                    mask, counts[t], idx, sm, max_pairs, ws, stream)
            else:
                iwp.step_threshold_segmented(plan, w, g, r, chosen[t], n_lead, fixed_thr, eps, scale, mask, counts[t],
                                             idx, sm, max_pairs, ws, stream)

    for t in range(first, first + args.warmup):
        step(t)
    torch.cuda.synchronize()
    iwp.timing_enable(dominant, args.steps)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # per-step times, same stream
    t0 = time.perf_counter()
    for q, t in enumerate(range(first + args.warmup, total)):
        marks[q].record(stream)
        step(t)
    marks[args.steps].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms = sorted(marks[q].elapsed_time(marks[q + 1]) for q in range(args.steps))
    k_ms, k_cnt = iwp.timing_collect()
    if thr_mode:
        c = counts[first + args.warmup:total].cpu().numpy()
        assert not c[:, -1].any(), "pair capacity exceeded in %d timed steps" % int(c[:, -1].sum())
        pairs_per_step = float(c[:, -2].mean())
        pairs_minmax = [int(c[:, -2].min()), int(c[:, -2].max())]

    # the parts on their own, after the timed region (they change r and w further, which no longer matters):
    # (i) compression of one worker (accumulate + score + select + compact, every layer leads itself),
    # (ii) the exchange as the two separate calls over the K pairs the last step produced
    parts = {}
    if not args.no_parts and not thr_mode:
        ws1 = torch.empty(max(1, plan.workspace_bytes), dtype=torch.uint8, device=dev)
        reps = 5
        def timed(fn):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / reps
        tc = timed(lambda: iwp.compress_segmented(plan, w, [grads[0]], [r[0]], None, eps, idx, val, thr2[0], ws1, stream))
        flip = [0]
        def hinted():                                      # hint: the records the previous call wrote
            flip[0] ^= 1
            iwp.compress_segmented(plan, w, [grads[0]], [r[0]], None, eps, idx, val, thr2[flip[0]], ws1, stream,
                                   thr_hint=thr2[flip[0] ^ 1])
        th = timed(hinted)
        tg = timed(lambda: iwp.gather_sum_at_indices(r, idx, ps.K, sm, stream))
        tu = timed(lambda: iwp.apply_sparse_update(w, idx, sm, ps.K, scale, r, stream))
        cb = 16 * ps.P + 8 * ps.K
        xb = (12 + 8 * W_list + 8) * ps.K
        parts = {
            "compress_one_worker": {"ms": tc * 1e3, "params_per_s": ps.P / tc, "algorithmic_GBps": cb / tc / 1e9,
                                    "frac_of_hbm_peak": cb / tc / 1e9 / HBM_PEAK_GBPS},
            "compress_one_worker_hinted": {"ms": th * 1e3, "params_per_s": ps.P / th,
                                           "algorithmic_GBps": cb / th / 1e9,
                                           "frac_of_hbm_peak": cb / th / 1e9 / HBM_PEAK_GBPS},
            "exchange_two_calls": {"ms": (tg + tu) * 1e3, "pairs_per_s": ps.K / (tg + tu),
                                   "algorithmic_GBps": xb / (tg + tu) / 1e9, "gather_ms": tg * 1e3, "update_ms": tu * 1e3},
        }
        del ws1

    ms_per_step = elapsed * 1e3 / args.steps
    params_per_s = ps.P * args.steps / elapsed
    if thr_mode:
        algo_bytes = threshold_step_bytes(ps, W_acc, W_list, n_lead, pairs_per_step)
        if lw_mode:
            algo_bytes += layerwise_extra_bytes(ps, n_lead)
        dom_bytes = threshold_dominant_bytes(ps, W_acc, W_list, n_lead, pairs_per_step)
    else:
        algo_bytes = step_bytes(ps, W_acc, W_list)
        dom_bytes = dominant_kernel_bytes(ps, W_acc, W_list, args.route)
    dom_ms = k_ms / max(1, k_cnt)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # HBM bytes the counters saw for one whole (hinted) step of this route, if such a run is on file
    step_traffic = traffic_from_profiles(args.workload, "step:" + args.route) if use_hint or thr_mode else None
    out = {
        "metric": "params/sec and achieved HBM GB/s (% of peak) for compress+exchange step",
        "value": params_per_s,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": ps.name, "config_id": cfg, "tensors": len(ps.layers), "params": ps.P,
                   "pairs_per_step": pairs_per_step, "workers_accumulating": W_acc, "residual_list": W_list,
                   "keep": "1/64" if cfg in (1, 2) else ("1/58.8" if cfg == 3 else ("U(0.5%,5%)" if cfg == 4 else "0.1%")),
                   "eps": eps, "gradient_pool": pool, "route": args.route,
                   "threshold_hint": "previous step" if use_hint else "none"},
        "worker_params_per_s": ps.P * W_acc * args.steps / elapsed,
        "ms_per_step_median": step_ms[len(step_ms) // 2],
        "ms_per_step_min": step_ms[0],
        "step_algorithmic_bytes": algo_bytes,
        "step_algorithmic_GBps": algo_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_traffic_bytes": step_traffic,
        "step_traffic_GBps": None if step_traffic is None else step_traffic / (ms_per_step * 1e-3) / 1e9,
        "copy_kernel_GBps": copy_gbps,
        "parts": parts,
        "input_generation_s": gen_s,
        "roofline": {
            "bound": "hbm",
            "kernel": dominant,
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": traffic_from_profiles(args.workload, dominant),
            "algorithmic_bytes_per_launch": dom_bytes,
            "avg_launch_ms": dom_ms,
            "launches_timed": k_cnt,
            "share_of_step_time": dom_ms / ms_per_step,
        },
    }

    if thr_mode:
        out["config"]["threshold_hint"] = "n/a"
        out["config"]["chosen_nodes_per_layer"] = n_lead
        out["config"]["random_selection"] = bool(args.random_selection)
        out["config"]["thresholds"] = "fixed per layer: k-th largest importance after %d top-k steps" % CAL
        if lw_mode:
            out["config"]["thresholds"] = "alpha +/- beta * var/mean per layer and chosen node"
            out["config"]["rule"] = {"alpha": rule[0], "beta": rule[1], "C": rule[2]}
        out["config"]["pairs_per_step_min_max"] = pairs_minmax
        out["config"]["pair_capacity"] = max_pairs
    if not args.no_cpu_baseline and thr_mode:
        import oracle
        # the oracle's threshold-mode step from the state the GPU run ended in
        w_ref = w.cpu().numpy()
        r_ref = [x.cpu().numpy() for x in r]
        thr_np = fixed_thr.cpu().numpy()
        n_steps, spent = 0, 0.0
        while n_steps < 1 or (spent < 10.0 and n_steps < args.steps):
            t = total + n_steps
            g = [grads_np[wl.gradient_set_of(ps, p, t, pool)] for p in range(ps.W)]
            t1 = time.perf_counter()
            if lw_mode:
                oracle.step_layerwise(w_ref, g, r_ref, ps.rows(), wl.chosen_nodes(ps, t, n_lead), rule[0], rule[1],
                                      rule[2], eps, scale, ps.P)
            else:
                oracle.step_threshold(w_ref, g, r_ref, ps.rows(), wl.chosen_nodes(ps, t, n_lead), thr_np, eps, scale,
                                      ps.P, random=(ps.seed, t) if args.random_selection else None)
            spent += time.perf_counter() - t1
            n_steps += 1
        out["cpu_baseline"] = {
            "value": ps.P * n_steps / spent, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": "%d whole threshold-mode step(s) of the same workload (all %d workers, all %d tensors), %.1f s"
                      % (n_steps, ps.W, len(ps.layers), spent),
            "host_cpus": os.cpu_count(),
        }
    elif not args.no_cpu_baseline and not flat_cfg:
        import oracle
        # the oracle as it stands, one host core, on a bounded sample: whole steps of the
        # same workload until ~10 s of CPU work have been spent (at least one step)
        w_ref = w_np.copy()
        r_ref = [np.zeros(ps.flat, np.float32) for _ in range(ps.W)]
        n_steps, spent = 0, 0.0
        while n_steps < 1 or (spent < 10.0 and n_steps < args.steps):
            g = [grads_np[wl.gradient_set_of(ps, p, n_steps, pool)] for p in range(ps.W)]
            lead = wl.leaders(ps, n_steps)
            t1 = time.perf_counter()
            oracle.step(w_ref, g, r_ref, ps.rows(), lead, eps, scale)
            spent += time.perf_counter() - t1
            n_steps += 1
        out["cpu_baseline"] = {
            "value": ps.P * n_steps / spent,
            "unit": "params/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "%d whole step(s) of the same workload (all %d workers, all %d tensors), %.1f s"
                      % (n_steps, ps.W, len(ps.layers), spent),
            "host_cpus": os.cpu_count(),
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
