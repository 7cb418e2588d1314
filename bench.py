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

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline|alexnet|resnet50|many_small|tiny|flat]

Prints ONE JSON line.  The headline fields (metric / value / ms_per_step / roofline /
cpu_baseline) are the AlexNet-shaped set, whole-step route, hinted with the previous
step's thresholds.  With the default workload ("headline") the same line carries, under
"also", the same measurement without hints and the ResNet-50-shaped set with and without
hints, each with its own roofline and (per workload) cpu_baseline: the target names both
sets.  All of these are taken in the steady state of the residuals (--preroll un-timed steps
first; hinted and unhinted run the same steps from the same saved state); the cold start
(first steps from zero residuals, where the selection has less to do) is listed beside them.  Timing: the K timed steps run back to back with nothing else on the stream; the
dominant kernel's launch durations and the per-step spread come from a second loop of K
steps, after the first.
"""
from __future__ import annotations

import argparse
import hashlib
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
METRIC = "params/sec and achieved HBM GB/s (% of peak) for compress+exchange step"
# Table 1 of the paper, quoted as context (other hardware, another quantity: not a target of this bench)
PAPER_CONTEXT = {
    "table1_gradient_compression_ratio": {"AlexNet": 64.0, "ResNet-50": 58.8},
    "setting": "ImageNet training on a ring of GTX 1080 Ti nodes without InfiniBand (ResNet-50: 96 nodes, one GPU "
               "each), fixed importance thresholds; the paper reports no timing or bandwidth of the compression step",
    "use_here": "taken as the keep fractions 1/64 and 1/58.8 of the synthetic sets (sum n / sum k = 63.99997 and 58.7876)",
}


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


def kernel_source_hash():
    """sha256 over the kernel sources (file names and contents, sorted): what a counter run was taken on."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1901_01544_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def traffic_from_profiles(workload, kernel, check_hash=True):
    """HBM bytes per launch of a kernel (or "step:<route>": all kernels of one hinted step) from the
    committed counter runs (profiles/traffic.json).  None if there is no such measurement, or if the
    file was taken on other kernel sources than the ones in this tree (its "_csrc_sha256" stamp)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            d = json.load(f)
    except (OSError, ValueError):
        return None
    if check_hash and d.get("_csrc_sha256") != kernel_source_hash():
        return None
    return d.get(workload, {}).get(kernel)


def copy_ceiling(iwp, torch, dev, stream):
    """Plain-copy rate of this machine (read 1 : write 1), quoted beside the results."""
    a = torch.empty(1 << 28, device=dev)
    b = torch.empty(1 << 28, device=dev)
    for _ in range(3):
        iwp.copy_f32(b, a, stream)
    iwp.timing_enable("k_copy", 16)
    for _ in range(10):
        iwp.copy_f32(b, a, stream)
    torch.cuda.synchronize()
    ms, cnt = iwp.timing_collect()
    return 2 * 4 * a.numel() * cnt / (ms * 1e-3) / 1e9


def timed_steps(torch, stream, step, first, steps):
    """`steps` consecutive steps, nothing else on the stream: (ms per step by the host clock between two
    synchronisations, the same by one event pair around the whole loop)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for t in range(first, first + steps):
        step(t)
    e1.record(stream)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def profiled_steps(iwp, torch, stream, step, first, steps, kernel):
    """A second loop: every launch of `kernel` timed with HIP events on its stream, and an event
    between steps for the spread.  -> (kernel ms per launch, launches, sorted per-step ms)."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    iwp.timing_enable(kernel, steps)
    for q, t in enumerate(range(first, first + steps)):
        marks[q].record(stream)
        step(t)
    marks[steps].record(stream)
    torch.cuda.synchronize()
    k_ms, k_cnt = iwp.timing_collect()
    return k_ms / max(1, k_cnt), k_cnt, sorted(marks[q].elapsed_time(marks[q + 1]) for q in range(steps))


def keep_label(cfg):
    return "1/64" if cfg in (1, 2) else ("1/58.8" if cfg == 3 else ("U(0.5%,5%)" if cfg == 4 else "0.1%"))


def oracle_baseline(ps, w_np, grads_np, pool, wl, max_steps, flat_note=None, W_list=None):
    """The oracle as it stands, one host core, on a bounded sample: whole steps of the workload until
    ~10 s of CPU work have been spent (at least one step)."""
    import numpy as np
    import oracle
    flat = flat_note is not None
    W = W_list if flat else ps.W
    w_ref = w_np.copy()
    if flat:
        r_ref = [np.zeros(ps.flat, np.float32)] + [wl.gen_gradient(ps, 100 + p) for p in range(W - 1)]
    else:
        r_ref = [np.zeros(ps.flat, np.float32) for _ in range(W)]
    n_steps, spent = 0, 0.0
    while n_steps < 1 or (spent < 10.0 and n_steps < max_steps):
        if flat:
            g = [grads_np[n_steps % pool]] + [grads_np[0]] * (W - 1)
            acc = [True] + [False] * (W - 1)
            lead = np.zeros(1, np.uint32)
        else:
            g = [grads_np[wl.gradient_set_of(ps, p, n_steps, pool)] for p in range(W)]
            acc = None
            lead = wl.leaders(ps, n_steps)
        t1 = time.perf_counter()
        oracle.step(w_ref, g, r_ref, ps.rows(), lead, float(ps.eps), float(ps.scale), accumulate_mask=acc)
        spent += time.perf_counter() - t1
        n_steps += 1
    sample = "%d whole step(s) of the same workload (all %d workers, all %d tensors), %.1f s" \
        % (n_steps, W, len(ps.layers), spent)
    if flat:
        sample = "%d whole step(s) of %s, %.1f s" % (n_steps, flat_note, spent)
    return {"value": ps.P * n_steps / spent, "unit": "params/s", "cores": 1, "kind": "oracle", "sample": sample,
            "host_cpus": os.cpu_count()}


def result_block(ps, cfg, route, hinted, W_acc, W_list, pool, steps, warmup, ms_host, ms_events, dom, dom_ms, dom_cnt,
                 step_ms_sorted, algo_bytes, dom_bytes, workload_key, pairs_per_step):
    ms = ms_host
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    step_traffic = traffic_from_profiles(workload_key, "step:" + route) if hinted else None
    traffic = traffic_from_profiles(workload_key, dom)
    return {
        "metric": METRIC,
        "value": ps.P / (ms * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": ps.name, "config_id": cfg, "tensors": len(ps.layers), "params": ps.P,
                   "pairs_per_step": pairs_per_step, "workers_accumulating": W_acc, "residual_list": W_list,
                   "keep": keep_label(cfg), "eps": float(ps.eps), "gradient_pool": pool, "route": route,
                   "threshold_hint": "previous step" if hinted else "none"},
        "worker_params_per_s": ps.P * W_acc / (ms * 1e-3),
        "ms_per_step_events": ms_events,
        "ms_per_step_median_second_loop": step_ms_sorted[len(step_ms_sorted) // 2],
        "ms_per_step_min_second_loop": step_ms_sorted[0],
        "step_algorithmic_bytes": algo_bytes,
        "step_algorithmic_GBps": algo_bytes / (ms * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": algo_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_traffic_bytes": step_traffic,
        "step_traffic_GBps": None if step_traffic is None else step_traffic / (ms * 1e-3) / 1e9,
        "roofline": {
            "bound": "hbm",
            "kernel": dom,
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": traffic,
            "traffic_source": ("profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on these kernel sources"
                               if traffic is not None else
                               "none on file for these kernel sources (profiles/traffic.json is stamped with a hash of csrc/)"),
            "algorithmic_bytes_per_launch": dom_bytes,
            "avg_launch_ms": dom_ms,
            "launches_timed": dom_cnt,
            "timed_in": "a second loop of %d steps after the timed one" % steps,
            "share_of_step_time": dom_ms / ms,
        },
    }


def bench_topk(iwp, wl, torch, np, args, workload, hint_modes, want_parts, want_cpu):
    """The top-k routes on one workload.  hint_modes: e.g. [True, False] -- measured one after the other
    on the same resident state.  -> list of result blocks, the first carrying parts and cpu_baseline."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    cfg = WORKLOADS[workload]
    ps = wl.make_config(cfg, scale_down=args.scale_down)
    flat_cfg = cfg == 5
    W_list = ps.W + 1 if flat_cfg else ps.W            # config 5: local worker + 8 static peers
    W_acc = 1 if flat_cfg else ps.W
    pool = 2 if flat_cfg else ps.W
    route = args.route
    fused = route == "whole_step"

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
    dominant = "k_leader_pass" if flat_cfg else DOMINANT_KERNEL[route]   # one accumulating worker: nothing follows
    ws_bytes = plan.step_workspace_bytes(W_list) if fused else plan.workspace_bytes
    ws = torch.empty(max(1, ws_bytes), dtype=torch.uint8, device=dev)
    idx = torch.empty(ps.K, dtype=torch.int32, device=dev)
    val = torch.empty(ps.K, dtype=torch.float32, device=dev)
    sm = torch.empty(ps.K, dtype=torch.float32, device=dev)
    thr2 = [torch.zeros(3 * len(ps.layers), dtype=torch.int32, device=dev) for _ in range(2)]   # ping-pong: the
    per_mode = args.warmup + 2 * args.steps           # records of step t-1 are the hint of step t
    total = args.preroll + per_mode
    if flat_cfg:
        lead_np = np.zeros((total, 1), np.int32)
    else:
        lead_np = np.stack([wl.leaders(ps, t).astype(np.int32) for t in range(total)])
    leaders = torch.from_numpy(lead_np).to(dev)
    eps, scale = float(ps.eps), float(ps.scale)
    use_hint = [False]

    def step(t):
        if flat_cfg:
            g = [grads[t % pool]] + [None] * 8
        else:
            g = [grads[wl.gradient_set_of(ps, p, t, pool)] for p in range(ps.W)]
        hint = thr2[(t + 1) % 2] if (use_hint[0] and t > 0) else None
        lead_t = None if flat_cfg else leaders[t]      # no leader table: the local worker (0) leads its one layer
        if fused:
            iwp.step_segmented(plan, w, g, r, lead_t, eps, scale, idx, val, sm, thr2[t % 2], ws, stream,
                               thr_hint=hint)
        else:
            iwp.compress_segmented(plan, w, g, r, lead_t, eps, idx, val, thr2[t % 2], ws, stream, thr_hint=hint)
            iwp.gather_sum_at_indices(r, idx, ps.K, sm, stream)
            iwp.apply_sparse_update(w, idx, sm, ps.K, scale, r, stream)

    algo_bytes = step_bytes(ps, W_acc, W_list)
    dom_bytes = dominant_kernel_bytes(ps, W_acc, W_list, route)
    blocks = []
    # Un-timed steps from zero residuals first: the residuals of elements that are not sent keep growing, so
    # over the first ~100 steps the importances pile up below the threshold (each 1/16-octave bin there ends
    # up holding about as many elements as a step sends).  That steady state, not the cold start, is what a
    # training run spends its time in, and it is the slower one for the selection.
    use_hint[0] = hint_modes[0]
    for t in range(args.preroll):
        step(t)
    # every mode then runs the same steps from the same state (the step time depends on how old the state is)
    snap = None
    if len(hint_modes) > 1:
        snap = (w.clone(), [x.clone() for x in r], [x.clone() for x in thr2])
    for hinted in hint_modes:
        use_hint[0] = hinted
        if snap is not None:
            w.copy_(snap[0])
            for x, y in zip(r, snap[1]):
                x.copy_(y)
            for x, y in zip(thr2, snap[2]):
                x.copy_(y)
        t_next = args.preroll
        for t in range(t_next, t_next + args.warmup):
            step(t)
        t_next += args.warmup
        ms_host, ms_ev = timed_steps(torch, stream, step, t_next, args.steps)
        t_next += args.steps
        dom_ms, dom_cnt, spread = profiled_steps(iwp, torch, stream, step, t_next, args.steps, dominant)
        t_next += args.steps
        b = result_block(ps, cfg, route, hinted, W_acc, W_list, pool, args.steps, args.warmup, ms_host, ms_ev, dominant,
                         dom_ms, dom_cnt, spread, algo_bytes, dom_bytes, workload, ps.K)
        blocks.append(b)
    blocks[0]["input_generation_s"] = gen_s
    for b in blocks:
        b["config"]["state"] = "%d un-timed steps from zero residuals precede the warm-up" % args.preroll

    # the parts on their own, after the timed regions (they change r and w further, which no longer matters):
    # (i) compression of one worker (accumulate + score + select + compact, every layer leads itself),
    # (ii) the exchange as the two separate calls over the K pairs the last step produced
    if want_parts:
        ws1 = torch.empty(max(1, plan.workspace_bytes), dtype=torch.uint8, device=dev)
        reps = 10

        def timed(fn):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / reps
        tc = timed(lambda: iwp.compress_segmented(plan, w, [grads[0]], [r[0]], None, eps, idx, val, thr2[0], ws1, stream))
        flip = [0]

        def hinted_call():                                 # hint: the records the previous call wrote
            flip[0] ^= 1
            iwp.compress_segmented(plan, w, [grads[0]], [r[0]], None, eps, idx, val, thr2[flip[0]], ws1, stream,
                                   thr_hint=thr2[flip[0] ^ 1])
        th = timed(hinted_call)
        tg = timed(lambda: iwp.gather_sum_at_indices(r, idx, ps.K, sm, stream))
        tu = timed(lambda: iwp.apply_sparse_update(w, idx, sm, ps.K, scale, r, stream))
        cb = 16 * ps.P + 8 * ps.K
        xb = (12 + 8 * W_list + 8) * ps.K
        blocks[0]["parts"] = {
            "compress_one_worker": {"ms": tc * 1e3, "params_per_s": ps.P / tc, "algorithmic_GBps": cb / tc / 1e9,
                                    "frac_of_hbm_peak": cb / tc / 1e9 / HBM_PEAK_GBPS},
            "compress_one_worker_hinted": {"ms": th * 1e3, "params_per_s": ps.P / th,
                                           "algorithmic_GBps": cb / th / 1e9,
                                           "frac_of_hbm_peak": cb / th / 1e9 / HBM_PEAK_GBPS},
            "exchange_two_calls": {"ms": (tg + tu) * 1e3, "pairs_per_s": ps.K / (tg + tu),
                                   "algorithmic_GBps": xb / (tg + tu) / 1e9, "gather_ms": tg * 1e3, "update_ms": tu * 1e3},
        }
        del ws1
    del w, grads, r, ws, idx, val, sm, snap
    torch.cuda.empty_cache()

    if want_cpu:
        if flat_cfg:
            # the oracle sorts every layer in full: at 1e9 elements one step takes minutes, so the sample is
            # the same workload at 1/50 of its length (2e7 elements, k = 2e4, local worker + 8 static peers)
            small = wl.make_config(5, scale_down=50 * args.scale_down)
            cb_ = oracle_baseline(small, wl.gen_weights(small), [wl.gen_gradient(small, 1 + s) for s in range(2)], 2, wl,
                                  args.steps, flat_note="the same workload at 1/50 of its length (%d elements, k = %d, "
                                  "local worker + 8 static peers)" % (small.P, small.K), W_list=9)
        else:
            cb_ = oracle_baseline(ps, w_np, grads_np, pool, wl, args.steps)
        blocks[0]["cpu_baseline"] = cb_
    return blocks


def bench_threshold(iwp, wl, torch, np, args):
    """Threshold routes (fixed, random selection, layer-wise) on one multi-worker workload."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    cfg = WORKLOADS[args.workload]
    assert cfg != 5, "the threshold route is measured on the multi-worker workloads"
    ps = wl.make_config(cfg, scale_down=args.scale_down)
    W = ps.W
    pool = W
    lw_mode = args.route == "layerwise"
    n_lead = args.n_lead
    t0 = time.time()
    w_np = wl.gen_weights(ps)
    grads_np = [wl.gen_gradient(ps, s) for s in range(pool)]
    w = torch.from_numpy(w_np).to(dev)
    grads = [torch.from_numpy(g).to(dev) for g in grads_np]
    r = [torch.zeros(ps.flat, device=dev) for _ in range(W)]
    gen_s = time.time() - t0
    plan = iwp.Plan(ps.rows())
    eps, scale = float(ps.eps), float(ps.scale)
    CAL = 8                                           # top-k steps that settle the thresholds
    total = CAL + 1 + args.warmup + 2 * args.steps
    ws = torch.empty(plan.step_workspace_bytes(W), dtype=torch.uint8, device=dev)
    idx = torch.empty(ps.K, dtype=torch.int32, device=dev)
    val = torch.empty(ps.K, dtype=torch.float32, device=dev)
    sm = torch.empty(ps.K, dtype=torch.float32, device=dev)
    thr2 = [torch.zeros(3 * len(ps.layers), dtype=torch.int32, device=dev) for _ in range(2)]
    leaders = torch.from_numpy(np.stack([wl.leaders(ps, t).astype(np.int32) for t in range(CAL)])).to(dev)
    # fixed thresholds: the k-th largest importance of each layer after CAL top-k steps,
    # so the mask keeps about the same share of every layer as the top-k route
    for t in range(CAL):
        g = [grads[wl.gradient_set_of(ps, p, t, pool)] for p in range(W)]
        iwp.step_segmented(plan, w, g, r, leaders[t], eps, scale, idx, val, sm, thr2[t % 2], ws, stream)
    torch.cuda.synchronize()
    fixed_thr = thr2[(CAL - 1) % 2].view(-1, 3)[:, 0].contiguous().view(torch.float32).clone()
    max_pairs = min(ps.P, (16 if args.random_selection else 8) * ps.K)
    del ws
    ws = torch.empty(plan.threshold_workspace_bytes(W, n_lead, max_pairs), dtype=torch.uint8, device=dev)
    mask = torch.empty(plan.mask_bytes, dtype=torch.uint8, device=dev)
    counts = torch.zeros(total, len(ps.layers) + 2, dtype=torch.int32, device=dev)
    idx = torch.empty(max_pairs, dtype=torch.int32, device=dev)
    sm = torch.empty(max_pairs, dtype=torch.float32, device=dev)
    chosen = torch.from_numpy(np.stack([wl.chosen_nodes(ps, t, n_lead).astype(np.int32).ravel()
                                        for t in range(total)])).to(dev)
    stats = torch.zeros(len(ps.layers), n_lead, 2, dtype=torch.float64, device=dev)
    thr_slots = torch.zeros(len(ps.layers), n_lead, dtype=torch.float32, device=dev)
    rule = None
    first = CAL
    if lw_mode:
        # one rule for all layers: alpha = the median calibrated threshold; one step with beta = 0
        # gives the layers' var/mean ratios; C = their median, beta = a 10 % correction at C
        alpha = float(fixed_thr.median())
        g0 = [grads[wl.gradient_set_of(ps, p, CAL, pool)] for p in range(W)]
        iwp.step_layerwise_segmented(plan, w, g0, r, chosen[CAL], n_lead, alpha, 0.0, 0.0, eps, scale, stats,
                                     thr_slots, mask, counts[CAL], idx, sm, max_pairs, ws, stream)
        torch.cuda.synchronize()
        ratio = (stats[:, :, 1] / stats[:, :, 0]).flatten()
        c_rule = float(ratio[torch.isfinite(ratio)].median())
        rule = (alpha, 0.1 * alpha / c_rule, c_rule)
        first = CAL + 1

    def step(t):
        g = [grads[wl.gradient_set_of(ps, p, t, pool)] for p in range(W)]
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
    t_a = first + args.warmup
    ms_host, ms_ev = timed_steps(torch, stream, step, t_a, args.steps)
    dominant = DOMINANT_KERNEL[args.route]
    dom_ms, dom_cnt, spread = profiled_steps(iwp, torch, stream, step, t_a + args.steps, args.steps, dominant)
    c = counts[t_a:t_a + args.steps].cpu().numpy()
    assert not c[:, -1].any(), "pair capacity exceeded in %d timed steps" % int(c[:, -1].sum())
    pairs_per_step = float(c[:, -2].mean())
    algo_bytes = threshold_step_bytes(ps, W, W, n_lead, pairs_per_step)
    if lw_mode:
        algo_bytes += layerwise_extra_bytes(ps, n_lead)
    dom_bytes = threshold_dominant_bytes(ps, W, W, n_lead, pairs_per_step)
    out = result_block(ps, cfg, args.route, True, W, W, pool, args.steps, args.warmup, ms_host, ms_ev, dominant, dom_ms,
                       dom_cnt, spread, algo_bytes, dom_bytes, args.workload, pairs_per_step)
    out["input_generation_s"] = gen_s
    out["config"]["threshold_hint"] = "n/a"
    out["config"]["chosen_nodes_per_layer"] = n_lead
    out["config"]["random_selection"] = bool(args.random_selection)
    out["config"]["thresholds"] = "fixed per layer: k-th largest importance after %d top-k steps" % CAL
    if lw_mode:
        out["config"]["thresholds"] = "alpha +/- beta * var/mean per layer and chosen node"
        out["config"]["rule"] = {"alpha": rule[0], "beta": rule[1], "C": rule[2]}
    out["config"]["pairs_per_step_min_max"] = [int(c[:, -2].min()), int(c[:, -2].max())]
    out["config"]["pair_capacity"] = max_pairs
    if not args.no_cpu_baseline:
        import oracle
        # the oracle's threshold-mode step from the state the GPU run ended in
        w_ref = w.cpu().numpy()
        r_ref = [x.cpu().numpy() for x in r]
        thr_np = fixed_thr.cpu().numpy()
        n_steps, spent = 0, 0.0
        while n_steps < 1 or (spent < 10.0 and n_steps < args.steps):
            t = total + n_steps
            g = [grads_np[wl.gradient_set_of(ps, p, t, pool)] for p in range(W)]
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
                      % (n_steps, W, len(ps.layers), spent),
            "host_cpus": os.cpu_count(),
        }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline", choices=["headline"] + sorted(WORKLOADS),
                    help="headline (default): the AlexNet-shaped set as the headline, plus under \"also\" the same "
                         "without hints and the ResNet-50-shaped set with and without hints; any other name: "
                         "that workload alone")
    ap.add_argument("--route", default="whole_step", choices=["whole_step", "three_calls", "threshold", "layerwise"],
                    help="whole_step: iwp_step_segmented; three_calls: compress_segmented + gather_sum_at_indices "
                         "+ apply_sparse_update (same results); threshold: iwp_step_threshold_segmented with fixed "
                         "per-layer thresholds (calibrated by a few top-k steps to the same keep ratio); layerwise: "
                         "iwp_step_layerwise_segmented, thresholds from each layer's importance mean / variance")
    ap.add_argument("--n-lead", type=int, default=1, help="threshold route: chosen nodes per layer")
    ap.add_argument("--random-selection", action="store_true",
                    help="threshold route: also send sub-threshold elements with probability importance / threshold")
    ap.add_argument("--no-hint", action="store_true",
                    help="top-k routes, single workload: measure only without the previous step's thresholds as a "
                         "hint (results are identical either way; the hint saves the second pass over the "
                         "leaders' layers)")
    ap.add_argument("--hinted-only", action="store_true",
                    help="top-k routes, single workload: skip the unhinted measurement (for profiler runs)")
    ap.add_argument("--preroll", type=int, default=200,
                    help="top-k routes: un-timed steps from zero residuals before the warm-up, so that the timed "
                         "steps see the steady state of the residuals (0 = cold start)")
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
    copy_gbps = copy_ceiling(iwp, torch, dev, torch.cuda.current_stream())
    thr_mode = args.route in ("threshold", "layerwise")
    if thr_mode:
        if args.workload == "headline":
            args.workload = "alexnet"
        out = bench_threshold(iwp, wl, torch, np, args)
    elif args.workload == "headline":
        a = bench_topk(iwp, wl, torch, np, args, "alexnet", [True, False], not args.no_parts, not args.no_cpu_baseline)
        b = bench_topk(iwp, wl, torch, np, args, "resnet50", [True, False], not args.no_parts, not args.no_cpu_baseline)
        out = a[0]
        out["also"] = {"alexnet_shaped_unhinted": a[1], "resnet50_shaped": b[0], "resnet50_shaped_unhinted": b[1]}
        if args.preroll:
            # the same two sets from zero residuals (the first steps of a run), hinted, for comparison
            cold = argparse.Namespace(**vars(args))
            cold.preroll = 0
            out["also"]["alexnet_shaped_cold_start"] = bench_topk(iwp, wl, torch, np, cold, "alexnet", [True], False, False)[0]
            out["also"]["resnet50_shaped_cold_start"] = bench_topk(iwp, wl, torch, np, cold, "resnet50", [True], False, False)[0]
    else:
        modes = [False] if args.no_hint else ([True] if args.hinted_only else [True, False])
        blocks = bench_topk(iwp, wl, torch, np, args, args.workload, modes, not args.no_parts, not args.no_cpu_baseline)
        out = blocks[0]
        if len(blocks) > 1:
            out["also"] = {out["config"]["workload"] + "_unhinted": blocks[1]}
    out["copy_kernel_GBps"] = copy_gbps
    out["paper_context"] = PAPER_CONTEXT
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
