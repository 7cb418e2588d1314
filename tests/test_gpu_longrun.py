"""GPU parity over the configurations' whole step loop (Alg. 1, `for t = 1, 2, ...`): the benchmarked
route (whole step, hint = the previous step's threshold records) and the three other routes, side by side
on the same inputs, every output compared bit for bit with the CPU oracle after every step, at full size.

The state such a run reaches is what a few steps cannot show: residuals many steps old, thresholds that
drift, hints that hit on some layers and miss on others inside one launch.  To force the latter, from step
DISTURB_AT on every third layer's gradients are scaled by 8 and every third layer's by 1/8 (powers of two:
the scaled sets are exact), and on the MIXED_HINT steps the hinted sets receive last step's records moved
three top-digit bins up (misses), three bins down (over-full slots) or zeroed, by layer.  Hints never
change a bit of the output; which layers' first looks were complete is derived from the records and
asserted to be a mix.

The oracle's step is the slow part (a full sort per layer), so one oracle run serves all four routes:
the sets step in lockstep and are compared on the device against one uploaded copy of the oracle's state.
Windows: config 2 (AlexNet-shaped) 12 of its 100 steps, config 3 (ResNet-50-shaped) 40 of 100,
config 4 (many small) all 10, config 1 all 10 (test_gpu_parity.py); threshold modes 5 consecutive steps each."""
import time

import numpy as np
import pytest

import oracle
from paper_1901_01544_amd import workloads as wl
from harness import DeviceRef, GpuSet, ThresholdSet, bits

pytestmark = pytest.mark.gpu
DISTURB_AT = 5
MIXED_HINT = (3, 8)
ROUTES = {"three_calls": dict(fused=False, hint="none"), "three_calls_hinted": dict(fused=False, hint="previous"),
          "whole_step": dict(fused=True, hint="none"), "whole_step_hinted": dict(fused=True, hint="previous")}
TOP_SHIFT = 19                                   # the selection's first key digit: bits 19..30


def _layer_factors(ps):
    """Per-element factor of the disturbed gradient sets: layer j is scaled by 8, 1 or 1/8 (j mod 3)."""
    f = np.ones(ps.flat, np.float32)
    for j, L in enumerate(ps.layers):
        f[L.offset:L.offset + L.n] = (8.0, 1.0, 0.125)[j % 3]
    return f


def _mixed_hint(prev_thr):
    h = prev_thr.astype(np.uint32).copy()
    j = np.arange(h.shape[0])
    key = h[:, 0].astype(np.int64)
    key = np.where(j % 4 == 1, key + (3 << TOP_SHIFT), key)
    key = np.where(j % 4 == 2, np.maximum(key - (3 << TOP_SHIFT), 0), key)
    key = np.where(j % 4 == 3, 0, key)
    h[:, 0] = np.minimum(key, 0x7F7FFFFF).astype(np.uint32)
    return h


def _first_look_complete(hint, thr_now, layers):
    """Per selecting layer: did a first look staged from `hint` already hold every candidate?  (The first
    look copies out everything from one bin below the hinted bin, if that bin is at least 2.)"""
    out = []
    for j, L in enumerate(layers):
        if L.k == 0:
            continue
        hb = int(hint[j][0] & 0x7FFFFFFF) >> TOP_SHIFT
        out.append(hb >= 2 and hb - 1 <= int(thr_now[j][0]) >> TOP_SHIFT)
    return np.array(out, bool)


def _long_run(iwp, cfg, steps, pool, tag):
    import torch
    ps = wl.make_config(cfg)
    W = ps.W
    w = wl.gen_weights(ps)
    base = [wl.gen_gradient(ps, s) for s in range(pool)]
    f = _layer_factors(ps)
    sets = base + [g * f for g in base]                       # ids pool.. = the disturbed sets
    del f
    grads_dev = [torch.from_numpy(g).to("cuda:0") for g in sets]
    gss = {name: GpuSet(iwp, ps, w, None, grads_dev=grads_dev, **kw) for name, kw in ROUTES.items()}
    w_ref = w.copy()
    r_ref = [np.zeros(ps.flat, np.float32) for _ in range(W)]
    rows = ps.rows()
    prev_thr = None
    mixes = []
    t0 = time.time()
    for t in range(steps):
        lead = wl.leaders(ps, t)
        ids = [wl.gradient_set_of(ps, p, t, pool) + (pool if t >= DISTURB_AT else 0) for p in range(W)]
        ref = oracle.step(w_ref, [sets[i] for i in ids], r_ref, rows, lead, float(ps.eps), float(ps.scale))
        dref = DeviceRef(torch, w_ref, r_ref, *ref)
        hint = _mixed_hint(prev_thr) if (t in MIXED_HINT and prev_thr is not None) else None
        for name, gs in gss.items():
            gs.step(ids, lead, hint_records=hint)
            dref.check(gs, ps.layers, tag="%s %s step %d" % (tag, name, t))
        thr_now = ref[3]
        if prev_thr is not None:
            done = _first_look_complete(prev_thr if hint is None else hint, thr_now, ps.layers)
            mixes.append((t, int(done.sum()), int((~done).sum())))
        prev_thr = np.array(thr_now, np.uint32).reshape(-1, 3).copy()
        del dref
        print("%s step %d ok, %.1f s" % (tag, t, time.time() - t0), flush=True)
    print(tag, "layers whose hinted first look was complete / not, per step:", mixes, flush=True)
    # the run saw hints hitting and missing inside one launch
    assert any(a > 0 and b > 0 for _, a, b in mixes), mixes
    return mixes, prev_thr


@pytest.mark.timeout(900)
def test_config3_resnet50_shaped_40_steps_all_routes(gpu_lib):
    _long_run(gpu_lib, 3, 40, pool=4, tag="cfg3")


@pytest.mark.timeout(900)
def test_config2_alexnet_shaped_12_steps_all_routes(gpu_lib):
    _long_run(gpu_lib, 2, 12, pool=3, tag="cfg2")


@pytest.mark.timeout(900)
def test_config4_many_small_all_10_steps_all_routes(gpu_lib):
    ps = wl.make_config(4)
    mixes, last_thr = _long_run(gpu_lib, 4, ps.steps, pool=3, tag="cfg4")
    assert len(mixes) == 9
    # the tie-heavy layers really put their cut inside the run of equal scores
    tie_cut = [j for j, L in enumerate(ps.layers) if L.block is not None and last_thr[j][0] == 0]
    assert len(tie_cut) >= 10


@pytest.mark.timeout(900)
@pytest.mark.parametrize("mode", ["threshold", "random", "layerwise"])
def test_config2_threshold_modes_5_consecutive_steps(gpu_lib, mode):
    """Five consecutive steps of each threshold mode on the AlexNet-shaped set at full size, two chosen
    nodes per layer, fixed thresholds that keep about 1/64 of the first accumulated gradient."""
    import torch
    iwp = gpu_lib
    ps = wl.make_config(2)
    W, nl, n_lead = ps.W, len(ps.layers), 2
    eps, scale = float(ps.eps), float(ps.scale)
    w = wl.gen_weights(ps)
    pool = [wl.gen_gradient(ps, s) for s in range(3)]
    r0 = [np.zeros(ps.flat, np.float32) for _ in range(W)]
    max_pairs = ps.flat // 4
    ts = ThresholdSet(iwp, ps, w, pool, r0, n_lead, max_pairs)
    w_ref, r_ref = w.copy(), [x.copy() for x in r0]
    rows = ps.rows()
    thr = np.zeros(nl, np.float32)
    for j, L in enumerate(ps.layers):
        sl = slice(L.offset, L.offset + L.n)
        s = oracle.score(np.ascontiguousarray(w[sl]), np.ascontiguousarray(pool[0][sl]), eps)
        kk = max(1, L.n // 64)
        thr[j] = np.partition(s, L.n - kk)[L.n - kk]
    i32 = lambda x: x.view(torch.int32)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).to("cuda:0")
    for t in range(5):
        ids = [(p + t) % 3 for p in range(W)]
        g = [pool[i] for i in ids]
        chosen = wl.chosen_nodes(ps, t, n_lead)
        if mode == "layerwise":
            alpha, beta, c = float(np.median(thr)), 1e-6, 50.0
            want = np.zeros((nl, n_lead, 2))
            for j, L in enumerate(ps.layers):
                sl = slice(L.offset, L.offset + L.n)
                for q in range(n_lead):
                    a = r_ref[chosen[j, q]][sl].copy()
                    oracle.accumulate(a, np.ascontiguousarray(g[chosen[j, q]][sl]))
                    want[j, q] = oracle.layer_stats(np.ascontiguousarray(w_ref[sl]), a, eps)
            ts.step_layerwise(ids, chosen, alpha, beta, c, scale)
            stats = ts.stats.cpu().numpy()
            thr_dev = ts.thr_slots.cpu().numpy().copy()
            assert np.all(np.abs(stats - want) <= 1e-6 * np.abs(want)), (t, stats, want)      # per-layer reductions
            for j in range(nl):
                for q in range(n_lead):
                    assert bits(oracle.layerwise_threshold(stats[j, q, 0], stats[j, q, 1], alpha, beta, c)) == \
                        bits(thr_dev[j, q])
            ref = oracle.step_threshold(w_ref, g, r_ref, rows, chosen, thr_dev, eps, scale, max_pairs)
        else:
            rnd = (ps.seed, t) if mode == "random" else None
            ref = oracle.step_threshold(w_ref, g, r_ref, rows, chosen, thr, eps, scale, max_pairs, random=rnd)
            ts.step(ids, chosen, thr, scale, random=rnd)
        mask_ref, cnt_ref, idx_ref, sum_ref = ref
        total = int(cnt_ref.sum())
        tag = "%s step %d" % (mode, t)
        assert 0 < total <= max_pairs, (tag, total)
        cnt = ts.count.cpu().numpy().view(np.uint32)
        assert np.array_equal(cnt[:nl], cnt_ref) and cnt[nl] == total and cnt[nl + 1] == 0, tag
        assert np.array_equal(ts.mask.cpu().numpy()[:ts.plan.mask_bytes], mask_ref), tag + " mask"
        assert np.array_equal(ts.idx.cpu().numpy().view(np.uint32)[:total], idx_ref), tag + " idx"
        assert np.array_equal(bits(ts.sum.cpu().numpy()[:total]), bits(sum_ref)), tag + " sum"
        assert torch.equal(i32(ts.w), up(w_ref)), tag + " w"
        for p in range(W):
            assert torch.equal(i32(ts.r[p]), up(r_ref[p])), "%s residual %d" % (tag, p)
        print("%s: %d pairs sent" % (tag, total), flush=True)
