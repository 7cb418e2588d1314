"""The whole-step entry points issue only kernel launches on the caller's stream (the
workspace is cleared by a fill kernel, not a memset), so a caller can capture them into
a HIP graph.  Each captured step is replayed several times, with eager work and
synchronisation between the replays, and every replay must reproduce the eager result
(which test_gpu_parity / test_gpu_threshold tie to the oracle) bit for bit."""
import numpy as np
import pytest

from paper_1901_01544_amd import workloads as wl
from harness import bits

pytestmark = pytest.mark.gpu
EPS = 1e-8


def _state(torch, ps, W, seed):
    rng = np.random.default_rng(seed)
    w = torch.from_numpy(wl.gen_weights(ps)).cuda()
    g = [torch.from_numpy(wl.gen_gradient(ps, s)).cuda() for s in range(W)]
    r = [torch.from_numpy((rng.standard_t(3, ps.flat) * 1e-3).astype(np.float32)).cuda() for _ in range(W)]
    return w, g, r


@pytest.mark.parametrize("route", ["whole_step", "threshold", "layerwise"])
def test_captured_step_replays_like_eager(gpu_lib, route):
    import torch
    iwp = gpu_lib
    sizes = [(300, 5), (4097, 70), (0, 0), (40000, 625), (32768 + 3, 600), (5, 0), (100_003, 1500)]
    ps = wl.custom_set(sizes, W=4, seed=61, align=64, zero_frac=0.01)
    W, nl = 4, len(ps.layers)
    plan = iwp.Plan(ps.rows())
    w0, g, r0 = _state(torch, ps, W, 3)
    w = w0.clone()
    r = [x.clone() for x in r0]
    K = ps.K
    cap = ps.flat
    leader = torch.tensor([1, 0, 3, 2, 1, 0, 2], dtype=torch.int32, device="cuda")
    outs = {}
    if route == "whole_step":
        ws = torch.empty(plan.step_workspace_bytes(W), dtype=torch.uint8, device="cuda")
        outs = dict(idx=torch.empty(K, dtype=torch.int32, device="cuda"), val=torch.empty(K, device="cuda"),
                    sum=torch.empty(K, device="cuda"), thr=torch.zeros(3 * nl, dtype=torch.int32, device="cuda"))
        hint = torch.zeros(3 * nl, dtype=torch.int32, device="cuda")

        def call():
            iwp.step_segmented(plan, w, g, r, leader, EPS, -0.01, outs["idx"], outs["val"], outs["sum"], outs["thr"],
                               ws, thr_hint=hint)
    else:
        ws = torch.empty(plan.threshold_workspace_bytes(W, 2, cap), dtype=torch.uint8, device="cuda")
        outs = dict(mask=torch.zeros(plan.mask_bytes, dtype=torch.uint8, device="cuda"),
                    count=torch.zeros(nl + 2, dtype=torch.int32, device="cuda"),
                    idx=torch.empty(cap, dtype=torch.int32, device="cuda"), sum=torch.empty(cap, device="cuda"),
                    stats=torch.zeros(nl, 2, 2, dtype=torch.float64, device="cuda"),
                    thr_slots=torch.zeros(nl, 2, dtype=torch.float32, device="cuda"))
        if route == "threshold":                                  # the statistics belong to the layer-wise route only
            stats_buf, thr_buf = outs.pop("stats"), outs.pop("thr_slots")
        chosen = torch.tensor([[1, 2], [0, 0], [3, 1], [2, 0], [1, 3], [0, 1], [2, 2]], dtype=torch.int32,
                              device="cuda").flatten().contiguous()
        thr = torch.full((nl,), 0.05, device="cuda")

        def call():
            if route == "threshold":
                iwp.step_threshold_random_segmented(plan, w, g, r, chosen, 2, thr, 11, 5, EPS, -0.01, outs["mask"],
                                                    outs["count"], outs["idx"], outs["sum"], cap, ws)
            else:
                iwp.step_layerwise_segmented(plan, w, g, r, chosen, 2, 0.05, 1e-5, 100.0, EPS, -0.01, outs["stats"],
                                             outs["thr_slots"], outs["mask"], outs["count"], outs["idx"], outs["sum"],
                                             cap, ws)

    def reset(fill):
        w.copy_(w0)
        for a, b in zip(r, r0):
            a.copy_(b)
        for k, v in outs.items():                                 # stale outputs must not survive a replay
            if v.dtype in (torch.float32, torch.float64):
                v.fill_(float(fill))
            else:
                v.fill_(fill % 100)

    def snapshot():
        torch.cuda.synchronize()
        d = {k: v.cpu().numpy().copy() for k, v in outs.items()}
        d["w"] = w.cpu().numpy().copy()
        for p in range(W):
            d["r%d" % p] = r[p].cpu().numpy().copy()
        if "thr" in d:                                            # records of layers without selection are not written
            keep = np.repeat(np.array([L.k > 0 for L in ps.layers]), 3)
            d["thr"] = d["thr"][keep]
        if "count" in d:                                          # only the valid part of the packed outputs
            n = int(d["count"][nl])
            d["idx"], d["sum"] = d["idx"][:n], d["sum"][:n]
        return d

    reset(7)
    call()
    want = snapshot()
    assert (want.get("count", np.ones(nl + 2))[nl] if "count" in want else K) > 0

    reset(9)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for replay in range(4):
        reset(20 + replay)
        (w * 2).sum().item()                                      # eager work and a synchronisation between replays
        graph.replay()
        got = snapshot()
        for k in want:
            a, b = got[k], want[k]
            same = np.array_equal(a.view(np.uint8), b.view(np.uint8)) if a.dtype.kind == "f" else np.array_equal(a, b)
            assert same, "replay %d: %s differs from the eager result" % (replay, k)
