"""Config 5 at its full size (one flat layer of 10^9 elements, local worker + 8
static peers, k = 10^6), in the launch configuration bench.py times (whole-step
route, second step hinted).  A full sort of 10^9 pairs is out of reach for the
oracle inside a test, so the outputs are checked against what the oracle can
compute at this size: its scores for every element (one pass), its rank-by-counting
for sampled elements, and its reduce / update on the compacted pairs; set-level
facts (cardinality, threshold record, membership of every element above the
threshold, tie quota) follow from the oracle's scores by plain comparisons."""
import numpy as np
import pytest

import oracle
from paper_1901_01544_amd import workloads as wl
from harness import bits

pytestmark = pytest.mark.gpu


def _check_step(tag, torch, keys, A_host, out_idx, out_val, thr, k, rng):
    n = keys.size
    idx = out_idx.cpu().numpy().view(np.uint32)
    val = out_val.cpu().numpy()
    key_t, n_gt, n_eq = [int(x) for x in thr.cpu().numpy().view(np.uint32)[:3]]
    # cardinality and order
    assert idx.size == k and np.all(np.diff(idx.astype(np.int64)) > 0) and int(idx[-1]) < n, tag
    # threshold record against the oracle's keys
    above = keys > np.uint32(key_t)
    ties = keys == np.uint32(key_t)
    assert int(above.sum()) == n_gt and n_gt < k <= n_gt + int(ties.sum()) and n_eq == k - n_gt, tag
    # membership: everything above the threshold, plus the first n_eq ties in index order
    want = np.concatenate([np.nonzero(above)[0], np.nonzero(ties)[0][:n_eq]])
    want.sort()
    assert np.array_equal(idx, want.astype(np.uint32)), tag
    # values are the accumulated residual bit for bit
    assert np.array_equal(bits(val), bits(A_host[idx])), tag
    # sampled elements, one by one, through the oracle's rank-by-counting
    s = keys.view(np.float32)
    sel = np.zeros(n, bool)
    sel[idx] = True
    lowest_kept = idx[np.argmin(keys[idx])]
    best_dropped = np.nonzero(~sel & (keys >= np.uint32(max(key_t, 1) - 1)))[0]
    picks = [int(idx[0]), int(idx[-1]), int(lowest_kept), int(rng.integers(0, n))]
    picks += [int(best_dropped[0])] if best_dropped.size else []
    for i in picks:
        assert (oracle.rank_of(s, i) < k) == bool(sel[i]), (tag, i)
    return idx, val


@pytest.mark.timeout(1500)
def test_config5_full_size_two_steps(gpu_lib):
    import torch
    iwp = gpu_lib
    dev = "cuda:0"
    ps = wl.make_config(5)
    n, k, W = ps.flat, ps.K, 9
    eps, scale = float(ps.eps), float(np.float32(-(ps.eta / W)))
    w = wl.gen_weights_device(ps, dev)
    w_host = w.cpu().numpy()
    r = [torch.zeros(n, device=dev)] + [wl.gen_laplace_device(ps, 100 + p, dev) for p in range(8)]
    plan = iwp.Plan(ps.rows())
    ws = torch.empty(plan.step_workspace_bytes(W), dtype=torch.uint8, device=dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    val = torch.empty(k, device=dev)
    sm = torch.empty(k, device=dev)
    thr = [torch.zeros(3, dtype=torch.int32, device=dev) for _ in range(2)]
    leader = torch.zeros(1, dtype=torch.int32, device=dev)
    rng = np.random.default_rng(5)
    A_host = np.zeros(n, np.float32)                      # the local worker's residual, mirrored on the host
    for t in range(2):
        g = wl.gen_laplace_device(ps, 1 + t, dev)
        oracle.accumulate(A_host, g.cpu().numpy())        # O1 on the host mirror
        keys = oracle.score_keys(w_host, A_host, eps)     # O2 for every element
        peers_before = [x.clone() for x in r[1:]]
        w_before = w.clone()
        iwp.step_segmented(plan, w, [g] + [None] * 8, r, leader, eps, scale, idx, val, sm, thr[t], ws,
                           thr_hint=thr[t - 1] if t else None)
        torch.cuda.synchronize()
        i_np, v_np = _check_step("step %d" % t, torch, keys, A_host, idx, val, thr[t], k, rng)
        # reduce and update on the compacted pairs through the oracle
        il = torch.from_numpy(i_np.astype(np.int64)).to(dev)
        rows = [v_np] + [peers_before[p].index_select(0, il).cpu().numpy() for p in range(8)]
        ar = np.arange(k, dtype=np.uint32)
        s_ref = oracle.gather_sum(rows, ar)
        assert np.array_equal(bits(sm.cpu().numpy()), bits(s_ref)), "sum step %d" % t
        w_sel = w_before.index_select(0, il).cpu().numpy()
        oracle.apply_sparse_update(w_sel, ar, s_ref, scale, [])
        assert np.array_equal(bits(w.index_select(0, il).cpu().numpy()), bits(w_sel)), "w step %d" % t
        w_before.index_copy_(0, il, w.index_select(0, il))
        assert torch.equal(w_before, w), "weights outside the index set changed"
        # residuals: cleared at the index set on all nine buffers, untouched elsewhere
        A_host[i_np] = 0.0
        assert torch.equal(r[0], torch.from_numpy(A_host).to(dev)), "local residual step %d" % t
        for p in range(8):
            peers_before[p].index_fill_(0, il, 0.0)
            assert torch.equal(peers_before[p], r[1 + p]), "peer %d step %d" % (p, t)
        del g, w_before, il, peers_before
        w_host = w.cpu().numpy()


@pytest.mark.timeout(900)
def test_config2_full_size_threshold_routes(gpu_lib):
    """The AlexNet-shaped set at full size (61.1 M parameters, 8 workers, one chosen node
    per layer: the configuration bench.py times on its threshold / layerwise routes): one
    fixed-threshold step, one with random selection, one with layer-wise thresholds, each
    against the oracle's whole step, every output bit for bit (the layer-wise statistics
    to 1e-6 relative, its decisions from the device's thresholds)."""
    import torch
    from harness import ThresholdSet
    iwp = gpu_lib
    ps = wl.make_config(2)
    W, nl = ps.W, len(ps.layers)
    eps, scale = float(ps.eps), float(ps.scale)
    w = wl.gen_weights(ps)
    pool = [wl.gen_gradient(ps, s) for s in range(2)]
    r0 = [np.zeros(ps.flat, np.float32) for _ in range(W)]
    max_pairs = ps.flat // 4
    ts = ThresholdSet(iwp, ps, w, pool, r0, 1, max_pairs)
    w_ref, r_ref = w.copy(), [x.copy() for x in r0]
    rows = ps.rows()
    # thresholds that keep about 1/64 of each layer on worker 0's first accumulated gradient
    thr = np.zeros(nl, np.float32)
    for j, L in enumerate(ps.layers):
        sl = slice(L.offset, L.offset + L.n)
        s = oracle.score(np.ascontiguousarray(w[sl]), np.ascontiguousarray(pool[0][sl]), eps)
        kk = max(1, L.n // 64)
        thr[j] = np.partition(s, L.n - kk)[L.n - kk]

    def compare(tag, ref):
        mask_ref, cnt_ref, idx_ref, sum_ref = ref
        got = ts.download()
        total = int(cnt_ref.sum())
        assert 0 < total <= max_pairs, (tag, total)
        assert np.array_equal(got["count"][:nl], cnt_ref) and got["count"][nl] == total and got["count"][nl + 1] == 0, tag
        assert np.array_equal(got["mask"], mask_ref), tag + " mask"
        assert np.array_equal(got["idx"][:total], idx_ref), tag + " idx"
        assert np.array_equal(bits(got["sum"][:total]), bits(sum_ref)), tag + " sum"
        assert np.array_equal(bits(got["w"]), bits(w_ref)), tag + " w"
        for p in range(W):
            assert np.array_equal(bits(got["r"][p]), bits(r_ref[p])), "%s residual %d" % (tag, p)
        return total

    for t, mode in enumerate(("threshold", "random", "layerwise")):
        ids = [(p + t) % 2 for p in range(W)]
        g = [pool[i] for i in ids]
        chosen = wl.chosen_nodes(ps, t, 1)
        if mode == "layerwise":
            alpha, beta, c = float(np.median(thr)), 1e-6, 50.0
            acc = [None] * nl
            want = np.zeros((nl, 2))
            for j, L in enumerate(ps.layers):
                sl = slice(L.offset, L.offset + L.n)
                a = r_ref[chosen[j, 0]][sl].copy()
                oracle.accumulate(a, np.ascontiguousarray(g[chosen[j, 0]][sl]))
                want[j] = oracle.layer_stats(np.ascontiguousarray(w_ref[sl]), a, eps)
            ts.step_layerwise(ids, chosen, alpha, beta, c, scale)
            stats = ts.stats.cpu().numpy()[:, 0, :]
            thr_dev = ts.thr_slots.cpu().numpy()[:, 0].copy()
            assert np.all(np.abs(stats - want) <= 1e-6 * np.abs(want)), (stats, want)
            for j in range(nl):
                assert bits(oracle.layerwise_threshold(stats[j, 0], stats[j, 1], alpha, beta, c)) == bits(thr_dev[j])
            ref = oracle.step_threshold(w_ref, g, r_ref, rows, chosen, thr_dev, eps, scale, max_pairs)
        else:
            rnd = (ps.seed, t) if mode == "random" else None
            ref = oracle.step_threshold(w_ref, g, r_ref, rows, chosen, thr, eps, scale, max_pairs, random=rnd)
            ts.step(ids, chosen, thr, scale, random=rnd)
        total = compare(mode, ref)
        print("%s: %d pairs sent" % (mode, total), flush=True)


@pytest.mark.timeout(2400)
def test_largest_supported_layer(gpu_lib):
    """One layer of the largest size the 32-bit positions allow (2^32 - 65536 - 3 elements, a
    ragged last tile), one worker: a top-k whole step and a threshold-mode step.  The oracle
    cannot sort this many pairs inside a test, so -- as for the 10^9-element set above -- the
    outputs are checked against what it can compute at this size: its scores for every
    element, its rank-by-counting for sampled elements, its encoded mask, its reduce / update
    on the compacted pairs, and set-level facts that follow from its scores by comparisons."""
    import torch
    iwp = gpu_lib
    dev = "cuda:0"
    n = 0xFFFF0000 - 3
    k = 1_000_003
    eps, scale = 1e-8, float(np.float32(-0.01))
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260)
    w = torch.empty(n, device=dev).normal_(0.0, 0.02, generator=gen)
    g = torch.empty(n, device=dev).normal_(0.0, 1e-4, generator=gen)
    g[-5000:] *= 50.0                                        # kept elements in the very last tiles and at the last position
    g[:3] = 1.0                                              # and at the first / last positions for certain
    g[-1] = -1.0
    r = torch.zeros(n, device=dev)
    print("inputs drawn", flush=True)
    w_host = w.cpu().numpy()
    A_host = np.zeros(n, np.float32)
    oracle.accumulate(A_host, g.cpu().numpy())               # O1 on the host mirror
    keys = oracle.score_keys(w_host, A_host, eps)            # O2 for every element
    print("oracle scores done", flush=True)
    plan = iwp.Plan([(0, n, k, 0)])
    ws = torch.empty(plan.step_workspace_bytes(1), dtype=torch.uint8, device=dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    val = torch.empty(k, device=dev)
    sm = torch.empty(k, device=dev)
    thr = torch.zeros(3, dtype=torch.int32, device=dev)
    leader = torch.zeros(1, dtype=torch.int32, device=dev)
    w_before = w.clone()
    iwp.step_segmented(plan, w, [g], [r], leader, eps, scale, idx, val, sm, thr, ws)
    torch.cuda.synchronize()
    print("top-k step done", flush=True)
    rng = np.random.default_rng(3)
    i_np, v_np = _check_step("largest layer", torch, keys, A_host, idx, val, thr, k, rng)
    assert int(i_np[-1]) == n - 1 and i_np[:3].tolist() == [0, 1, 2], "the planted extremes at both ends are kept"
    print("selection checked", flush=True)
    il = torch.from_numpy(i_np.astype(np.int64)).to(dev)
    ar = np.arange(k, dtype=np.uint32)
    s_ref = oracle.gather_sum([v_np], ar)                    # one worker: the sum is the value, through O5
    assert np.array_equal(bits(sm.cpu().numpy()), bits(s_ref))
    w_sel = w_before.index_select(0, il).cpu().numpy()
    oracle.apply_sparse_update(w_sel, ar, s_ref, scale, [])
    assert np.array_equal(bits(w.index_select(0, il).cpu().numpy()), bits(w_sel))
    w_before.index_copy_(0, il, w.index_select(0, il))
    assert torch.equal(w_before, w), "weights outside the index set changed"
    del w_before
    A_host[i_np] = 0.0
    assert torch.equal(r, torch.from_numpy(A_host).to(dev)), "residual after the top-k step"
    w_host[i_np] = w_sel
    print("top-k step checked", flush=True)

    # threshold mode on the state the first step left (no new gradient): a threshold somewhat below the
    # k-th largest importance of before, so the mask holds the next few hundred thousand elements
    key_t = int(thr.cpu().numpy().view(np.uint32)[0])
    t_f = np.float32(np.array([key_t], np.uint32).view(np.float32)[0] * np.float32(0.9))
    del keys
    mask_ref = oracle.mask_threshold(w_host, A_host, eps, float(t_f))      # T1 + T2 over the whole layer
    want = np.nonzero(np.unpackbits(mask_ref, bitorder="little")[:n])[0].astype(np.uint32)
    total = want.size
    assert 1000 < total < 4_000_000, total
    print("oracle mask done: %d marked" % total, flush=True)
    cap = 4_000_000
    ws2 = torch.empty(plan.threshold_workspace_bytes(1, 1, cap), dtype=torch.uint8, device=dev)
    mask = torch.zeros(plan.mask_bytes, dtype=torch.uint8, device=dev)
    count = torch.zeros(3, dtype=torch.int32, device=dev)
    idx2 = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    sum2 = torch.full((cap,), float("nan"), device=dev)
    thr_d = torch.tensor([float(t_f)], device=dev)
    w_before = w.clone()
    iwp.step_threshold_segmented(plan, w, [None], [r], leader, 1, thr_d, eps, scale, mask, count, idx2, sum2, cap, ws2)
    torch.cuda.synchronize()
    print("threshold step done", flush=True)
    assert count.cpu().tolist() == [total, total, 0]
    assert np.array_equal(mask.cpu().numpy(), mask_ref), "encoded mask"
    got_idx = idx2.cpu().numpy().view(np.uint32)
    assert np.array_equal(got_idx[:total], want) and np.all(got_idx[total:] == 0xFFFFFFFF)
    s2 = oracle.gather_sum([A_host[want]], np.arange(total, dtype=np.uint32))
    assert np.array_equal(bits(sum2.cpu().numpy()[:total]), bits(s2))
    il = torch.from_numpy(want.astype(np.int64)).to(dev)
    w_sel = w_before.index_select(0, il).cpu().numpy()
    oracle.apply_sparse_update(w_sel, np.arange(total, dtype=np.uint32), s2, scale, [])
    assert np.array_equal(bits(w.index_select(0, il).cpu().numpy()), bits(w_sel))
    w_before.index_copy_(0, il, w.index_select(0, il))
    assert torch.equal(w_before, w), "weights outside the mask changed"
    A_host[want] = 0.0
    assert torch.equal(r, torch.from_numpy(A_host).to(dev)), "residual after the threshold step"
