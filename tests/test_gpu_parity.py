"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs, bit for bit (index sets, sent values, thresholds, sums,
weights and every residual buffer).  Tolerance: none -- all outputs are integers
or fp32 values produced by a fixed sequence of IEEE operations."""
import numpy as np
import pytest

import oracle
from paper_1901_01544_amd import workloads as wl
from harness import GpuSet, assert_step_equal, bits

pytestmark = pytest.mark.gpu
TILE = 4096          # streaming tile; the leader-side passes work on super-tiles of 8 tiles
STILE = 8 * TILE
EPS = 1e-8


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _run_single(iwp, torch, w, g, r, k, eps=EPS, misalign=0):
    """compress_layer on one layer; returns (idx, val, r_after).  misalign: shift
    every buffer by that many elements off its 16-byte boundary."""
    n = r.size

    def place(a, dtype):
        buf = torch.zeros(n + 8, dtype=dtype, device="cuda:0")
        view = buf[misalign:misalign + n]
        view.copy_(torch.from_numpy(a))
        return buf, view

    _, wd = place(w, torch.float32)
    _, gd = place(g, torch.float32)
    rb, rd = place(r, torch.float32)
    ib = torch.full((max(1, k) + 8,), -1, dtype=torch.int32, device="cuda:0")
    vb = torch.full((max(1, k) + 8,), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(iwp.workspace_bytes(n, k), dtype=torch.uint8, device="cuda:0")
    iwp.compress_layer(wd, gd, rd, k, eps, ib[misalign:], vb[misalign:], ws, n=n)
    torch.cuda.synchronize()
    idx = ib.cpu().numpy().view(np.uint32)
    val = vb.cpu().numpy()
    # nothing written outside [misalign, misalign + k)
    assert np.all(idx[:misalign] == 0xFFFFFFFF) and np.all(idx[misalign + k:] == 0xFFFFFFFF)
    assert np.all(np.isnan(val[:misalign])) and np.all(np.isnan(val[misalign + k:]))
    rall = rb.cpu().numpy()
    assert not rall[:misalign].any() and not rall[misalign + n:].any()
    return idx[misalign:misalign + k], val[misalign:misalign + k], rall[misalign:misalign + n]


def _check_single(iwp, torch, w, g, r, k, eps=EPS, misalign=0, tag=""):
    r_ref = r.copy()
    idx_ref, val_ref, _ = oracle.compress_layer(w, g, r_ref, k, eps) if k else (np.empty(0, np.uint32), np.empty(0, np.float32), None)
    if k == 0:
        oracle.accumulate(r_ref, g)
    idx, val, r_after = _run_single(iwp, torch, w, g, r, k, eps, misalign)
    assert np.array_equal(bits(r_after), bits(r_ref)), tag + " residual"
    assert np.array_equal(idx, idx_ref), "%s idx: got %s want %s" % (tag, idx[:8], idx_ref[:8])
    assert np.array_equal(bits(val), bits(val_ref)), tag + " val"


def _layer(rng, n, zero_w=0.001):
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    w[rng.random(n) < zero_w] = 0.0
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    r = (rng.standard_t(3, n) * 2e-3).astype(np.float32)
    return w, g, r


# ---------------------------------------------------------------- device arithmetic

def test_device_arithmetic_matches_ieee(gpu_lib):
    """Importance keys computed on the device equal the oracle's for random and edge
    bit patterns: correctly rounded divide, denormals kept, eps added first."""
    import torch
    rng = np.random.default_rng(1)
    n = 1 << 20
    w = rng.standard_normal(n).astype(np.float32)
    r = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    edge_w = np.array([0.0, -0.0, 1e-8, -1e-8, 0.25, 3e38, 1e-30, -1e-38, 1.0, 0.0, 1e-45, 3.4e38], np.float32)
    edge_r = np.array([1e-3, 0.0, -1e-8, 2e-8, 1e-3, 1e-38, 1e-44, 1e-45, 1e-40, 3e38, 1e-45, 1e-45], np.float32)
    w[:12], r[:12] = edge_w, edge_r
    raw = rng.integers(0, 1 << 32, 4096, dtype=np.uint64).astype(np.uint32)      # arbitrary finite bit patterns
    wr = raw.view(np.float32).copy()
    wr[~np.isfinite(wr)] = 1.0
    rr = np.roll(wr, 7)
    w[100:100 + 4096], r[100:100 + 4096] = wr, rr
    for eps in (1e-8, 0.0, 1e-3):
        if eps == 0.0:
            ww = np.where(w == 0, np.float32(1.0), w)       # 0/0 is NaN: inputs must keep scores defined
        else:
            ww = w
        key = torch.empty(n, dtype=torch.int32, device="cuda:0")
        gpu_lib.score_keys(_dev(torch, ww), _dev(torch, r), eps, key)
        torch.cuda.synchronize()
        ref = oracle.score_keys(ww, r, eps)
        got = key.cpu().numpy().view(np.uint32)
        bad = np.nonzero(got != ref)[0]
        assert bad.size == 0, (eps, bad[:5], ww[bad[:5]], r[bad[:5]], got[bad[:5]], ref[bad[:5]])


def test_update_is_two_roundings_not_fma(gpu_lib):
    import torch
    rng = np.random.default_rng(2)
    k = 100000
    w = rng.standard_normal(k).astype(np.float32)
    s = rng.standard_normal(k).astype(np.float32)
    w[0], s[0], scale = 1.0, 1 + 2.0 ** -12, np.float32(-(1 + 2.0 ** -12))
    idx = np.arange(k, dtype=np.uint32)
    w_ref = w.copy()
    oracle.apply_sparse_update(w_ref, idx, s, float(scale), [])
    wd = _dev(torch, w)
    gpu_lib.apply_sparse_update(wd, _dev(torch, idx.view(np.int32)), _dev(torch, s), k, float(scale), [])
    torch.cuda.synchronize()
    assert np.array_equal(bits(wd.cpu().numpy()), bits(w_ref))


# ---------------------------------------------------------------- one layer, edge cases

@pytest.mark.parametrize("n", [1, 2, 3, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4097,
                               TILE - 1, TILE, TILE + 1, STILE - 1, STILE, STILE + 1, 65535, 65537, 3 * STILE + 5])
def test_single_layer_sizes(gpu_lib, n):
    import torch
    rng = np.random.default_rng(n)
    w, g, r = _layer(rng, n)
    for k in sorted({1, n, max(1, n // 64), max(1, n // 2)}):
        _check_single(gpu_lib, torch, w, g, r, k, tag="n=%d k=%d" % (n, k))
    _check_single(gpu_lib, torch, w, g, r, 0, tag="n=%d accumulate only" % n)


@pytest.mark.parametrize("misalign", [1, 2, 3])
def test_single_layer_misaligned_buffers(gpu_lib, misalign):
    import torch
    rng = np.random.default_rng(40 + misalign)
    for n in (5, 1000, TILE + 77, STILE + TILE + 77, 70001):
        w, g, r = _layer(rng, n)
        _check_single(gpu_lib, torch, w, g, r, max(1, n // 50), misalign=misalign, tag="n=%d mis=%d" % (n, misalign))


def test_single_layer_degenerate_values(gpu_lib):
    import torch
    rng = np.random.default_rng(50)
    n = 2 * STILE + 100
    w, g, r = _layer(rng, n)
    z = np.zeros(n, np.float32)
    one = np.ones(n, np.float32)
    # all-zero residual and gradient: every score +0, first k positions
    _check_single(gpu_lib, torch, w, z, z, 300, tag="all zero")
    # all scores equal; the tie cut falls on, just before and just after a tile boundary
    for k in (1, TILE - 1, TILE, TILE + 1, STILE - 1, STILE, STILE + 1, n - 1, n):
        _check_single(gpu_lib, torch, one, z, np.full(n, 0.5, np.float32), k, eps=0.0, tag="all equal k=%d" % k)
    # w == 0 everywhere: score = |r| / eps
    _check_single(gpu_lib, torch, z, g, r, 777, tag="w zero")
    # +inf and denormal scores
    r2, w2 = r.copy(), w.copy()
    r2[[5, 9000, n - 1]] = [3e38, -3e38, 3e38]
    w2[[5, 9000, n - 1]] = 0.0
    r2[100:200] = 1e-42
    w2[100:200] = 1.0
    _check_single(gpu_lib, torch, w2, z, r2, 2, tag="inf ties")
    _check_single(gpu_lib, torch, w2, z, r2, n - 50, tag="denormal scores kept in order")
    # few distinct values: heavy ties at every level of the key
    r3 = (np.round(rng.standard_normal(n) * 4) / 4).astype(np.float32)
    for k in (10, n // 3, n - 10):
        _check_single(gpu_lib, torch, one, z, r3, k, eps=0.0, tag="quantised k=%d" % k)
    # a block-concentrated residual: 99 % of the layer ties at +0 and the cut falls inside the tie
    r4 = z.copy()
    r4[TILE - 50:TILE + 150] = rng.standard_normal(200).astype(np.float32)
    _check_single(gpu_lib, torch, w, z, r4, 1000, tag="block concentrated")
    # keys that differ only in the lowest digit
    base = np.float32(1.0).view(np.uint32)
    r5 = (base + rng.integers(0, 1024, n).astype(np.uint32)).view(np.float32)
    _check_single(gpu_lib, torch, one, z, r5, n // 7, eps=0.0, tag="low digit only")


def test_select_then_compact_equals_compress(gpu_lib):
    import torch
    rng = np.random.default_rng(60)
    n, k = 5 * STILE + 123, 4000
    w, g, r = _layer(rng, n)
    wd, rd = _dev(torch, w), _dev(torch, r)
    ws = torch.empty(gpu_lib.workspace_bytes(n, k), dtype=torch.uint8, device="cuda:0")
    thr = torch.zeros(3, dtype=torch.int32, device="cuda:0")
    idx = torch.empty(k, dtype=torch.int32, device="cuda:0")
    val = torch.empty(k, dtype=torch.float32, device="cuda:0")
    gpu_lib.select_threshold(wd, rd, k, EPS, thr, ws)
    gpu_lib.compact_pairs(wd, rd, EPS, thr, k, idx, val, ws)
    torch.cuda.synchronize()
    assert np.array_equal(bits(rd.cpu().numpy()), bits(r))                     # r is read-only here
    thr_ref = oracle.select_threshold(w, r, k, EPS)
    assert tuple(thr.cpu().numpy().view(np.uint32).tolist()) == thr_ref
    idx_ref, _ = oracle.select(oracle.score(w, r, EPS), k)
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), idx_ref)
    assert np.array_equal(bits(val.cpu().numpy()), bits(oracle.take(r, idx_ref)))


def test_exchange_kernels(gpu_lib):
    import torch
    rng = np.random.default_rng(70)
    n, k = 300000, 5000
    for W in (1, 2, 8, 9):
        R = [(rng.standard_t(3, n) * 1e-3).astype(np.float32) for _ in range(W)]
        R[0][:4] = [-0.0, 1.0, 2.0 ** -24, 1e-40]
        w = rng.standard_normal(n).astype(np.float32)
        idx = np.sort(rng.choice(n, k, replace=False)).astype(np.uint32)
        idx[:4] = [0, 1, 2, 3]
        Rd = [_dev(torch, x) for x in R]
        wd, idxd = _dev(torch, w), _dev(torch, idx.view(np.int32))
        s = torch.empty(k, dtype=torch.float32, device="cuda:0")
        gpu_lib.gather_sum_at_indices(Rd, idxd, k, s)
        gpu_lib.apply_sparse_update(wd, idxd, s, k, -0.00125, Rd)
        torch.cuda.synchronize()
        s_ref = oracle.gather_sum(R, idx)
        oracle.apply_sparse_update(w, idx, s_ref, -0.00125, R)
        assert np.array_equal(bits(s.cpu().numpy()), bits(s_ref))
        assert np.array_equal(bits(wd.cpu().numpy()), bits(w))
        for a, b in zip(Rd, R):
            assert np.array_equal(bits(a.cpu().numpy()), bits(b))


# ---------------------------------------------------------------- whole steps on parameter sets

def _route(fused):
    """Test parameter -> GpuSet arguments: False / "3:<hint>" = the three separate calls."""
    if not fused:
        return dict(fused=False, hint="none")
    if fused.startswith("3:"):
        return dict(fused=False, hint=fused[2:])
    return dict(fused=True, hint=fused)


# The oracle's side of the large configurations (inputs, and after every step its outputs, weights and
# residuals) does not depend on the route under test: it is computed once per configuration and kept
# for the other routes, which saves the oracle's sorts (most of these tests' time) three times over.
_ORACLE_RUNS = {}


def _oracle_run(ps, steps, pool, W, r0, g_ids_fn, leader_fn, momentum, sets):
    w = wl.gen_weights(ps)
    sets = [wl.gen_gradient(ps, s) for s in range(pool)] if sets is None else sets
    r_ref = [np.zeros(ps.flat, np.float32) for _ in range(W)] if r0 is None else [x.copy() for x in r0]
    w_ref = w.copy()
    per_step = []
    for t in range(steps):
        lead = wl.leaders(ps, t, n_candidates=W) if leader_fn is None else leader_fn(t)
        ids = [wl.gradient_set_of(ps, p, t, pool) for p in range(W)] if g_ids_fn is None else g_ids_fn(t)
        g = [sets[i] if i is not None else sets[0] for i in ids]
        acc = [i is not None for i in ids]
        ref = oracle.step(w_ref, g, r_ref, ps.rows(), lead, float(ps.eps), float(ps.scale), accumulate_mask=acc,
                          momentum=1.0 if momentum is None else momentum)
        per_step.append((lead, ids, ref, w_ref.copy(), [x.copy() for x in r_ref]))
    return w, sets, per_step


def _run_steps(iwp, ps, steps, pool, W=None, r0=None, g_ids_fn=None, leader_fn=None, tag="", fused=False,
               momentum=None, sets=None, keep=None, leader_table=True):
    """keep: a name under which the oracle's run is kept for the other routes (only for calls whose
    inputs are fully determined by the configuration)."""
    W = ps.W if W is None else W
    if keep is not None and keep in _ORACLE_RUNS:
        w, sets, per_step = _ORACLE_RUNS[keep]
    else:
        w, sets, per_step = _oracle_run(ps, steps, pool, W, r0, g_ids_fn, leader_fn, momentum, sets)
        if keep is not None:
            _ORACLE_RUNS[keep] = (w, sets, per_step)
    gs = GpuSet(iwp, ps, w, sets, r_np=r0, W=W, **_route(fused))
    if momentum is not None:
        gs.plan.set_momentum(momentum)
    for t, (lead, ids, (idx_ref, val_ref, sum_ref, thr_ref), w_ref, r_ref) in enumerate(per_step):
        gs.step(ids, lead if leader_table else None)
        assert_step_equal(gs.download(), w_ref, r_ref, idx_ref, val_ref, sum_ref, thr_ref, ps.layers,
                          tag="%s step %d" % (tag, t))
    return gs


# fused: False = the three separate calls; otherwise the whole-step entry point with the named kind of
# threshold hint ("previous" = last step's records, the intended use; the others must not change a bit either)
ROUTES = pytest.mark.parametrize("fused", [False, "3:previous", "none", "previous"],
                                 ids=["three_calls", "three_calls_hinted", "whole_step", "whole_step_hinted"])
HINTS = pytest.mark.parametrize("fused", ["garbage", "high", "low"], ids=["hint_garbage", "hint_high", "hint_low"])


@ROUTES
def test_config1_tiny_mlp_all_steps(gpu_lib, fused):
    ps = wl.make_config(1)
    _run_steps(gpu_lib, ps, ps.steps, pool=4, tag="cfg1", fused=fused)


@ROUTES
def test_config1_packed_layout_misaligned_layers(gpu_lib, fused):
    ps = wl.make_config(1, align=1)
    _run_steps(gpu_lib, ps, 3, pool=4, tag="cfg1 packed", fused=fused)


@ROUTES
def test_custom_edge_set_segmented(gpu_lib, fused):
    """Ragged mix in one table: empty layer, k = 0 rows, n = 1, k = n, tile-boundary sizes."""
    sizes = [(300, 5), (0, 0), (1, 1), (TILE, 256), (64, 64), (1000, 0), (TILE + 1, 1), (777, 13),
             (2 * TILE - 1, 2 * TILE - 1), (5, 0), (40000, 625), (STILE + 3, 600), (3 * STILE, 3 * STILE - 1)]
    for align, start in ((1, 0), (1, 3), (4, 0), (64, 0)):
        ps = wl.custom_set(sizes, W=3, seed=80 + align + start, align=align, start=start, zero_frac=0.01)
        _run_steps(gpu_lib, ps, 3, pool=3, tag="edge align=%d start=%d" % (align, start), fused=fused)


@ROUTES
def test_leader_table_out_of_range_reads_as_worker_zero(gpu_lib, fused):
    ps = wl.custom_set([(5000, 80), (300, 5)], W=2, seed=91, align=4)
    bad = np.array([7, 0xFFFFFFFF], np.uint32)
    w = wl.gen_weights(ps)
    sets = [wl.gen_gradient(ps, s) for s in range(2)]
    gs = GpuSet(gpu_lib, ps, w, sets, **_route(fused))
    gs.step([0, 1], bad)
    r_ref = [np.zeros(ps.flat, np.float32) for _ in range(2)]
    ref = oracle.step(w, sets, r_ref, ps.rows(), np.zeros(2, np.uint32), float(ps.eps), float(ps.scale))
    assert_step_equal(gs.download(), w, r_ref, *ref, ps.layers, tag="bad leader")


@ROUTES
@pytest.mark.timeout(600)
def test_config3_resnet50_shaped(gpu_lib, fused):
    ps = wl.make_config(3)
    _run_steps(gpu_lib, ps, 3, pool=4, tag="cfg3", fused=fused, keep="cfg3")


# Configs 2 and 4 at full size, every route, over 12 and all 10 steps: tests/test_gpu_longrun.py.


@ROUTES
@pytest.mark.timeout(600)
def test_config5_scaled_local_plus_static_peers(gpu_lib, fused):
    """Config 5's structure at 1/50 of its length: one flat layer, a local worker
    that accumulates and leads, and 8 peers whose residuals are static (no gradient
    buffer): the pointer list is [local, peer 0..7]."""
    ps = wl.make_config(5, scale_down=50)
    W = 9
    peers = [wl.gen_gradient(ps, 100 + p) for p in range(8)]
    r0 = [np.zeros(ps.flat, np.float32)] + peers
    ps.W = 9
    _run_steps(gpu_lib, ps, 3, pool=2, W=W, r0=r0, tag="cfg5/50", fused=fused, keep="cfg5/50",
               g_ids_fn=lambda t: [t % 2] + [None] * 8, leader_fn=lambda t: np.zeros(1, np.uint32))


@ROUTES
@pytest.mark.timeout(600)
def test_config5_scaled_without_a_leader_table(gpu_lib, fused):
    """The same run with no leader table (NULL: worker 0 leads everything), which is how a single local worker
    calls the library; the whole-step entry point then launches no followers' pass at all (the one worker with
    a gradient has been through look 1 on every tile).  Also with a second layer that selects nothing, where
    that pass is still needed for the local worker."""
    ps = wl.make_config(5, scale_down=50)
    peers = [wl.gen_gradient(ps, 100 + p) for p in range(8)]
    r0 = [np.zeros(ps.flat, np.float32)] + peers
    ps.W = 9
    _run_steps(gpu_lib, ps, 3, pool=2, W=9, r0=r0, tag="cfg5/50 no leader table", fused=fused, keep="cfg5/50",
               g_ids_fn=lambda t: [t % 2] + [None] * 8, leader_fn=lambda t: np.zeros(1, np.uint32), leader_table=False)
    ps1 = wl.custom_set([(300000, 300), (4097, 65), (5000, 50)], W=1, seed=96, align=4)
    _run_steps(gpu_lib, ps1, 3, pool=2, W=1, tag="one worker, no leader table", fused=fused,
               leader_fn=lambda t: np.zeros(3, np.uint32), leader_table=False)
    ps2 = wl.custom_set([(300000, 300), (70000, 0), (5000, 50)], W=3, seed=97, align=4)
    _run_steps(gpu_lib, ps2, 3, pool=2, W=3, tag="k=0 layer, no leader table", fused=fused,
               g_ids_fn=lambda t: [t % 2, None, None], leader_fn=lambda t: np.zeros(3, np.uint32), leader_table=False)


@ROUTES
def test_staging_overflow_takes_the_raw_route(gpu_lib, fused):
    """Layers whose threshold bin is far larger than the staging capacity (nearly all
    scores equal, or all in one top-digit bin) next to ordinary layers."""
    n = 3 * STILE + 17
    ps = wl.custom_set([(n, 700), (n, 5000), (50000, 800), (n, 100)], W=2, seed=92, align=4)
    w = wl.gen_weights(ps)
    rng = np.random.default_rng(5)
    L0, L1, L2, L3 = ps.layers
    g0 = wl.gen_gradient(ps, 0)
    g1 = wl.gen_gradient(ps, 1)
    for g in (g0, g1):
        # layer 0: all scores identical; layer 1: identical top digit, different low bits; layer 3: zeros but a block
        g[L0.offset:L0.offset + n] = 0.5
        g[L1.offset:L1.offset + n] = (np.float32(1.0).view(np.uint32) + rng.integers(0, 4096, n).astype(np.uint32)).view(np.float32)
        g[L3.offset:L3.offset + n] = 0.0
        g[L3.offset + 1000:L3.offset + 1050] = rng.standard_normal(50).astype(np.float32)
    w[L0.offset:L0.offset + n] = 1.0
    w[L1.offset:L1.offset + n] = 1.0
    sets = [g0, g1]
    gs = GpuSet(gpu_lib, ps, w, sets, **_route(fused))
    w_ref = w.copy()
    r_ref = [np.zeros(ps.flat, np.float32) for _ in range(2)]
    for t in range(3):
        lead = wl.leaders(ps, t)
        ref = oracle.step(w_ref, sets, r_ref, ps.rows(), lead, 0.0, float(ps.scale))
        ps.eps = 0.0
        gs.step([0, 1], lead)
        assert_step_equal(gs.download(), w_ref, r_ref, *ref, ps.layers, tag="raw route step %d" % t)


@HINTS
def test_wrong_hints_change_nothing(gpu_lib, fused):
    """A threshold hint is only a shortcut: random records, records far above and far
    below the true thresholds all give the oracle's bytes (config 1 and a ragged set)."""
    ps = wl.make_config(1)
    _run_steps(gpu_lib, ps, 5, pool=4, tag="cfg1 " + fused, fused=fused)
    sizes = [(300, 5), (0, 0), (1, 1), (TILE, 256), (64, 64), (1000, 0), (TILE + 1, 1), (777, 13),
             (2 * TILE - 1, 2 * TILE - 1), (5, 0), (40000, 625), (STILE + 3, 600), (3 * STILE, 3 * STILE - 1)]
    ps = wl.custom_set(sizes, W=3, seed=97, align=1, start=1, zero_frac=0.01)
    _run_steps(gpu_lib, ps, 4, pool=3, tag="edge " + fused, fused=fused)


@HINTS
@pytest.mark.timeout(600)
def test_wrong_hints_config3(gpu_lib, fused):
    ps = wl.make_config(3)
    _run_steps(gpu_lib, ps, 3, pool=4, tag="cfg3 " + fused, fused=fused, keep="cfg3")


@ROUTES
def test_momentum_weighted_residual(gpu_lib, fused):
    """Eq. 3: r <- m * r + g on every accumulating worker (leaders, followers, ragged and
    misaligned layers), two roundings: one layer carries values for which a fused
    multiply-add would give a different residual."""
    m = float(np.float32(1 + 2.0 ** -12))
    sizes = [(300, 5), (TILE + 1, 70), (777, 13), (40000, 625), (STILE + 3, 600), (2 * TILE, 100)]
    for align, start in ((1, 3), (64, 0)):
        ps = wl.custom_set(sizes, W=3, seed=90 + align, align=align, start=start, zero_frac=0.01)
        sets = [wl.gen_gradient(ps, s) for s in range(3)]
        r0 = [np.zeros(ps.flat, np.float32) for _ in range(3)]
        L = ps.layers[-1]
        for p in range(3):                                     # m * r = 1 + 2^-11 + 2^-24 -> tie; g cancels the rounded product
            r0[p][L.offset:L.offset + L.n] = np.float32(1 + 2.0 ** -12)
            for g in sets:
                g[L.offset:L.offset + L.n:2] = np.float32(-(1 + 2.0 ** -11))
        _run_steps(gpu_lib, ps, 3, pool=3, W=3, r0=r0, sets=sets, tag="momentum fma", fused=fused, momentum=m,
                   g_ids_fn=lambda t: [(p + t) % 3 if p != 1 or t != 1 else None for p in range(3)])
    ps = wl.make_config(1)
    _run_steps(gpu_lib, ps, 4, pool=4, tag="cfg1 m=0.9", fused=fused, momentum=0.9)


@ROUTES
def test_most_workers(gpu_lib, fused):
    """32 workers, the limit of the interface, some of them without a gradient."""
    sizes = [(300, 5), (TILE + 1, 70), (40000, 625), (STILE + 3, 600)]
    ps = wl.custom_set(sizes, W=32, seed=95, align=64, zero_frac=0.01)
    rng = np.random.default_rng(7)
    r0 = [(rng.standard_t(3, ps.flat) * 1e-3).astype(np.float32) for _ in range(32)]
    _run_steps(gpu_lib, ps, 2, pool=3, W=32, r0=r0, tag="W=32", fused=fused,
               g_ids_fn=lambda t: [None if p in (4, 31) else (p + t) % 3 for p in range(32)])


def test_determinism_run_to_run(gpu_lib):
    ps = wl.make_config(1)
    outs = []
    for _ in range(2):
        w = wl.gen_weights(ps)
        sets = [wl.gen_gradient(ps, s) for s in range(2)]
        gs = GpuSet(gpu_lib, ps, w, sets)
        for t in range(3):
            gs.step([(p + t) % 2 for p in range(ps.W)], wl.leaders(ps, t))
        outs.append(gs.download())
    a, b = outs
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(bits(a["val"]), bits(b["val"]))
    assert np.array_equal(bits(a["w"]), bits(b["w"]))
    assert all(np.array_equal(bits(x), bits(y)) for x, y in zip(a["r"], b["r"]))


def test_argument_errors_launch_nothing(gpu_lib):
    import torch
    iwp = gpu_lib
    n = 1000
    w = torch.ones(n, device="cuda:0")
    g = torch.ones(n, device="cuda:0")
    r = torch.zeros(n, device="cuda:0")
    idx = torch.empty(n, dtype=torch.int32, device="cuda:0")
    val = torch.empty(n, device="cuda:0")
    ws = torch.empty(iwp.workspace_bytes(n, n), dtype=torch.uint8, device="cuda:0")
    for kwargs, code in [
        (dict(k=n + 1), iwp.IWP_EINVAL),
        (dict(k=5, eps=-1.0), iwp.IWP_EINVAL),
        (dict(k=5, eps=float("nan")), iwp.IWP_EINVAL),
        (dict(k=5, workspace=ws[:64]), iwp.IWP_EWORKSPACE),
        (dict(k=5, workspace=None), iwp.IWP_EWORKSPACE),
        (dict(k=5, idx_out=None), iwp.IWP_EINVAL),
    ]:
        a = dict(w=w, g=g, r=r, k=5, eps=1e-8, idx_out=idx, val_out=val, workspace=ws)
        a.update(kwargs)
        with pytest.raises(iwp.IwpError) as e:
            iwp.compress_layer(**a)
        assert e.value.code == code
    torch.cuda.synchronize()
    assert not r.any()                                   # nothing ran
    with pytest.raises(iwp.IwpError):
        iwp.gather_sum_at_indices([], idx, 5, val)
    with pytest.raises(iwp.IwpError):
        iwp.Plan([(0, 10, 11, 0)])                       # k > n
    with pytest.raises(iwp.IwpError):
        iwp.Plan([(0, 10, 1, 0), (5, 10, 1, 1)])         # overlap
    with pytest.raises(iwp.IwpError):
        iwp.Plan([(0, 10, 1, 0), (10, 10, 1, 5)])        # outputs not packed
