"""compress_segmented_static (the entry point that allocates nothing: its kernels work in a static
device buffer inside the library) against compress_segmented on identical state, through the C ABI,
bit for bit: two calls in a row, the second on a smaller table, so the second call meets the first
call's leftovers in the shared buffer."""
import numpy as np
import pytest

from paper_1901_01544_amd import workloads as wl
from harness import bits

pytestmark = pytest.mark.gpu
TILE = 4096
STILE = 8 * TILE
EPS = 1e-8


def _both(iwp, torch, ps, seed, hint_from=None):
    """One compression of the set through both entry points; returns the static call's threshold records."""
    dev = "cuda:0"
    W = ps.W
    rng = np.random.default_rng(seed)
    w = wl.gen_weights(ps)
    g = [wl.gen_gradient(ps, s) for s in range(W)]
    r0 = [(rng.standard_t(3, ps.flat) * 1e-3).astype(np.float32) for _ in range(W)]
    lead = wl.leaders(ps, seed).astype(np.int32)
    plan = iwp.Plan(ps.rows())
    assert plan.workspace_bytes <= iwp.IWP_STATIC_SCRATCH_BYTES
    K = max(1, ps.K)
    nl = len(ps.layers)
    out = []
    for static in (False, True):
        wd = torch.from_numpy(w).to(dev)
        gd = [torch.from_numpy(x).to(dev) for x in g]
        gd[W - 1] = None if W > 2 else gd[W - 1]                  # one worker without a gradient
        rd = [torch.from_numpy(x).to(dev) for x in r0]
        ld = torch.from_numpy(lead).to(dev)
        idx = torch.full((K,), -1, dtype=torch.int32, device=dev)
        val = torch.full((K,), float("nan"), dtype=torch.float32, device=dev)
        thr = torch.zeros(nl * 3, dtype=torch.int32, device=dev)
        hint = None if hint_from is None else torch.from_numpy(hint_from.view(np.int32).ravel().copy()).to(dev)
        if static:
            iwp.compress_segmented_static(plan, wd, gd, rd, ld, EPS, idx, val, thr, thr_hint=hint)
        else:
            ws = torch.empty(max(1, plan.workspace_bytes), dtype=torch.uint8, device=dev)
            iwp.compress_segmented(plan, wd, gd, rd, ld, EPS, idx, val, thr, ws, thr_hint=hint)
        torch.cuda.synchronize()
        out.append(dict(idx=idx.cpu().numpy(), val=val.cpu().numpy(), thr=thr.cpu().numpy().view(np.uint32).reshape(-1, 3),
                        r=[x.cpu().numpy() for x in rd], w=wd.cpu().numpy()))
    a, b = out
    assert np.array_equal(a["idx"], b["idx"]) and (a["idx"][:ps.K] >= 0).all()
    assert np.array_equal(bits(a["val"]), bits(b["val"]))
    for j, L in enumerate(ps.layers):
        if L.k:
            assert np.array_equal(a["thr"][j], b["thr"][j]), j
    assert np.array_equal(bits(a["w"]), bits(b["w"]))
    for x, y in zip(a["r"], b["r"]):
        assert np.array_equal(bits(x), bits(y))
    return b["thr"]


def test_static_scratch_entry_point_matches_compress_segmented(gpu_lib):
    import torch
    big = [(300, 5), (0, 0), (TILE, 256), (1000, 0), (TILE + 1, 1), (3 * STILE + 17, 3000), (2 * TILE - 1, 2 * TILE - 1),
           (40000, 625), (STILE + 3, 600), (5 * STILE, 9000), (64, 64)]
    ps1 = wl.custom_set(big, W=3, seed=501, align=4, zero_frac=0.01)
    thr1 = _both(gpu_lib, torch, ps1, seed=1)
    # second call, smaller input: fewer and shorter layers land on the first call's leftovers
    small = [(777, 13), (TILE + 77, 300), (STILE - 1, 100)]
    ps2 = wl.custom_set(small, W=2, seed=502, align=1, start=1, zero_frac=0.01)
    _both(gpu_lib, torch, ps2, seed=2)
    # and the first table again, now with a threshold hint (the first look stages into the shared buffer)
    _both(gpu_lib, torch, ps1, seed=1, hint_from=thr1)


def test_static_scratch_rejects_a_plan_that_does_not_fit(gpu_lib):
    import torch
    iwp = gpu_lib
    n = 200_000_000
    plan = iwp.Plan([(0, n, n // 10, 0)])
    assert plan.workspace_bytes > iwp.IWP_STATIC_SCRATCH_BYTES
    fake = torch.zeros(16, device="cuda:0")              # never touched: the size check comes before any launch
    with pytest.raises(iwp.IwpError) as e:
        iwp.compress_segmented_static(plan, fake, [fake], [fake], None, EPS, fake, fake, None)
    assert e.value.code == iwp.IWP_ESCRATCH
    torch.cuda.synchronize()
    assert not fake.any()
