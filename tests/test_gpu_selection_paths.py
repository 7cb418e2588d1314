"""GPU parity for the branches of the selection that ordinary data rarely takes, each forced on purpose and
compared with the CPU oracle bit for bit through the C ABI:
  * the staging bin guessed from a sample of the layer (no hint given), on layouts that fool a sample:
    sorted scores, all of the mass in a block between the sampled runs, a pattern with the sample's period;
  * first-digit histograms kept in several copies (layers of more than 512 tiles);
  * tiles whose keys are all equal, above, at and below the threshold (recorded as one entry);
  * slots that overflow in the first look and are filled again by the second (hints far too low)."""
import numpy as np
import pytest

import oracle
from paper_1901_01544_amd import workloads as wl
from harness import GpuSet, assert_step_equal, bits

pytestmark = pytest.mark.gpu
TILE = 4096
STILE = 8 * TILE
EPS = 1e-8


def _compress(iwp, torch, w, g, r, k, eps=EPS):
    n = r.size
    dev = "cuda:0"
    wd, gd, rd = (torch.from_numpy(a).to(dev) for a in (w, g, r))
    idx = torch.full((max(1, k),), -1, dtype=torch.int32, device=dev)
    val = torch.full((max(1, k),), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty(iwp.workspace_bytes(n, k), dtype=torch.uint8, device=dev)
    iwp.compress_layer(wd, gd, rd, k, eps, idx, val, ws, n=n)
    torch.cuda.synchronize()
    return idx.cpu().numpy().view(np.uint32)[:k], val.cpu().numpy()[:k], rd.cpu().numpy()


def _check(iwp, torch, w, g, r, k, tag, eps=EPS):
    r_ref = r.copy()
    idx_ref, val_ref, _ = oracle.compress_layer(w, g, r_ref, k, eps)
    idx, val, r_after = _compress(iwp, torch, w, g, r, k, eps)
    assert np.array_equal(bits(r_after), bits(r_ref)), tag + " residual"
    assert np.array_equal(idx, idx_ref), "%s idx: got %s want %s" % (tag, idx[:8], idx_ref[:8])
    assert np.array_equal(bits(val), bits(val_ref)), tag + " val"


@pytest.mark.parametrize("n", [70_001, 300_007, 1_200_003])
def test_sampled_staging_bin_on_layouts_that_fool_a_sample(gpu_lib, n):
    """compress_layer takes no hint, so the first look's staging bin comes from the sample (up to 256 evenly
    spaced runs of 256 elements).  Whatever the sample suggests, the result is the oracle's."""
    import torch
    rng = np.random.default_rng(n)
    one = np.ones(n, np.float32)
    z = np.zeros(n, np.float32)
    k = max(1, n // 64)
    base = (np.abs(rng.standard_t(3, n)) * 1e-3 + 1e-6).astype(np.float32)
    # sorted ascending / descending: the kept elements sit at one end
    _check(gpu_lib, torch, one, z, np.sort(base), k, "sorted ascending n=%d" % n)
    _check(gpu_lib, torch, one, z, np.sort(base)[::-1].copy(), k, "sorted descending n=%d" % n)
    # everything that matters inside one block that no sampled run touches: the sample sees only tiny scores
    # the library's sampling plan (if it changes, these cases still check exactness, only less pointedly)
    runs_total = (n + 255) // 256
    runs = min(runs_total, min(256, max(16, (256 * n // k + 255) // 256)))
    sampled = {(i * runs_total) // runs for i in range(runs)}
    free = [q for q in range(1, runs_total - 1) if q not in sampled and q + 1 not in sampled]
    r = (base * np.float32(1e-4)).astype(np.float32)
    if free:
        q = free[len(free) // 2]
        r[q * 256:(q + 2) * 256] = (1.0 + rng.random(512)).astype(np.float32)
    _check(gpu_lib, torch, one, z, r, k, "block between the runs n=%d" % n)
    _check(gpu_lib, torch, one, z, r, 300, "block between the runs, k inside the block n=%d" % n)
    # a pattern with the sample's own period: large scores exactly where the runs start
    r = (base * np.float32(1e-3)).astype(np.float32)
    for s in sorted(sampled):
        r[s * 256:s * 256 + 64] = (5.0 + rng.random(min(64, n - s * 256))).astype(np.float32)[:max(0, n - s * 256)]
    _check(gpu_lib, torch, one, z, r, k, "period of the sample n=%d" % n)
    # and the complement: large scores everywhere but in the sampled runs
    r = (1.0 + rng.random(n)).astype(np.float32)
    for s in sorted(sampled):
        r[s * 256:(s + 1) * 256] = base[s * 256:(s + 1) * 256] * np.float32(1e-3)
    _check(gpu_lib, torch, one, z, r, k, "sample sees only the small n=%d" % n)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n", [513 * TILE + 5, 1100 * TILE + 1, 2200 * TILE - 3])
def test_layers_with_several_first_digit_histogram_copies(gpu_lib, n):
    """More than 512 tiles: the first look's workgroups flush into 2, 4 and 8 copies of the histogram."""
    import torch
    rng = np.random.default_rng(n)
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    r = (rng.standard_t(3, n) * 2e-3).astype(np.float32)
    for k in (n // 64, 1, n // 3):
        _check(gpu_lib, torch, w, g, r, k, "n=%d k=%d" % (n, k))


@pytest.mark.timeout(600)
def test_table_between_the_two_cache_policy_bounds(gpu_lib):
    """The first look keeps the weights and the residual it writes cacheable on small tables, only the weights
    on medium ones, nothing on large ones (three instantiations of the same kernel).  The configurations cover
    the small and the large variant; this layer of 7000 tiles (109 MiB per buffer) takes the middle one.  Two
    compressions in a row, the second on the residual the first left."""
    import torch
    n = 7000 * TILE + 11
    rng = np.random.default_rng(7000)
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    r = np.zeros(n, np.float32)
    k = n // 64
    r_ref = r.copy()
    for rep in range(2):
        idx_ref, val_ref, _ = oracle.compress_layer(w, g, r_ref, k, EPS)
        idx, val, r = _compress(gpu_lib, torch, w, g, r, k)
        # what compress_layer leaves: the accumulated residual (nothing is cleared by this call)
        assert np.array_equal(bits(r), bits(r_ref)), "residual, call %d" % rep
        assert np.array_equal(idx, idx_ref) and np.array_equal(bits(val), bits(val_ref)), "pairs, call %d" % rep


def test_tiles_of_equal_keys_above_at_and_below_the_threshold(gpu_lib):
    import torch
    rng = np.random.default_rng(77)
    n = 6 * STILE + 1234
    one = np.ones(n, np.float32)
    z = np.zeros(n, np.float32)
    # a run of equal large scores over 3 tiles and a bit, a run of equal medium scores over 5 tiles, zeros
    # elsewhere except a sprinkle of distinct values
    r = z.copy()
    a0, a1 = TILE + 100, 4 * TILE + 300
    b0, b1 = 2 * STILE - 7, 2 * STILE + 5 * TILE + 11
    r[a0:a1] = -8.0
    r[b0:b1] = 0.5
    sprinkle = rng.choice(n, 2000, replace=False)
    sprinkle = sprinkle[((sprinkle < a0) | (sprinkle >= a1)) & ((sprinkle < b0) | (sprinkle >= b1))]
    r[sprinkle] = (rng.standard_normal(sprinkle.size) * 0.1).astype(np.float32)
    na, nb = a1 - a0, b1 - b0
    for k in (na - 5, na, na + 1,                      # the cut inside / at the end of / just after the large run
              na + nb // 2, na + TILE, na + nb,        # inside the medium run, on tile boundaries of it
              na + nb + 1000, n - 10, n):              # into the sprinkle and the zeros
        _check(gpu_lib, torch, one, z, r, k, "equal runs k=%d" % k, eps=0.0)
    # all zeros with -0.0 mixed in: ties at score 0, the values keep their sign bits
    r0 = z.copy()
    r0[::3] = -0.0
    _check(gpu_lib, torch, one, z, r0, 5 * TILE + 17, "signed zeros", eps=0.0)


@pytest.mark.parametrize("route", ["whole_step", "three_calls"])
def test_hints_far_too_low_overflow_the_first_look(gpu_lib, route):
    """A hint of a few bins above zero makes the first look copy out nearly everything: every slot overflows,
    the second look fills them again from the real bin.  Same bytes as without hints."""
    sizes = [(3 * STILE + 17, 900), (TILE + 1, 70), (40000, 625), (5 * STILE, 20000), (300, 5)]
    ps = wl.custom_set(sizes, W=3, seed=123, align=64, zero_frac=0.01)
    w = wl.gen_weights(ps)
    sets = [wl.gen_gradient(ps, s) for s in range(3)]
    gs = GpuSet(gpu_lib, ps, w, sets, fused=route == "whole_step", hint="previous")
    w_ref = w.copy()
    r_ref = [np.zeros(ps.flat, np.float32) for _ in range(3)]
    for t in range(4):
        lead = wl.leaders(ps, t)
        ids = [(p + t) % 3 for p in range(3)]
        ref = oracle.step(w_ref, [sets[i] for i in ids], r_ref, ps.rows(), lead, float(ps.eps), float(ps.scale))
        low = np.zeros((len(ps.layers), 3), np.uint32)
        low[:, 0] = (3 + t) << 19                                    # top-digit bin 3 .. 6: denormal-range scores
        gs.step(ids, lead, hint_records=low)
        assert_step_equal(gs.download(), w_ref, r_ref, *ref, ps.layers, tag="low hints %s step %d" % (route, t))
