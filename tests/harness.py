"""Drivers shared by the GPU parity tests: run the same emulated step through the
HIP library (via the binding) and through the CPU oracle on the same bytes, and
compare every output bit for bit."""
from __future__ import annotations

import numpy as np


def bits(x):
    return np.ascontiguousarray(x, np.float32).view(np.uint32)


class GpuSet:
    """Device-resident state of one parameter set: weights, W residuals, a pool of
    gradient sets, plan and workspace.  All compute goes through ``iwp``: either the
    three separate calls (compress_segmented, gather_sum_at_indices,
    apply_sparse_update) or, with fused=True, the whole-step entry point."""

    def __init__(self, iwp, ps, w_np, grads_np, r_np=None, W=None, fused=False, hint="none", grads_dev=None):
        """grads_dev: gradient sets already on the device (shared between several sets), instead of grads_np."""
        import torch
        self.torch = torch
        self.iwp = iwp
        self.ps = ps
        self.W = ps.W if W is None else W
        dev = torch.device("cuda:0")
        self.w = torch.from_numpy(w_np).to(dev)
        self.grads = [torch.from_numpy(g).to(dev) for g in grads_np] if grads_dev is None else grads_dev
        if r_np is None:
            self.r = [torch.zeros(ps.flat, dtype=torch.float32, device=dev) for _ in range(self.W)]
        else:
            self.r = [torch.from_numpy(x).to(dev) for x in r_np]
        self.plan = iwp.Plan(ps.rows())
        assert self.plan.total_pairs == ps.K
        self.fused = fused
        # hint: "none" | "previous" (last step's thresholds, the intended use) | "garbage" | "high" | "low"
        self.hint_mode = hint
        self.hint = torch.zeros(len(ps.layers) * 3, dtype=torch.int32, device=dev)
        self.steps_done = 0
        ws_bytes = self.plan.step_workspace_bytes(self.W) if fused else self.plan.workspace_bytes
        self.ws = torch.empty(max(1, ws_bytes), dtype=torch.uint8, device=dev)
        K = max(1, ps.K)
        self.idx = torch.empty(K, dtype=torch.int32, device=dev)
        self.val = torch.empty(K, dtype=torch.float32, device=dev)
        self.sum = torch.empty(K, dtype=torch.float32, device=dev)
        self.thr = torch.zeros(len(ps.layers) * 3, dtype=torch.int32, device=dev)
        self.leader = torch.zeros(len(ps.layers), dtype=torch.int32, device=dev)

    def step(self, g_ids, leader_np, scale=None, hint_records=None):
        """g_ids[p]: index into the gradient pool for worker p, or None (no accumulate).
        leader_np: the chosen node per layer, or None to pass no leader table at all.
        hint_records: (layers, 3) uint32 records to pass as this step's threshold hint, whatever the set's
        hint mode says (a set with hint mode "none" ignores them)."""
        iwp, ps = self.iwp, self.ps
        self.idx.fill_(-1)
        self.val.fill_(float("nan"))
        lead = None                                # leader_np None: no leader table (worker 0 leads every layer)
        if leader_np is not None:
            self.leader.copy_(self.torch.from_numpy(leader_np.astype(np.int32)))
            lead = self.leader
        g = [None if i is None else self.grads[i] for i in g_ids]
        sc = float(ps.scale if scale is None else scale)
        hint = None
        if hint_records is not None and self.hint_mode != "none":
            self.hint.copy_(self.torch.from_numpy(np.ascontiguousarray(hint_records, np.uint32).view(np.int32).ravel()))
            hint = self.hint
        elif self.hint_mode == "previous" and self.steps_done > 0:
            self.hint.copy_(self.thr)
            hint = self.hint
        elif self.hint_mode == "garbage":
            self.hint.copy_(self.torch.randint(-2 ** 31, 2 ** 31 - 1, (self.hint.numel(),), dtype=self.torch.int64,
                                               device=self.hint.device).to(self.torch.int32))
            hint = self.hint
        elif self.hint_mode in ("high", "low") and self.steps_done > 0:
            # last step's keys moved up / down by a few top-digit bins
            key = self.thr.view(-1, 3)[:, 0].to(self.torch.int64)
            key = key + (5 << 19) if self.hint_mode == "high" else self.torch.clamp(key - (5 << 19), min=0)
            self.hint.view(-1, 3)[:, 0] = key.clamp(max=2 ** 31 - 1).to(self.torch.int32)
            hint = self.hint
        self.steps_done += 1
        if self.fused:
            self.sum.fill_(float("nan"))
            iwp.step_segmented(self.plan, self.w, g, self.r, lead, float(ps.eps), sc, self.idx, self.val,
                               self.sum, self.thr, self.ws, thr_hint=hint)
            self.torch.cuda.synchronize()
            return
        iwp.compress_segmented(self.plan, self.w, g, self.r, lead, float(ps.eps), self.idx, self.val,
                               self.thr, self.ws, thr_hint=hint)
        iwp.gather_sum_at_indices(self.r, self.idx, ps.K, self.sum)
        iwp.apply_sparse_update(self.w, self.idx, self.sum, ps.K, sc, self.r)
        self.torch.cuda.synchronize()

    def download(self):
        K = self.ps.K
        return dict(
            idx=self.idx.cpu().numpy().view(np.uint32)[:K],
            val=self.val.cpu().numpy()[:K],
            sum=self.sum.cpu().numpy()[:K],
            thr=self.thr.cpu().numpy().view(np.uint32).reshape(-1, 3),
            w=self.w.cpu().numpy(),
            r=[x.cpu().numpy() for x in self.r],
        )


class DeviceRef:
    """The oracle's state after a step, uploaded once, for bit-exact comparison on the device against
    several GpuSets (downloading 2 GB of residuals per set and step is what would dominate a long run)."""

    def __init__(self, torch, w_ref, r_ref, idx_ref, val_ref, sum_ref, thr_ref):
        up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to("cuda:0")
        self.torch = torch
        self.host = (w_ref, r_ref, idx_ref, val_ref, sum_ref, thr_ref)
        self.w = up(w_ref, np.int32)
        self.r = [up(x, np.int32) for x in r_ref]
        self.idx = up(idx_ref.astype(np.uint32), np.int32)
        self.val = up(val_ref, np.int32)
        self.sum = up(sum_ref, np.int32)

    def check(self, gs, layers, tag=""):
        t = self.torch
        K = self.idx.numel()
        i32 = lambda x: x.view(t.int32)
        same = (t.equal(gs.idx[:K], self.idx) and t.equal(i32(gs.val)[:K], self.val)
                and t.equal(i32(gs.sum)[:K], self.sum) and t.equal(i32(gs.w), self.w)
                and all(t.equal(i32(a), b) for a, b in zip(gs.r, self.r)))
        thr = gs.thr.cpu().numpy().view(np.uint32).reshape(-1, 3)
        same = same and all(np.array_equal(thr[j], self.host[5][j]) for j, L in enumerate(layers) if L.k)
        if not same:                                   # the host comparison names what differs
            assert_step_equal(gs.download(), *self.host, layers, tag=tag)
            raise AssertionError(tag + ": device comparison failed but the host comparison passed")


def assert_step_equal(got, w_ref, r_ref, idx_ref, val_ref, sum_ref, thr_ref, layers, tag=""):
    """Bit-exact comparison of every output of a step; reports the first layer that differs."""
    if not np.array_equal(got["idx"], idx_ref):
        for j, L in enumerate(layers):
            sl = slice(L.out_offset, L.out_offset + L.k)
            if not np.array_equal(got["idx"][sl], idx_ref[sl]):
                bad = np.nonzero(got["idx"][sl] != idx_ref[sl])[0][:5]
                raise AssertionError("%s idx differs in layer %d (n=%d k=%d) at %s: got %s want %s; thr got %s want %s"
                                     % (tag, j, L.n, L.k, bad, got["idx"][sl][bad], idx_ref[sl][bad],
                                        got["thr"][j], thr_ref[j]))
    assert np.array_equal(bits(got["val"]), bits(val_ref)), tag + " val"
    for j, L in enumerate(layers):
        if L.k:
            assert np.array_equal(got["thr"][j], thr_ref[j]), "%s thr of layer %d: %s vs %s" % (tag, j, got["thr"][j], thr_ref[j])
    assert np.array_equal(bits(got["sum"]), bits(sum_ref)), tag + " sum"
    assert np.array_equal(bits(got["w"]), bits(w_ref)), tag + " w"
    for p, (a, b) in enumerate(zip(got["r"], r_ref)):
        assert np.array_equal(bits(a), bits(b)), "%s residual of worker %d" % (tag, p)


class ThresholdSet:
    def __init__(self, iwp, ps, w_np, grads_np, r_np, n_lead, max_pairs):
        import torch
        self.torch, self.iwp, self.ps = torch, iwp, ps
        dev = "cuda:0"
        self.W = len(r_np)
        self.w = torch.from_numpy(w_np).to(dev)
        self.grads = [torch.from_numpy(g).to(dev) for g in grads_np]
        self.r = [torch.from_numpy(x).to(dev) for x in r_np]
        self.plan = iwp.Plan(ps.rows())
        self.n_lead, self.max_pairs = n_lead, max_pairs
        self.eps = 1e-8
        nl = len(ps.layers)
        self.mask = torch.full((max(4, self.plan.mask_bytes),), 0xAA, dtype=torch.uint8, device=dev)
        self.count = torch.full((nl + 2,), -1, dtype=torch.int32, device=dev)
        self.idx = torch.full((max_pairs + 8,), -1, dtype=torch.int32, device=dev)
        self.sum = torch.full((max_pairs + 8,), float("nan"), dtype=torch.float32, device=dev)
        self.ws = torch.empty(max(1, self.plan.threshold_workspace_bytes(self.W, n_lead, max_pairs)),
                              dtype=torch.uint8, device=dev)
        self.leaders = torch.zeros(nl * n_lead, dtype=torch.int32, device=dev)
        self.thr = torch.zeros(nl, dtype=torch.float32, device=dev)

    def step(self, g_ids, leaders_np, thr_np, scale, random=None):
        """random = (seed, step): with random gradient selection."""
        t = self.torch
        self.idx.fill_(-1)
        self.sum.fill_(float("nan"))
        self.leaders.copy_(t.from_numpy(np.ascontiguousarray(leaders_np, np.uint32).view(np.int32).ravel()))
        self.thr.copy_(t.from_numpy(np.ascontiguousarray(thr_np, np.float32)))
        g = [None if i is None else self.grads[i] for i in g_ids]
        if random is not None:
            self.iwp.step_threshold_random_segmented(self.plan, self.w, g, self.r, self.leaders, self.n_lead, self.thr,
                                                     int(random[0]), int(random[1]), self.eps, float(scale), self.mask,
                                                     self.count, self.idx, self.sum, self.max_pairs, self.ws)
        else:
            self.iwp.step_threshold_segmented(self.plan, self.w, g, self.r, self.leaders, self.n_lead, self.thr,
                                              self.eps, float(scale), self.mask, self.count, self.idx, self.sum,
                                              self.max_pairs, self.ws)
        t.cuda.synchronize()

    def step_layerwise(self, g_ids, leaders_np, alpha, beta, c, scale):
        """Thresholds derived on the device; afterwards self.stats (layers, n_lead, 2) float64 and
        self.thr_slots (layers, n_lead) float32 hold what each chosen node used."""
        t = self.torch
        nl = len(self.ps.layers)
        self.idx.fill_(-1)
        self.sum.fill_(float("nan"))
        self.leaders.copy_(t.from_numpy(np.ascontiguousarray(leaders_np, np.uint32).view(np.int32).ravel()))
        self.stats = t.full((nl, self.n_lead, 2), float("nan"), dtype=t.float64, device="cuda:0")
        self.thr_slots = t.full((nl, self.n_lead), 12345.0, dtype=t.float32, device="cuda:0")
        g = [None if i is None else self.grads[i] for i in g_ids]
        self.iwp.step_layerwise_segmented(self.plan, self.w, g, self.r, self.leaders, self.n_lead, alpha, beta, c,
                                          self.eps, float(scale), self.stats, self.thr_slots, self.mask, self.count,
                                          self.idx, self.sum, self.max_pairs, self.ws)
        t.cuda.synchronize()

    def download(self):
        nl = len(self.ps.layers)
        return dict(mask=self.mask.cpu().numpy()[:self.plan.mask_bytes],
                    count=self.count.cpu().numpy().view(np.uint32),
                    idx=self.idx.cpu().numpy().view(np.uint32), sum=self.sum.cpu().numpy(),
                    w=self.w.cpu().numpy(), r=[x.cpu().numpy() for x in self.r], nl=nl)
