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

    def __init__(self, iwp, ps, w_np, grads_np, r_np=None, W=None, fused=False, hint="none"):
        import torch
        self.torch = torch
        self.iwp = iwp
        self.ps = ps
        self.W = ps.W if W is None else W
        dev = torch.device("cuda:0")
        self.w = torch.from_numpy(w_np).to(dev)
        self.grads = [torch.from_numpy(g).to(dev) for g in grads_np]
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

    def step(self, g_ids, leader_np, scale=None):
        """g_ids[p]: index into the gradient pool for worker p, or None (no accumulate)."""
        iwp, ps = self.iwp, self.ps
        self.idx.fill_(-1)
        self.val.fill_(float("nan"))
        self.leader.copy_(self.torch.from_numpy(leader_np.astype(np.int32)))
        g = [None if i is None else self.grads[i] for i in g_ids]
        sc = float(ps.scale if scale is None else scale)
        hint = None
        if self.hint_mode == "previous" and self.steps_done > 0:
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
            iwp.step_segmented(self.plan, self.w, g, self.r, self.leader, float(ps.eps), sc, self.idx, self.val,
                               self.sum, self.thr, self.ws, thr_hint=hint)
            self.torch.cuda.synchronize()
            return
        iwp.compress_segmented(self.plan, self.w, g, self.r, self.leader, float(ps.eps), self.idx, self.val,
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
