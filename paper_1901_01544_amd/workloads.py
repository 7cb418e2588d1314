"""Seeded synthetic parameter sets shaped like the paper's workloads.

This module only *describes and generates inputs*: layer tables (offset, n, k),
weights, per-worker gradients and the leader draw.  It holds none of the
method's arithmetic (no accumulation, scoring, selection or update), imports
neither the HIP binding nor the CPU oracle, and is the one piece both sides of
a parity test share: the same bytes go to the GPU path and to the oracle.

The paper measures on AlexNet / ResNet-50 trained on ImageNet (Section 4.1,
Table 1).  Neither the dataset nor trained weights exist here, so the sets
below take the *shapes* of those models' parameter tensors and fill them with
seeded random values; they stand in for the paper's workloads.

Configs (ids follow the order in which the build's baseline file lists them):
  1 tiny MLP            6 tensors,     235 146 params, keep 1/64,   W=4
  2 AlexNet-shaped      16 tensors, 61 100 840 params, keep 1/64,   W=8
  3 ResNet-50-shaped   161 tensors, 25 557 032 params, keep 1/58.8, W=8
  4 many small layers 1000 tensors, ~1.2e8 params, keep U(0.5%,5%), W=8, tie-heavy
  5 one flat layer       1 tensor,  1.0e9 params, keep 0.1%, local + 8 peers
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_CHUNK = 1 << 22          # elements per independently seeded generation chunk
_GEN_THREADS = 8


@dataclass
class LayerSpec:
    name: str
    shape: Tuple[int, ...]
    fan_in: int
    n: int = 0
    k: int = 0
    offset: int = 0        # first element in the flat buffers
    out_offset: int = 0    # first (index, value) pair in the packed outputs
    grad_scale: float = 1.0
    block: Optional[Tuple[int, int]] = None   # (start, length): gradient is zero outside it


@dataclass
class ParamSet:
    cfg: int
    name: str
    layers: List[LayerSpec]
    W: int
    steps: int
    seed: int
    eps: float = 1e-8
    eta: float = 0.01
    weight_std: Optional[float] = None     # fixed std instead of He-normal
    grad_law: str = "student_t3"           # or "laplace"
    grad_b: float = 1e-4                   # Laplace scale
    zero_frac: float = 0.0                 # fraction of weights set exactly to 0
    flat: int = 0                          # flat buffer length (with padding)
    P: int = 0                             # sum of n
    K: int = 0                             # sum of k
    extra: dict = field(default_factory=dict)

    @property
    def scale(self) -> np.float32:
        """-(eta / W) computed once in double and rounded to fp32 once (Eq. 3 sign)."""
        return np.float32(-(self.eta / self.W))

    def rows(self):
        """(offset, n, k, out_offset) per layer, the form both C ABIs take."""
        return [(L.offset, L.n, L.k, L.out_offset) for L in self.layers]


# --------------------------------------------------------------------------
# keep ratio -> integer k (always in integers or in double, once, on the host)
# --------------------------------------------------------------------------

def k_ratio_64(n: int) -> int:
    """ceil(n / 64), the paper's 64x AlexNet ratio (Table 1) as a keep fraction."""
    return max(1, min(n, (n + 63) // 64))


def k_ratio_58_8(n: int) -> int:
    """ceil(n / 58.8) = ceil(10 n / 588), the paper's 58.8x ResNet-50 ratio (Table 1)."""
    return max(1, min(n, (10 * n + 587) // 588))


def k_from_keep(n: int, keep: float) -> int:
    return max(1, min(n, int(math.ceil(float(keep) * float(n)))))


# --------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------

def _prod(shape):
    p = 1
    for s in shape:
        p *= int(s)
    return p


def _mlp_shapes():
    out = []
    for i, (o, ins) in enumerate([(256, 784), (128, 256), (10, 128)]):
        out.append(LayerSpec("fc%d.weight" % i, (o, ins), ins))
        out.append(LayerSpec("fc%d.bias" % i, (o,), ins))
    return out


def _alexnet_shapes():
    convs = [(64, 3, 11, 11), (192, 64, 5, 5), (384, 192, 3, 3), (256, 384, 3, 3), (256, 256, 3, 3)]
    fcs = [(4096, 9216), (4096, 4096), (1000, 4096)]
    out = []
    for i, s in enumerate(convs):
        fi = s[1] * s[2] * s[3]
        out.append(LayerSpec("conv%d.weight" % i, s, fi))
        out.append(LayerSpec("conv%d.bias" % i, (s[0],), fi))
    for i, s in enumerate(fcs):
        out.append(LayerSpec("fc%d.weight" % i, s, s[1]))
        out.append(LayerSpec("fc%d.bias" % i, (s[0],), s[1]))
    return out


def _resnet50_shapes():
    out = []

    def conv_bn(name, o, i, kh):
        out.append(LayerSpec(name + ".weight", (o, i, kh, kh), i * kh * kh))
        out.append(LayerSpec(name + ".bn.gamma", (o,), o))
        out.append(LayerSpec(name + ".bn.beta", (o,), o))

    conv_bn("stem", 64, 3, 7)
    inplanes = 64
    for si, (blocks, width) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512])):
        for b in range(blocks):
            pre = "layer%d.%d" % (si + 1, b)
            conv_bn(pre + ".conv1", width, inplanes, 1)
            conv_bn(pre + ".conv2", width, width, 3)
            conv_bn(pre + ".conv3", width * 4, width, 1)
            if b == 0:
                conv_bn(pre + ".downsample", width * 4, inplanes, 1)
            inplanes = width * 4
    out.append(LayerSpec("fc.weight", (1000, 2048), 2048))
    out.append(LayerSpec("fc.bias", (1000,), 2048))
    return out


def _layout(layers: List[LayerSpec], align: int, start: int = 0):
    """Assign flat offsets (each a multiple of ``align`` elements past ``start``)
    and packed output offsets (prefix sums of k).  Padding belongs to no layer."""
    off = start
    oo = 0
    for L in layers:
        L.n = _prod(L.shape)
        off = start + ((off - start + align - 1) // align) * align
        L.offset = off
        L.out_offset = oo
        off += L.n
        oo += L.k
    return off, oo


def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(k) for k in key])))


def make_config(cfg: int, align: int = 64, scale_down: int = 1, seed: Optional[int] = None) -> ParamSet:
    """Build the layer table of config ``cfg`` (1..5).

    ``align``: layer offsets are multiples of this many elements (1 = packed,
    exercising the misaligned paths).  ``scale_down`` > 1 shrinks config 4's
    tensor count and config 5's length for tests; the named configs themselves
    are ``scale_down == 1``.
    """
    if cfg == 1:
        ps = ParamSet(1, "tiny_mlp", _mlp_shapes(), W=4, steps=10, seed=1, zero_frac=1e-3)
        rule = k_ratio_64
    elif cfg == 2:
        ps = ParamSet(2, "alexnet_shaped", _alexnet_shapes(), W=8, steps=100, seed=2)
        rule = k_ratio_64
    elif cfg == 3:
        ps = ParamSet(3, "resnet50_shaped", _resnet50_shapes(), W=8, steps=100, seed=3)
        rule = k_ratio_58_8
    elif cfg == 4:
        ps = ParamSet(4, "many_small", [], W=8, steps=10, seed=4)
        rule = None
    elif cfg == 5:
        n = 1_000_000_000 // scale_down
        ps = ParamSet(5, "single_flat", [LayerSpec("flat", (n,), 1)], W=8, steps=20, seed=5,
                      weight_std=0.02, grad_law="laplace", grad_b=1e-4)
        rule = lambda m: k_from_keep(m, 0.001)  # noqa: E731
    else:
        raise ValueError("config id must be 1..5")
    if seed is not None:
        ps.seed = seed

    if cfg == 4:
        rg = _rng(ps.seed, 10)
        L = 1000 // scale_down
        sizes = np.rint(np.exp(rg.uniform(math.log(256.0), math.log(float(1 << 20)), L))).astype(np.int64)
        keeps = rg.uniform(0.005, 0.05, L)
        concentrated = rg.random(L) < 0.05
        starts = rg.random(L)
        for j in range(L):
            n = int(sizes[j])
            spec = LayerSpec("t%03d" % j, (n,), 256)
            spec.k = k_from_keep(n, float(keeps[j]))
            if concentrated[j]:
                blen = int(math.ceil(0.01 * n))
                spec.block = (int(starts[j] * (n - blen)), blen)
            ps.layers.append(spec)
            ps.extra.setdefault("keep", []).append(float(keeps[j]))
    else:
        for L in ps.layers:
            L.k = rule(_prod(L.shape))

    ps.flat, ps.K = _layout(ps.layers, align)
    ps.P = sum(L.n for L in ps.layers)
    if ps.grad_law == "student_t3":
        rs = _rng(ps.seed, 2)
        for L in ps.layers:
            L.grad_scale = float(rs.lognormal(math.log(1e-3), 1.0))
    return ps


def custom_set(sizes_and_k: Sequence[Tuple[int, int]], W: int, seed: int, align: int = 1,
               start: int = 0, zero_frac: float = 0.0) -> ParamSet:
    """An ad-hoc set for edge-case tests: [(n, k), ...], He-normal with fan_in 256."""
    layers = []
    for j, (n, k) in enumerate(sizes_and_k):
        L = LayerSpec("e%d" % j, (int(n),), 256)
        L.k = int(k)
        layers.append(L)
    ps = ParamSet(0, "custom", layers, W=W, steps=1, seed=seed, zero_frac=zero_frac)
    ps.flat, ps.K = _layout(ps.layers, align, start)
    ps.P = sum(L.n for L in ps.layers)
    rs = _rng(seed, 2)
    for L in ps.layers:
        L.grad_scale = float(rs.lognormal(math.log(1e-3), 1.0))
    return ps


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------

def _chunks(n):
    return [(c, c * _CHUNK, min(n, (c + 1) * _CHUNK)) for c in range((n + _CHUNK - 1) // _CHUNK)]


def _run(jobs):
    if len(jobs) <= 1:
        for f in jobs:
            f()
        return
    with ThreadPoolExecutor(_GEN_THREADS) as ex:
        for fut in [ex.submit(f) for f in jobs]:
            fut.result()


def gen_weights(ps: ParamSet) -> np.ndarray:
    """Flat fp32 weights: N(0, sqrt(2/fan_in)) per tensor (or N(0, weight_std)),
    ``zero_frac`` of the elements set exactly to +0; padding is +0."""
    w = np.zeros(ps.flat, np.float32)
    jobs = []
    for j, L in enumerate(ps.layers):
        std = ps.weight_std if ps.weight_std is not None else math.sqrt(2.0 / L.fan_in)
        for (c, a, b) in _chunks(L.n):
            def job(j=j, L=L, c=c, a=a, b=b, std=std):
                rg = _rng(ps.seed, 0, j, c)
                x = rg.standard_normal(b - a, dtype=np.float32) * np.float32(std)
                if ps.zero_frac > 0:
                    x[rg.random(b - a) < ps.zero_frac] = 0.0
                w[L.offset + a:L.offset + b] = x
            jobs.append(job)
    _run(jobs)
    return w


def gen_gradient(ps: ParamSet, set_id: int) -> np.ndarray:
    """One flat fp32 gradient set (a member of the pool that workers rotate
    through): Student-t(nu=3) times the tensor's lognormal scale, or
    Laplace(0, grad_b); zero outside a tensor's block if it has one."""
    g = np.zeros(ps.flat, np.float32)
    jobs = []
    for j, L in enumerate(ps.layers):
        for (c, a, b) in _chunks(L.n):
            def job(j=j, L=L, c=c, a=a, b=b):
                rg = _rng(ps.seed, 1, set_id, j, c)
                if ps.grad_law == "laplace":
                    x = rg.laplace(0.0, ps.grad_b, b - a).astype(np.float32)
                else:
                    x = (rg.standard_t(3.0, b - a) * L.grad_scale).astype(np.float32)
                if L.block is not None:
                    s, ln = L.block
                    keep = np.zeros(b - a, bool)
                    lo, hi = max(a, s), min(b, s + ln)
                    if hi > lo:
                        keep[lo - a:hi - a] = True
                    x[~keep] = 0.0
                g[L.offset + a:L.offset + b] = x
            jobs.append(job)
    _run(jobs)
    return g


def gradient_set_of(ps: ParamSet, worker: int, step: int, pool: int) -> int:
    """Which pool member worker ``worker`` receives at step ``step``."""
    return (worker + step) % pool


def _splitmix64(x: int) -> int:
    m = (1 << 64) - 1
    x = (x + 0x9E3779B97F4A7C15) & m
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def leaders(ps: ParamSet, step: int, n_candidates: Optional[int] = None) -> np.ndarray:
    """The randomly chosen node of Alg. 1 for every layer at ``step``:
    splitmix64(seed xor (step * L + j)) mod W.  An input to both sides."""
    W = ps.W if n_candidates is None else n_candidates
    L = len(ps.layers)
    return np.array([_splitmix64(ps.seed ^ (step * L + j)) % W for j in range(L)], np.uint32)


def chosen_nodes(ps: ParamSet, step: int, n_lead: int, n_candidates: Optional[int] = None) -> np.ndarray:
    """Threshold mode: the n_lead randomly chosen nodes of Alg. 1 for every layer at
    ``step``, shape (layers, n_lead); slot 0 is ``leaders``; a node may come up twice."""
    W = ps.W if n_candidates is None else n_candidates
    L = len(ps.layers)
    return np.array([[_splitmix64((ps.seed ^ (step * L + j)) + 0x51ED270B * q) % W for q in range(n_lead)]
                     for j in range(L)], np.uint32).reshape(L, n_lead)


# --------------------------------------------------------------------------
# device-side generation for the 1e9-element config (host generation of eleven
# 4 GB buffers would take minutes); same laws, torch's seeded generator
# --------------------------------------------------------------------------

def device_generator(ps: ParamSet, stream_id: int, device="cuda:0"):
    """A torch generator on ``device`` seeded from (set seed, stream_id)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(ps.seed) * 1000003 + int(stream_id))
    return gen


def gen_weights_device(ps: ParamSet, device="cuda:0"):
    """Flat fp32 weights N(0, weight_std) drawn on the device (config 5)."""
    import torch
    assert ps.weight_std is not None
    return torch.empty(ps.flat, device=device).normal_(0.0, ps.weight_std, generator=device_generator(ps, 0, device))


def gen_laplace_device(ps: ParamSet, stream_id: int, device="cuda:0"):
    """Flat fp32 Laplace(0, grad_b) buffer drawn on the device by inverse CDF:
    stream_id 1.. = gradient sets, 100.. = peer residuals."""
    import torch
    u = torch.empty(ps.flat, device=device).uniform_(-0.5, 0.5, generator=device_generator(ps, stream_id, device))
    x = torch.log1p(-2.0 * u.abs())
    x.mul_(torch.sign(u)).mul_(-ps.grad_b)
    return x
