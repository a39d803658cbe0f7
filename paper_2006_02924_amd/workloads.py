"""Seeded synthetic worker gradients for the Adasum tree combiner.

This module only *makes inputs*: layer-size tables shaped like the parameter
tensors of the networks the paper trains (ResNet-50 and BERT-Large, Section 5)
and random per-worker gradients with a controlled per-layer correlation.  It
holds none of the combiner's arithmetic and is shared by the tests (which feed
the same stored values to the CPU oracle and to the HIP library) and by
``bench.py``.

Every gradient is a flat "fused" buffer of ``N`` elements plus one table of
layer boundaries that is the same for all workers, which is the layout the
paper's tensor-fusion bookkeeping describes (Section 4.4.3).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Sequence

import torch


# ----------------------------------------------------------------------------
# layer-size tables
# ----------------------------------------------------------------------------

def resnet50_layer_sizes() -> List[int]:
    """Element counts of ResNet-50's parameter tensors in network order.

    161 tensors, 25 557 032 elements: stem 7x7 conv + BN, four stages of
    [3, 4, 6, 3] bottleneck blocks (1x1, 3x3, 1x1 convs, each followed by BN
    gamma/beta; the first block of a stage has a 1x1 downsample conv + BN),
    then the 1000x2048 classifier and its bias.
    """
    sizes = [64 * 3 * 7 * 7, 64, 64]
    fan_in = 64
    for width, blocks in zip((64, 128, 256, 512), (3, 4, 6, 3)):
        for b in range(blocks):
            sizes += [width * fan_in, width, width]
            sizes += [width * width * 9, width, width]
            sizes += [4 * width * width, 4 * width, 4 * width]
            if b == 0:
                sizes += [4 * width * fan_in, 4 * width, 4 * width]
            fan_in = 4 * width
    sizes += [1000 * 2048, 1000]
    return sizes


def bert_large_layer_sizes() -> List[int]:
    """Element counts of BERT-Large's parameter tensors in network order.

    391 tensors, 335 141 888 elements: word (30522x1024), position (512x1024)
    and token-type (2x1024) embeddings, embedding LayerNorm; 24 encoder layers
    of Q/K/V/O weights and biases, attention LayerNorm, the two feed-forward
    matrices (1024x4096, 4096x1024) with biases, output LayerNorm; pooler.
    """
    h, f = 1024, 4096
    sizes = [30522 * h, 512 * h, 2 * h, h, h]
    for _ in range(24):
        sizes += [h * h, h] * 4
        sizes += [h, h]
        sizes += [h * f, f, f * h, h]
        sizes += [h, h]
    sizes += [h * h, h]
    return sizes


def offsets_from_sizes(sizes: Sequence[int]) -> List[int]:
    """Prefix sums: ``offsets[l] .. offsets[l+1]`` is layer ``l`` (element units)."""
    offs = [0]
    for s in sizes:
        offs.append(offs[-1] + int(s))
    return offs


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    """K flat gradient buffers that share one layer-boundary table."""
    name: str
    K: int
    dtype: torch.dtype
    layer_offsets: List[int]
    grads: List[torch.Tensor]
    #: per-layer recipe notes (correlation, scale, kind) for tests that need them
    meta: Dict[str, list] = field(default_factory=dict)

    @property
    def N(self) -> int:
        return self.layer_offsets[-1]

    @property
    def n_layers(self) -> int:
        return len(self.layer_offsets) - 1

    @property
    def input_bytes(self) -> int:
        return self.K * self.N * self.grads[0].element_size() if self.grads else 0


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _host_gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def correlated_gaussian(sizes: Sequence[int], K: int, *, dtype=torch.float32,
                        device="cpu", seed: int = 0, corr=None, scale=None,
                        name: str = "custom") -> Workload:
    """``g_i = scale_l * (a_l * c + sqrt(1 - a_l^2) * n_i)`` per layer ``l``.

    ``c`` (shared by all workers) and ``n_i`` (one per worker) are N(0,1) per
    element, so two workers' gradients of a layer have correlation ``a_l^2``.
    ``corr``/``scale`` are a float, a per-layer sequence, or None; None draws
    ``a_l ~ U(0,1)`` (``scale``: 1).  The arithmetic is done in fp32 and the
    result is rounded to ``dtype`` (round-to-nearest-even for bf16).

    Draw order: ``c`` for the whole fused buffer (N values), then ``n_0``,
    ``n_1``, ... (N values each); ``g_i = c * (a_l scale_l) + n_i * (sqrt(1 -
    a_l^2) scale_l)`` element by element.  The per-layer parameters come from a
    separate host generator so that they do not depend on the device.
    """
    L = len(sizes)
    hg = _host_gen(seed)
    if corr is None:
        corr_l = torch.rand(L, generator=hg, dtype=torch.float64).tolist()
    elif isinstance(corr, (int, float)):
        corr_l = [float(corr)] * L
    else:
        corr_l = [float(a) for a in corr]
    if scale is None:
        scale_l = [1.0] * L
    elif isinstance(scale, (int, float)):
        scale_l = [float(scale)] * L
    else:
        scale_l = [float(s) for s in scale]
    offs = offsets_from_sizes(sizes)
    N = offs[-1]
    dg = _gen(device, seed)
    # per-element multipliers of the shared and the private component
    reps = torch.tensor([int(x) for x in sizes], dtype=torch.int64)
    coef_c = torch.tensor([a * sc for a, sc in zip(corr_l, scale_l)], dtype=torch.float32)
    coef_n = torch.tensor([math.sqrt(max(0.0, 1.0 - a * a)) * sc for a, sc in zip(corr_l, scale_l)],
                          dtype=torch.float32)
    coef_c = torch.repeat_interleave(coef_c, reps).to(device)
    coef_n = torch.repeat_interleave(coef_n, reps).to(device)
    shared = torch.randn(N, generator=dg, device=device, dtype=torch.float32) * coef_c
    del coef_c
    grads = []
    for _ in range(K):
        g = torch.randn(N, generator=dg, device=device, dtype=torch.float32)
        g.mul_(coef_n).add_(shared)
        grads.append(g.to(dtype) if dtype != torch.float32 else g)
    del shared, coef_n
    return Workload(name, K, dtype, offs, grads,
                    {"corr": corr_l, "scale": scale_l, "kind": ["gauss"] * L})


def after_local_step(sizes: Sequence[int], K: int, *, dtype=torch.float32, device="cpu", seed: int = 0,
                     step: float = 0.1, corr=None, scale=None, name: str = "after_local_step") -> Workload:
    """Inputs of the Adasum-after-optimizer form (Section 4.1): one starting
    parameter buffer and K buffers of parameters after each worker's local step.

    ``start = scale_l * N(0,1)`` (drawn after everything ``correlated_gaussian``
    draws, from a generator seeded ``seed + 1``); worker k's local update is
    ``-step * g_k`` with ``g_k`` the correlated Gaussian gradients of the same
    seed, so ``current_k = start - step * g_k``, computed in fp32 and rounded
    to ``dtype``.  ``start`` (also rounded to ``dtype``) is in ``meta["start"]``;
    ``grads`` holds the K current-parameter buffers."""
    w = correlated_gaussian(sizes, K, dtype=torch.float32, device=device, seed=seed, corr=corr, scale=scale,
                            name=name)
    reps = torch.tensor([int(x) for x in sizes], dtype=torch.int64)
    per_elem = torch.repeat_interleave(torch.tensor(w.meta["scale"], dtype=torch.float32), reps).to(device)
    start = torch.randn(w.N, generator=_gen(device, seed + 1), device=device, dtype=torch.float32) * per_elem
    del per_elem
    start = start.to(dtype)
    wide = start.to(torch.float32)
    current = []
    for g in w.grads:
        g.mul_(-step).add_(wide)
        current.append(g.to(dtype) if dtype != torch.float32 else g)
    meta = dict(w.meta)
    meta["start"] = start
    meta["step"] = step
    return Workload(name, K, dtype, w.layer_offsets, current, meta)


def log_uniform_scales(L: int, seed: int, lo_exp=-4.0, hi_exp=0.0) -> List[float]:
    """Per-layer magnitudes ``10^U(lo_exp, hi_exp)`` (layer-wise gradient spread)."""
    hg = _host_gen(seed + 7919)
    u = torch.rand(L, generator=hg, dtype=torch.float64)
    return (10.0 ** (lo_exp + (hi_exp - lo_exp) * u)).tolist()


def config1(device="cpu") -> Workload:
    """K=4, fp32, layers of 1000/4096/65536 elements, a = 0.6, seed 0."""
    return correlated_gaussian([1000, 4096, 65536], 4, dtype=torch.float32,
                               device=device, seed=0, corr=0.6, name="config1")


def config2(device="cpu", K: int = 8) -> Workload:
    """K=8, fp32, ResNet-50-shaped, per-layer a ~ U(0,1), seed 1."""
    return correlated_gaussian(resnet50_layer_sizes(), K, dtype=torch.float32,
                               device=device, seed=1, name="config2")


def config3(device="cpu", K: int = 16, sizes=None) -> Workload:
    """K=16, fp32, BERT-Large-shaped, per-layer a ~ U(0,1), seed 2."""
    sizes = bert_large_layer_sizes() if sizes is None else sizes
    return correlated_gaussian(sizes, K, dtype=torch.float32, device=device,
                               seed=2, name="config3")


def config4(device="cpu", K: int = 64, sizes=None) -> Workload:
    """K=64, bf16, BERT-Large-shaped, a ~ U(0,1), scale 10^U(-4,0), seed 3."""
    sizes = bert_large_layer_sizes() if sizes is None else sizes
    return correlated_gaussian(sizes, K, dtype=torch.bfloat16, device=device,
                               seed=3, scale=log_uniform_scales(len(sizes), 3),
                               name="config4")


def config5(device="cpu", K: int = 128, sizes=None, n_scalar_layers: int = 16) -> Workload:
    """K=128, bf16, BERT-Large-shaped with the method's degenerate cases, seed 4.

    Starting from the config-4 recipe, a seeded draw gives each layer a kind:
      * ``parallel``  (10 %): a = 0.999, workers almost collinear;
      * ``orth_pairs`` (10 %): every leaf pair (2j, 2j+1) orthogonalised in fp64
        (one Gram-Schmidt step on worker 2j+1) before rounding to bf16;
      * ``zero``      (2 %, at least three layers): cycling through "all workers
        zero", "one worker of a leaf pair zero" and "a whole quarter subtree
        zero";
      * ``orth_all``  (one layer of >= K elements): all K workers mutually
        orthogonal (Gram-Schmidt, applied twice, on a Gaussian matrix in fp64,
        then rounded);
      * ``gauss``     everything else.
    ``n_scalar_layers`` one-element tensors are inserted at seeded positions;
    they make every later boundary odd, so no later layer starts on a 16-byte
    boundary.

    Only element-wise kernels and short row sums are used on the device (no BLAS
    or solver library call, no reduction that spans workgroups), so the generator
    also runs under a counter-collecting profiler.
    """
    base = list(bert_large_layer_sizes() if sizes is None else sizes)
    hg = _host_gen(4)
    # insert 1-element "bias" tensors
    for _ in range(n_scalar_layers):
        pos = int(torch.randint(0, len(base) + 1, (1,), generator=hg).item())
        base.insert(pos, 1)
    L = len(base)
    corr_l = torch.rand(L, generator=hg, dtype=torch.float64).tolist()
    scale_l = log_uniform_scales(L, 4)
    kind = ["gauss"] * L
    perm = torch.randperm(L, generator=hg).tolist()
    n_par = max(1, round(0.10 * L))
    n_orth = max(1, round(0.10 * L))
    n_zero = max(3, round(0.02 * L))
    it = iter(perm)
    for _ in range(n_par):
        kind[next(it)] = "parallel"
    for _ in range(n_orth):
        kind[next(it)] = "orth_pairs"
    zero_modes = []
    for z in range(n_zero):
        kind[next(it)] = "zero"
    for l in it:
        if base[l] >= K and base[l] <= 1 << 20:
            kind[l] = "orth_all"
            break
    offs = offsets_from_sizes(base)
    dtype = torch.bfloat16
    for l, k in enumerate(kind):
        if k == "parallel":
            corr_l[l] = 0.999
    # every layer first gets the plain correlated-Gaussian recipe; the special kinds overwrite theirs
    grads = correlated_gaussian(base, K, dtype=dtype, device=device, seed=4, corr=corr_l, scale=scale_l).grads
    dg = _gen(device, 4 + 1000)
    zero_seen = 0
    for l, n in enumerate(base):
        k = kind[l]
        if n == 0 or k in ("gauss", "parallel"):
            continue
        a = corr_l[l]
        b = math.sqrt(max(0.0, 1.0 - a * a))
        sl = slice(offs[l], offs[l + 1])
        if k == "orth_all":
            q = _orthonormal_columns(torch.randn(n, K, generator=dg, device=device, dtype=torch.float64))
            for i in range(K):
                grads[i][sl] = (q[:, i] * (scale_l[l] * math.sqrt(n))).to(dtype)
        elif k == "orth_pairs":
            c = torch.randn(n, generator=dg, device=device, dtype=torch.float32)
            prev64 = None
            for i in range(K):
                ni = torch.randn(n, generator=dg, device=device, dtype=torch.float32)
                g64 = ((c * a + ni * b) * scale_l[l]).to(torch.float64)
                if i % 2 == 0:
                    prev64 = g64
                else:
                    pn = _sum_last(prev64 * prev64).clamp_min(1e-300)
                    g64 = g64 - (_sum_last(g64 * prev64) / pn) * prev64
                grads[i][sl] = g64.to(dtype)
        elif k == "zero":
            mode = zero_seen % 3
            zero_seen += 1
            zero_modes.append((l, mode))
            if mode == 0:
                dead = range(K)
            elif mode == 1:
                dead = [1] if K > 1 else [0]
            else:
                q4 = max(1, K // 4)
                dead = range(q4, 2 * q4) if K >= 4 else [0]
            for i in dead:
                grads[i][sl] = 0
    return Workload("config5", K, dtype, offs, grads,
                    {"corr": corr_l, "scale": scale_l, "kind": kind,
                     "zero_modes": zero_modes})


def _sum_last(x: torch.Tensor) -> torch.Tensor:
    """Sum over the last dimension in stages of at most 1024 terms per output, so that no
    single reduction is split over several workgroups."""
    c = 1024
    while x.shape[-1] > c:
        pad = (-x.shape[-1]) % c
        if pad:
            x = torch.nn.functional.pad(x, (0, pad))
        x = x.reshape(*x.shape[:-1], -1, c).sum(-1)
    return x.sum(-1)


def _orthonormal_columns(m: torch.Tensor) -> torch.Tensor:
    """Columns of ``m`` (n x k, fp64, n >= k) made orthonormal by classical Gram-Schmidt
    applied twice per column, with element-wise products and short row sums only."""
    q = m.t().contiguous()            # rows are the vectors
    for i in range(q.shape[0]):
        v = q[i].clone()
        for _ in range(2):
            if i > 0:
                coef = _sum_last(q[:i] * v[None, :])
                v = v - (q[:i] * coef[:, None]).sum(0)
        q[i] = v / _sum_last(v * v).sqrt()
    return q.t()


def scaled_down(sizes: Sequence[int], factor: int, floor: int = 1) -> List[int]:
    """Divide every layer size by ``factor`` (at least ``floor``): the same
    length *mix* at a size a CPU oracle finishes quickly."""
    return [max(floor, int(s) // factor) for s in sizes]
