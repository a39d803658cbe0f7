"""CPU oracle for the Adasum combiner -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.

A plain, slow, fp64 NumPy evaluation of what "Scaling Distributed Training with
Adaptive Summation" (arXiv 2006.02924) defines.  Only the tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import it; the HIP library shares
no code, table or helper with it and never calls it.

What each function follows:

* ``adasum_pair``    -- the two-gradient operator stated in Section 1 and again
  at the start of Section 3 (and as the "apply" step of Algorithm 1):
  ``(1 - g1.g2 / (2 |g1|^2)) g1 + (1 - g1.g2 / (2 |g2|^2)) g2``.
* ``adasum_tree``    -- the recursive halving application of Section 3.4 that
  the paper uses in practice (a balanced binary tree over the workers).
* ``adasum_linear``  -- the left-to-right application, also Section 3.4
  (a different result: the operator is not associative).
* ``adasum_reduce``  -- per-layer application, Section 3.6 (last paragraph) and
  the boundary bookkeeping of Section 4.4.3: each layer of the fused buffer is
  reduced on its own.
* ``orthogonality``  -- the per-layer metric defined in Section 3.6.
* ``adasum_after_optimizer`` -- Section 4.1: when the optimizer is stateful the
  operator is applied to each worker's *effective gradient*, the parameters
  after its local optimizer step minus the parameters before it; the combined
  effective gradient is added to the parameters before the step.

Dot products and squared norms are accumulated in double precision, as
Section 4.4.1 prescribes; every intermediate tree node stays fp64 and nothing
is rounded.  Inputs are the *stored* values (fp32 or bf16) widened exactly.

Readings where the paper is silent:

* zero-norm operand: the division is undefined; the convention taken is
  "coefficient of a zero-norm operand is 1", so Adasum(0, g) = g and
  Adasum(0, 0) = 0.  The test is ``norm == 0`` exactly.  (The dot product with
  a zero vector is 0, so the other operand's coefficient is exactly 1 and any
  finite value would do for the zero one; the convention only removes 0/0.)
* number of workers that is not a power of two: Algorithm 1 (the distributed
  exchange) requires a power of two, the recursion of Section 3.4 does not.
  It writes the two parts of g_[0,n] (n + 1 gradients) as [0, n/2) and
  [n/2, n]; read literally, with n/2 a real number, the left part holds
  ceil(n/2) = floor(K/2) of the K = n + 1 gradients.  ``adasum_tree`` splits
  there (``K // 2``), at every node.  The written-out expansions for K = 3, 5,
  6, 7 are pinned; that this reading is the authors' intent is not (their
  implementation only runs on powers of two).
* NaN/Inf inputs: propagated by IEEE arithmetic (a non-finite value poisons its
  own layer and no other; pinned).

``rel_l2_per_layer`` is the comparison metric of the parity tests, not part of
the method; it is pinned by hand values and planted slips like the rest.
Sums of products go through ``numpy.dot`` (a library routine in fp64, whose
summation order differs from a plain loop by rounding only).

Everything else is pinned by ``tests/test_oracle_pins.py``.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def _as_f64(v) -> np.ndarray:
    a = np.asarray(v)
    if a.dtype != np.float64:
        a = a.astype(np.float64)
    return a


def pair_scalars(g1: np.ndarray, g2: np.ndarray):
    """``(g1.g2, |g1|^2, |g2|^2)`` in fp64 -- the triple of Algorithm 1's
    "partial dot products" step, over the whole vectors."""
    g1 = _as_f64(g1)
    g2 = _as_f64(g2)
    d = float(np.dot(g1, g2))
    n1 = float(np.dot(g1, g1))
    n2 = float(np.dot(g2, g2))
    return d, n1, n2


def pair_coefficients(d: float, n1: float, n2: float):
    """Scalars multiplying g1 and g2 in the operator of Section 3; a zero-norm
    operand gets coefficient 1 (convention, see module header)."""
    a = 1.0 - d / (2.0 * n1) if n1 > 0.0 else 1.0
    b = 1.0 - d / (2.0 * n2) if n2 > 0.0 else 1.0
    return a, b


def adasum_pair(g1, g2) -> np.ndarray:
    """Adasum(g1, g2) of Section 3 for two vectors of equal length."""
    g1 = _as_f64(g1)
    g2 = _as_f64(g2)
    if g1.shape != g2.shape:
        raise ValueError("operands differ in shape")
    d, n1, n2 = pair_scalars(g1, g2)
    a, b = pair_coefficients(d, n1, n2)
    return a * g1 + b * g2


def adasum_tree(gs: Sequence) -> np.ndarray:
    """Adasum of ``gs[0..K)`` by recursive halving (Section 3.4, second form):
    the left half and the right half are reduced first, then combined."""
    K = len(gs)
    if K == 0:
        raise ValueError("need at least one gradient")
    if K == 1:
        return _as_f64(gs[0]).copy()
    mid = K // 2
    left = adasum_tree(gs[:mid])
    right = adasum_tree(gs[mid:])
    return adasum_pair(left, right)


def adasum_linear(gs: Sequence) -> np.ndarray:
    """Adasum of ``gs[0..K)`` applied left to right (Section 3.4, first form)."""
    if len(gs) == 0:
        raise ValueError("need at least one gradient")
    acc = _as_f64(gs[0]).copy()
    for g in gs[1:]:
        acc = adasum_pair(acc, g)
    return acc


def adasum_reduce(grads: Sequence, layer_offsets: Sequence[int], order: str = "tree") -> np.ndarray:
    """Per-layer Adasum of K flat gradients (Section 3.6 / Section 4.4.3).

    ``grads[i]`` is worker i's fused buffer of ``layer_offsets[-1]`` elements;
    layer ``l`` is ``[layer_offsets[l], layer_offsets[l+1])``.  Returns the fp64
    fused result.
    """
    offs = [int(o) for o in layer_offsets]
    if not offs or offs[0] != 0:
        raise ValueError("layer_offsets must start at 0")
    N = offs[-1]
    combine = adasum_tree if order == "tree" else adasum_linear
    out = np.zeros(N, dtype=np.float64)
    for l in range(len(offs) - 1):
        lo, hi = offs[l], offs[l + 1]
        if hi < lo:
            raise ValueError("layer_offsets must not decrease")
        if hi == lo:
            continue
        out[lo:hi] = combine([np.asarray(g)[lo:hi] for g in grads])
    return out


def adasum_after_optimizer(start, currents: Sequence, layer_offsets: Sequence[int]) -> np.ndarray:
    """New parameters of Section 4.1's scheme: every worker starts from ``start``,
    takes its own optimizer step to ``currents[i]``; the effective gradients
    ``currents[i] - start`` are combined per layer by the Adasum tree and the
    result is added to ``start``."""
    w0 = _as_f64(start)
    deltas = [_as_f64(c) - w0 for c in currents]
    return w0 + adasum_reduce(deltas, layer_offsets)


def orthogonality(grads: Sequence, layer_offsets: Sequence[int]) -> np.ndarray:
    """Per-layer ``|Adasum(g_1..g_K)|^2 / sum_i |g_i|^2`` (Section 3.6).
    Layers whose gradients are all zero give NaN."""
    offs = [int(o) for o in layer_offsets]
    res = np.full(len(offs) - 1, np.nan)
    for l in range(len(offs) - 1):
        lo, hi = offs[l], offs[l + 1]
        parts = [_as_f64(np.asarray(g)[lo:hi]) for g in grads]
        den = sum(float(np.dot(p, p)) for p in parts)
        if den > 0.0:
            r = adasum_tree(parts)
            res[l] = float(np.dot(r, r)) / den
    return res


def rel_l2_per_layer(test, ref, layer_offsets: Sequence[int]) -> np.ndarray:
    """Comparison metric: per layer ``|test - ref|_2 / |ref|_2`` in fp64.
    A layer whose reference is exactly zero scores 0 if the test output is
    exactly zero there and +inf otherwise; empty layers score 0."""
    t = _as_f64(test)
    r = _as_f64(ref)
    offs = [int(o) for o in layer_offsets]
    res = np.zeros(len(offs) - 1)
    for l in range(len(offs) - 1):
        lo, hi = offs[l], offs[l + 1]
        if hi == lo:
            continue
        den = float(np.sqrt(np.dot(r[lo:hi], r[lo:hi])))
        diff = t[lo:hi] - r[lo:hi]
        num = float(np.sqrt(np.dot(diff, diff)))
        if den == 0.0:
            res[l] = 0.0 if num == 0.0 else np.inf
        else:
            res[l] = num / den
    return res
