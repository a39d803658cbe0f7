"""Pins for the CPU oracle: what the paper and the mathematics fix.

None of these restate the oracle's code.  Each pin is a hand-derived value, a
closed form, an invariant, or a different computational route, chosen so that a
plausible slip in the oracle (a dropped factor 2, swapped norms, a wrong sign,
the wrong recursion shape, whole-buffer instead of per-layer scalars) fails at
least one of them; ``test_mutants_are_caught`` plants such slips in copies of
the oracle (on the CPU) and checks that the pins notice.
"""
import math
import os
import types
from fractions import Fraction

import numpy as np
import pytest

from oracle import adasum_oracle as ORACLE

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# individual pins; every one takes the oracle module so that mutants can be
# pushed through the same checks
# --------------------------------------------------------------------------

def pin_closed_form_two_vectors(O):
    # Section 3 operator by hand: g1=(1,0), g2=(1,1): d=1, n1=1, n2=2,
    # coefficients 1/2 and 3/4, result (5/4, 3/4).
    r = O.adasum_pair([1.0, 0.0], [1.0, 1.0])
    np.testing.assert_allclose(r, [1.25, 0.75], rtol=0, atol=1e-15)
    # asymmetric norms, negative dot: g1=(2,0), g2=(-1,1): d=-2, n1=4, n2=2,
    # a = 1 + 2/8 = 5/4, b = 1 + 2/4 = 3/2, result (5/2 - 3/2, 3/2) = (1, 3/2)
    r = O.adasum_pair([2.0, 0.0], [-1.0, 1.0])
    np.testing.assert_allclose(r, [1.0, 1.5], rtol=0, atol=1e-15)


def pin_worked_tree_fixture(O):
    rows = {}
    with open(os.path.join(GOLDEN, "k4_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            rows[name] = [float(Fraction(v)) for v in vals]
    g = [rows["g0"], rows["g1"], rows["g2"], rows["g3"]]
    np.testing.assert_allclose(O.adasum_pair(g[0], g[1]), rows["P"], rtol=1e-15)
    np.testing.assert_allclose(O.adasum_pair(g[2], g[3]), rows["Q"], rtol=1e-15)
    np.testing.assert_allclose(O.adasum_tree(g), rows["R"], rtol=4e-16)
    # the same data as one 2-element layer of a fused buffer
    np.testing.assert_allclose(O.adasum_reduce(g, [0, 2]), rows["R"], rtol=4e-16)


def pin_idempotent(O):
    # Section 3.5: parallel gradients are averaged, so K copies of g give g,
    # and the Section 3.6 metric reaches its minimum 1/K.
    g = _rng(1).standard_normal(257)
    for K in (2, 4, 8, 64):
        np.testing.assert_allclose(O.adasum_tree([g] * K), g, rtol=1e-13)
        m = O.orthogonality([g] * K, [0, g.size])
        np.testing.assert_allclose(m, [1.0 / K], rtol=1e-12)


def pin_orthogonal_is_sum(O):
    # Section 3.5: zero dot product => plain sum; Section 3.6: metric = 1.
    rng = _rng(2)
    q, _ = np.linalg.qr(rng.standard_normal((40, 8)))
    gs = [q[:, i] * (i + 1.0) for i in range(8)]
    np.testing.assert_allclose(O.adasum_tree(gs), np.sum(gs, axis=0), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(O.orthogonality(gs, [0, 40]), [1.0], rtol=1e-12)
    # exactly orthogonal by disjoint support: exact sum
    e = np.eye(4)
    np.testing.assert_array_equal(O.adasum_tree([3 * e[0], -2 * e[1], e[2], 5 * e[3]]),
                                  [3.0, -2.0, 1.0, 5.0])


def pin_collinear_is_mean(O):
    # g2 = c*g1 (either sign): coefficients (1 - c/2) and (1 - 1/(2c)), so the
    # result is ((1 - c/2) + (c - 1/2)) g1 = (1 + c)/2 g1 = (g1 + g2)/2.
    g = _rng(3).standard_normal(33)
    for c in (3.0, 0.25, -0.5, -4.0):
        np.testing.assert_allclose(O.adasum_pair(g, c * g), (g + c * g) / 2, rtol=1e-13, atol=1e-15)
    # hence a one-element layer is the arithmetic mean of the K scalars
    x = _rng(4).standard_normal(16) + 3.0
    r = O.adasum_tree([np.array([v]) for v in x])
    np.testing.assert_allclose(r, [x.mean()], rtol=1e-13)


def pin_output_norm_closed_form(O):
    # expanding |a g1 + b g2|^2 with a = 1 - d/(2 n1), b = 1 - d/(2 n2):
    # n1 + n2 - (3/4) d^2 (1/n1 + 1/n2) + d^3 / (2 n1 n2);  never above n1 + n2
    rng = _rng(5)
    for _ in range(5):
        g1 = rng.standard_normal(50)
        g2 = 0.3 * g1 + rng.standard_normal(50) * rng.uniform(0.1, 3)
        d, n1, n2 = float(g1 @ g2), float(g1 @ g1), float(g2 @ g2)
        want = n1 + n2 - 0.75 * d * d * (1 / n1 + 1 / n2) + d ** 3 / (2 * n1 * n2)
        r = O.adasum_pair(g1, g2)
        assert math.isclose(float(r @ r), want, rel_tol=1e-12)
        assert float(r @ r) <= (n1 + n2) * (1 + 1e-14)


def pin_symmetry_homogeneity(O):
    rng = _rng(6)
    gs = [rng.standard_normal(19) for _ in range(8)]
    r = O.adasum_tree(gs)
    np.testing.assert_allclose(O.adasum_pair(gs[1], gs[0]), O.adasum_pair(gs[0], gs[1]), rtol=1e-14)
    # degree-1 homogeneous
    np.testing.assert_allclose(O.adasum_tree([-2.5 * g for g in gs]), -2.5 * r, rtol=1e-13)
    # swapping siblings at any level of the tree changes nothing
    sw = [gs[1], gs[0], gs[2], gs[3], gs[6], gs[7], gs[4], gs[5]]
    np.testing.assert_allclose(O.adasum_tree(sw), r, rtol=1e-13)
    # but the tree is NOT the left-to-right fold (Section 3.4: two recursions)
    sw2 = [gs[0], gs[2], gs[1], gs[3]] + gs[4:]
    assert np.linalg.norm(O.adasum_tree(sw2) - r) > 1e-6 * np.linalg.norm(r)


def pin_layer_independence(O):
    # Section 3.6 / 4.4.3: the operator is applied per layer of the fused buffer
    rng = _rng(7)
    sizes = [5, 1, 0, 12, 3]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    K = 4
    grads = [rng.standard_normal(offs[-1]) * (1 + i) for i in range(K)]
    fused = O.adasum_reduce(grads, offs)
    for l in range(len(sizes)):
        lo, hi = offs[l], offs[l + 1]
        if hi > lo:
            alone = O.adasum_tree([g[lo:hi] for g in grads])
            np.testing.assert_allclose(fused[lo:hi], alone, rtol=1e-14)
    # and it is NOT the whole-buffer operator
    whole = O.adasum_tree(grads)
    assert np.linalg.norm(whole - fused) > 1e-6 * np.linalg.norm(fused)


def _exact_tree(vs):
    """Section 3.4 halving recursion in exact rational arithmetic."""
    if len(vs) == 1:
        return vs[0]
    mid = len(vs) // 2
    A, B = _exact_tree(vs[:mid]), _exact_tree(vs[mid:])
    d = sum(x * y for x, y in zip(A, B))
    n1 = sum(x * x for x in A)
    n2 = sum(y * y for y in B)
    a = 1 - d / (2 * n1) if n1 != 0 else Fraction(1)
    b = 1 - d / (2 * n2) if n2 != 0 else Fraction(1)
    return [a * x + b * y for x, y in zip(A, B)]


def pin_exact_rational_small(O):
    rng = _rng(8)
    for K in (2, 4, 8):
        for dim in (1, 2, 5):
            ints = rng.integers(-4, 5, size=(K, dim))
            ints[ints == 0] = 1
            exact = _exact_tree([[Fraction(int(v)) for v in row] for row in ints])
            got = O.adasum_tree([row.astype(np.float64) for row in ints])
            np.testing.assert_allclose(got, [float(v) for v in exact], rtol=1e-12, atol=1e-14)


def _gram_route(gs):
    """Independent route: the tree output is sum_i w_i g_i; the weights follow
    from the K x K Gram matrix alone by a scalar recursion over weight vectors."""
    X = np.stack([np.asarray(g, dtype=np.float64) for g in gs])
    G = X @ X.T
    K = len(gs)

    def rec(lo, hi):
        if hi - lo == 1:
            w = np.zeros(K)
            w[lo] = 1.0
            return w
        mid = (lo + hi) // 2
        u, v = rec(lo, mid), rec(mid, hi)
        d, n1, n2 = u @ G @ v, u @ G @ u, v @ G @ v
        a = 1 - d / (2 * n1) if n1 > 0 else 1.0
        b = 1 - d / (2 * n2) if n2 > 0 else 1.0
        return a * u + b * v

    return rec(0, K) @ X


def pin_gram_route(O):
    rng = _rng(9)
    for K in (2, 4, 8, 16):
        c = rng.standard_normal(300)
        gs = [0.5 * c + rng.standard_normal(300) for _ in range(K)]
        np.testing.assert_allclose(O.adasum_tree(gs), _gram_route(gs), rtol=1e-11, atol=1e-13)


def pin_generator_limit(O):
    # g_i = alpha c + sqrt(1-alpha^2) n_i with unit Gaussians, large layers:
    # per-element node energy s and sibling dot p obey s0=1, p0=alpha^2,
    # gamma = 1 - p/(2s), s' = gamma^2 (2s + 2p), p' = 4 gamma^2 p.
    # alpha = 0.6: gamma0 = 0.82, s1 = 1.828928, p1 = 0.968256,
    # gamma1 = 0.735294..., s2 = 3.02464...
    rng = _rng(10)
    n = 200_000
    c = rng.standard_normal(n)
    gs = [0.6 * c + 0.8 * rng.standard_normal(n) for _ in range(4)]
    d, n1, n2 = O.pair_scalars(gs[0], gs[1])
    a, b = O.pair_coefficients(d, n1, n2)
    assert abs(a - 0.82) < 0.01 and abs(b - 0.82) < 0.01
    P, Q = O.adasum_pair(gs[0], gs[1]), O.adasum_pair(gs[2], gs[3])
    assert abs(float(P @ P) / n - 1.828928) < 0.03
    d, n1, n2 = O.pair_scalars(P, Q)
    assert abs(d / n - 0.968256) < 0.03
    a, b = O.pair_coefficients(d, n1, n2)
    assert abs(a - 0.735294) < 0.01 and abs(b - 0.735294) < 0.01
    R = O.adasum_tree(gs)
    assert abs(float(R @ R) / n - 3.02464) < 0.05
    np.testing.assert_allclose(O.orthogonality(gs, [0, n]), [3.02464 / 4], rtol=0.03)


def pin_zero_convention(O):
    g = np.array([1.0, -2.0, 3.0])
    z = np.zeros(3)
    np.testing.assert_array_equal(O.adasum_pair(z, g), g)
    np.testing.assert_array_equal(O.adasum_pair(g, z), g)
    np.testing.assert_array_equal(O.adasum_pair(z, z), z)
    # a zero leaf / zero subtree passes its sibling up
    h = np.array([0.5, 0.5, -1.0])
    np.testing.assert_allclose(O.adasum_tree([z, g, h, z]), O.adasum_pair(g, h), rtol=1e-15)
    np.testing.assert_allclose(O.adasum_tree([z, z, g, h]), O.adasum_pair(g, h), rtol=1e-15)
    np.testing.assert_array_equal(O.adasum_tree([z, z, z, z]), z)
    assert np.isnan(O.orthogonality([z, z], [0, 3])[0])


def pin_linear_order(O):
    # Section 3.4 first recursion: fold left to right.
    rng = _rng(11)
    gs = [rng.standard_normal(7) for _ in range(4)]
    want = O.adasum_pair(O.adasum_pair(O.adasum_pair(gs[0], gs[1]), gs[2]), gs[3])
    np.testing.assert_allclose(O.adasum_linear(gs), want, rtol=1e-15)
    # for K = 2 both recursions coincide
    np.testing.assert_allclose(O.adasum_linear(gs[:2]), O.adasum_tree(gs[:2]), rtol=1e-15)
    # orthogonal inputs: any order is the plain sum
    e = np.eye(4)
    np.testing.assert_array_equal(O.adasum_linear([e[0], e[1], e[2], e[3]]), np.ones(4))


def pin_low_precision_inputs_are_widened(O):
    # Section 4.4.1: accumulation in double even for low-precision inputs.
    # 2^24 + 1 is not representable in fp32: an fp32 accumulator would lose it.
    n = (1 << 24) + 1
    g1 = np.ones(n, dtype=np.float32)
    d, n1, n2 = O.pair_scalars(g1, g1)
    assert d == float(n) and n1 == float(n) and n2 == float(n)


def pin_worker_counts_that_are_no_power_of_two(O):
    # Section 3.4, second recursion, read literally: g_[0,n] -> g_[0,n/2) and g_[n/2,n], so of K = n + 1
    # gradients the left part takes floor(K/2).  Written out by hand for K = 3, 5, 6, 7.
    rng = _rng(13)
    g = [rng.standard_normal(6) for _ in range(7)]
    P = O.adasum_pair
    np.testing.assert_allclose(O.adasum_tree(g[:3]), P(g[0], P(g[1], g[2])), rtol=1e-14)
    np.testing.assert_allclose(O.adasum_tree(g[:5]), P(P(g[0], g[1]), P(g[2], P(g[3], g[4]))), rtol=1e-14)
    np.testing.assert_allclose(O.adasum_tree(g[:6]), P(P(g[0], P(g[1], g[2])), P(g[3], P(g[4], g[5]))), rtol=1e-14)
    np.testing.assert_allclose(O.adasum_tree(g[:7]),
                               P(P(g[0], P(g[1], g[2])), P(P(g[3], g[4]), P(g[5], g[6]))), rtol=1e-14)
    # properties that hold for any K: K copies give the copy, orthogonal inputs give the sum
    np.testing.assert_allclose(O.adasum_tree([g[0]] * 5), g[0], rtol=1e-14)
    e = np.eye(7)
    np.testing.assert_array_equal(O.adasum_tree(list(e)), np.ones(7))


def pin_after_optimizer(O):
    # Section 4.1.  Hand-worked, K = 2, one layer: start (1,1); worker steps to (2,1) and (2,2), so the
    # effective gradients are (1,0) and (1,1): d = 1, n1 = 1, n2 = 2, coefficients 1/2 and 3/4, combined
    # (5/4, 3/4), new parameters (9/4, 7/4).  (The operator applied to the parameters themselves would
    # give (2.05, 1.65).)
    got = O.adasum_after_optimizer(np.array([1.0, 1.0]), [np.array([2.0, 1.0]), np.array([2.0, 2.0])], [0, 2])
    np.testing.assert_allclose(got, [2.25, 1.75], rtol=1e-15)
    rng = _rng(12)
    start = rng.standard_normal(12)
    # every worker took the same step: that step is taken (the operator is idempotent)
    cur = start + 0.1 * rng.standard_normal(12)
    np.testing.assert_allclose(O.adasum_after_optimizer(start, [cur] * 4, [0, 5, 12]), cur, rtol=1e-14)
    # steps with disjoint supports are orthogonal: all of them are taken in full
    curs = []
    for k in range(4):
        c = start.copy()
        c[3 * k:3 * k + 3] += rng.standard_normal(3)
        curs.append(c)
    want = start + sum(c - start for c in curs)
    np.testing.assert_allclose(O.adasum_after_optimizer(start, curs, [0, 12]), want, rtol=1e-14)
    # per layer: a layer nobody moved keeps its parameters exactly
    curs = [start.copy() for _ in range(2)]
    curs[0][:5] += 1.0
    got = O.adasum_after_optimizer(start, curs, [0, 5, 12])
    np.testing.assert_array_equal(got[5:], start[5:])
    np.testing.assert_allclose(got[:5], start[:5] + 1.0, rtol=1e-15)


def pin_non_finite_inputs(O):
    """IEEE arithmetic on the Section 3 formula: one NaN or infinity in a layer of one worker makes
    a scalar of the first node that sees it NaN (d or a norm is NaN, or Inf / Inf), so that node
    and every ancestor is NaN in every element; other layers never see it (Section 3.6)."""
    rng = np.random.default_rng(17)
    for K in (2, 3, 8):
        for bad in (np.nan, np.inf, -np.inf):
            gs = [rng.standard_normal(14) for _ in range(K)]
            gs[K // 2][9] = bad
            clean = [g.copy() for g in gs]
            clean[K // 2][9] = 0.25
            with np.errstate(all="ignore"):
                got = O.adasum_reduce(gs, [0, 6, 14])
                lin = O.adasum_reduce(gs, [0, 6, 14], order="linear")
            want = O.adasum_reduce(clean, [0, 6, 14])
            assert np.isnan(got[6:]).all() and np.isnan(lin[6:]).all()
            np.testing.assert_array_equal(got[:6], want[:6])


def pin_comparison_metric(O):
    """rel_l2_per_layer: per layer |test - ref|_2 / |ref|_2.  Hand values: against ref (3, 4)
    (norm 5) the test (4, 6) is off by (1, 2), norm sqrt 5: the score is sqrt(5)/5; against
    ref (3, 0) the test (3, 4) scores 4/3.  Each layer is scored on its own norm; a zero
    reference scores 0 for a zero output and +inf otherwise; an empty layer scores 0; the roles
    of test and ref are not interchangeable; fp32 inputs are widened."""
    got = O.rel_l2_per_layer([4.0, 6.0], [3.0, 4.0], [0, 2])
    assert got.shape == (1,) and got[0] == pytest.approx(np.sqrt(5.0) / 5.0, rel=1e-15)
    assert O.rel_l2_per_layer([3.0, 4.0], [3.0, 0.0], [0, 2])[0] == pytest.approx(4.0 / 3.0, rel=1e-15)
    # two layers of very different scale, an empty one between them: 0 and exactly 1
    ref = np.array([1000.0, 0.0, 1e-3, 0.0])
    test = np.array([1000.0, 0.0, 2e-3, 0.0])
    np.testing.assert_allclose(O.rel_l2_per_layer(test, ref, [0, 2, 2, 4]), [0.0, 0.0, 1.0], rtol=1e-15)
    # zero reference
    z = O.rel_l2_per_layer([0.0, 0.0, 0.0, 1e-30], [0.0, 0.0, 0.0, 0.0], [0, 2, 4])
    assert z[0] == 0.0 and np.isinf(z[1])
    # exact agreement scores exactly 0; sign flips of both leave the score alone
    r = _rng(3).standard_normal(50)
    assert np.all(O.rel_l2_per_layer(r, r, [0, 20, 50]) == 0.0)
    t = r + 1e-3 * _rng(4).standard_normal(50)
    np.testing.assert_allclose(O.rel_l2_per_layer(-t, -r, [0, 20, 50]), O.rel_l2_per_layer(t, r, [0, 20, 50]),
                               rtol=1e-15)
    # homogeneous of degree 0; scaled error scales the score
    np.testing.assert_allclose(O.rel_l2_per_layer(7.0 * t, 7.0 * r, [0, 50]), O.rel_l2_per_layer(t, r, [0, 50]),
                               rtol=1e-13)
    np.testing.assert_allclose(O.rel_l2_per_layer(r + 2.0 * (t - r), r, [0, 50]),
                               2.0 * O.rel_l2_per_layer(t, r, [0, 50]), rtol=1e-12)
    # low-precision inputs are widened, not compared in their own precision
    t32 = np.array([1.0, 1.0 + 2.0 ** -20], dtype=np.float32)
    r64 = np.array([1.0, 1.0])
    assert O.rel_l2_per_layer(t32, r64, [0, 2])[0] == pytest.approx(2.0 ** -20 / np.sqrt(2.0), rel=1e-12)


PINS = [
    pin_closed_form_two_vectors,
    pin_worked_tree_fixture,
    pin_idempotent,
    pin_orthogonal_is_sum,
    pin_collinear_is_mean,
    pin_output_norm_closed_form,
    pin_symmetry_homogeneity,
    pin_layer_independence,
    pin_exact_rational_small,
    pin_gram_route,
    pin_generator_limit,
    pin_zero_convention,
    pin_linear_order,
    pin_low_precision_inputs_are_widened,
    pin_after_optimizer,
    pin_worker_counts_that_are_no_power_of_two,
    pin_non_finite_inputs,
    pin_comparison_metric,
]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(ORACLE)


# --------------------------------------------------------------------------
# planted mistakes (in copies of the oracle, on the CPU)
# --------------------------------------------------------------------------

def _clone():
    """A fresh copy of the oracle module whose functions resolve their globals
    inside the copy, so patching one function affects its callers."""
    src = open(ORACLE.__file__).read()
    m = types.ModuleType("oracle_mutant")
    m.__file__ = ORACLE.__file__
    exec(compile(src, ORACLE.__file__, "exec"), m.__dict__)
    return m


def _mut_drop_two(m):
    m.pair_coefficients = lambda d, n1, n2: (1 - d / n1 if n1 > 0 else 1.0,
                                             1 - d / n2 if n2 > 0 else 1.0)


def _mut_swap_norms(m):
    m.pair_coefficients = lambda d, n1, n2: (1 - d / (2 * n2) if n2 > 0 else 1.0,
                                             1 - d / (2 * n1) if n1 > 0 else 1.0)


def _mut_plus_sign(m):
    m.pair_coefficients = lambda d, n1, n2: (1 + d / (2 * n1) if n1 > 0 else 1.0,
                                             1 + d / (2 * n2) if n2 > 0 else 1.0)


def _mut_norm_not_squared(m):
    orig = m.pair_scalars

    def ps(g1, g2):
        d, n1, n2 = orig(g1, g2)
        return d, math.sqrt(n1), math.sqrt(n2)
    m.pair_scalars = ps


def _mut_tree_is_fold(m):
    m.adasum_tree = m.adasum_linear


def _mut_uneven_split(m):
    def tree(gs):
        if len(gs) == 1:
            return np.asarray(gs[0], dtype=np.float64).copy()
        mid = 1 if len(gs) > 2 else len(gs) // 2
        return m.adasum_pair(tree(gs[:mid]), tree(gs[mid:]))
    m.adasum_tree = tree


def _mut_left_takes_the_larger_part(m):
    def tree(gs):
        if len(gs) == 1:
            return np.asarray(gs[0], dtype=np.float64).copy()
        mid = (len(gs) + 1) // 2
        return m.adasum_pair(tree(gs[:mid]), tree(gs[mid:]))
    m.adasum_tree = tree


def _mut_whole_buffer(m):
    def red(grads, offs, order="tree"):
        return m.adasum_tree([np.asarray(g, dtype=np.float64) for g in grads])
    m.adasum_reduce = red


def _mut_no_zero_guard(m):
    # the bare formula: a zero-norm operand divides by zero.  (Any *finite*
    # coefficient for the zero operand gives the same vector, because the dot
    # product is then 0 and the other coefficient is exactly 1; what the
    # convention must rule out is the NaN / the exception.)
    def pc(d, n1, n2):
        with np.errstate(all="ignore"):
            return (float(1 - np.float64(d) / np.float64(2 * n1)),
                    float(1 - np.float64(d) / np.float64(2 * n2)))
    m.pair_coefficients = pc


def _mut_fp32_accumulate(m):
    def ps(g1, g2):
        a = np.asarray(g1, dtype=np.float32)
        b = np.asarray(g2, dtype=np.float32)
        one = np.float32(0)
        d = n1 = n2 = one
        # strictly sequential fp32 accumulation on a prefix is enough to show it
        d = float(np.cumsum(a * b, dtype=np.float32)[-1])
        n1 = float(np.cumsum(a * a, dtype=np.float32)[-1])
        n2 = float(np.cumsum(b * b, dtype=np.float32)[-1])
        return d, n1, n2
    m.pair_scalars = ps


def _mut_linear_is_tree(m):
    m.adasum_linear = m.adasum_tree


def _mut_delta_sign(m):
    def f(start, currents, layer_offsets):
        w0 = m._as_f64(start)
        return w0 + m.adasum_reduce([w0 - m._as_f64(c) for c in currents], layer_offsets)
    m.adasum_after_optimizer = f


def _mut_delta_not_added_back(m):
    def f(start, currents, layer_offsets):
        w0 = m._as_f64(start)
        return m.adasum_reduce([m._as_f64(c) - w0 for c in currents], layer_offsets)
    m.adasum_after_optimizer = f


def _mut_operator_on_parameters(m):
    m.adasum_after_optimizer = lambda start, currents, layer_offsets: m.adasum_reduce(currents, layer_offsets)


def _metric_mutant(score):
    """rel_l2_per_layer with the per-layer score replaced by score(test_layer, ref_layer, test, ref)."""
    def install(m):
        def f(test, ref, layer_offsets):
            t, r = m._as_f64(test), m._as_f64(ref)
            offs = [int(o) for o in layer_offsets]
            res = np.zeros(len(offs) - 1)
            for l in range(len(offs) - 1):
                lo, hi = offs[l], offs[l + 1]
                if hi > lo:
                    with np.errstate(all="ignore"):
                        res[l] = score(t[lo:hi], r[lo:hi], t, r)
            return res
        m.rel_l2_per_layer = f
    return install


def _named(name, fn):
    fn.__name__ = name
    return fn


_norm = np.linalg.norm
METRIC_MUTANTS = [
    _named("_mut_metric_squared", _metric_mutant(lambda t, r, T, R: _norm(t - r) ** 2 / _norm(r) ** 2)),
    _named("_mut_metric_denominator_not_rooted", _metric_mutant(lambda t, r, T, R: _norm(t - r) / np.dot(r, r))),
    _named("_mut_metric_whole_buffer_norm", _metric_mutant(lambda t, r, T, R: _norm(t - r) / _norm(R))),
    _named("_mut_metric_max_norm", _metric_mutant(lambda t, r, T, R: np.abs(t - r).max() / np.abs(r).max())),
    _named("_mut_metric_l1_norm", _metric_mutant(lambda t, r, T, R: np.abs(t - r).sum() / np.abs(r).sum())),
    _named("_mut_metric_relative_to_test", _metric_mutant(lambda t, r, T, R: _norm(t - r) / _norm(t))),
    _named("_mut_metric_zero_reference_passes",
           _metric_mutant(lambda t, r, T, R: 0.0 if _norm(r) == 0.0 else _norm(t - r) / _norm(r))),
    _named("_mut_metric_mean_square", _metric_mutant(lambda t, r, T, R: _norm(t - r) / _norm(r) / np.sqrt(len(r)))),
]


MUTANTS = [_mut_drop_two, _mut_swap_norms, _mut_plus_sign, _mut_norm_not_squared,
           _mut_tree_is_fold, _mut_uneven_split, _mut_whole_buffer,
           _mut_no_zero_guard, _mut_fp32_accumulate, _mut_linear_is_tree,
           _mut_delta_sign, _mut_delta_not_added_back, _mut_operator_on_parameters,
           _mut_left_takes_the_larger_part] + METRIC_MUTANTS


@pytest.mark.parametrize("mutate", MUTANTS, ids=lambda f: f.__name__)
def test_mutants_are_caught(mutate):
    m = _clone()
    mutate(m)
    caught = []
    for pin in PINS:
        try:
            pin(m)
        except (AssertionError, ArithmeticError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices {mutate.__name__}"


def test_clone_is_faithful():
    m = _clone()
    for pin in PINS:
        pin(m)
