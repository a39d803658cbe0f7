"""The comparison helpers of the GPU parity tests, checked on the CPU: which
layers count as having no reference value, and that nothing else is excused."""
import numpy as np
import torch

from oracle import adasum_oracle as O
from tests import gpu_util as U


def test_exactly_cancelling_node_is_flagged_and_nothing_else():
    # layer 0 (one element): (1 + 3)/2 = 2 and (-1 + -3)/2 = -2 cancel exactly at the root's children
    # layer 1 (one element): ordinary values
    # layer 2 (three elements): all workers zero -- a legitimate zero, children are zero too
    # layer 3 (40 elements): larger than the excusable size even though two workers are opposite
    K = 4
    big = np.arange(1.0, 41.0)
    rows = [
        np.concatenate([[1.0], [0.5], np.zeros(3), big]),
        np.concatenate([[3.0], [0.25], np.zeros(3), -big]),
        np.concatenate([[-1.0], [2.0], np.zeros(3), big]),
        np.concatenate([[-3.0], [1.5], np.zeros(3), big]),
    ]
    offs = [0, 1, 2, 5, 45]
    ref = O.adasum_reduce(rows, offs)
    marked = U.mark_ill_posed(ref.copy(), rows, offs)
    assert np.isnan(marked[0])
    assert not np.isnan(marked[1:]).any()
    np.testing.assert_array_equal(marked[1:], ref[1:])
    # the left-to-right fold of the same values does not cancel at any node
    lin = O.adasum_reduce(rows, offs, order="linear")
    assert not np.isnan(U.mark_ill_posed(lin.copy(), rows, offs, "linear")).any()


def test_assert_parity_skips_only_marked_layers():
    offs = [0, 1, 5]
    ref = np.array([np.nan, 1.0, 2.0, 3.0, 4.0])
    good = torch.tensor([123.0, 1.0, 2.0, 3.0, 4.0])
    U.assert_parity(good, ref, offs)
    bad = torch.tensor([123.0, 1.0, 2.0, 3.0, 4.1])
    try:
        U.assert_parity(bad, ref, offs)
    except AssertionError:
        pass
    else:
        raise AssertionError("a wrong value in an ordinary layer must fail")
    try:
        U.assert_parity(torch.tensor([float("inf"), 1.0, 2.0, 3.0, 4.0]), ref, offs)
    except AssertionError:
        pass
    else:
        raise AssertionError("a non-finite output must fail even in a skipped layer")
