"""Host planner: tile table and pass schedule (no GPU needed)."""
import numpy as np
import pytest

from paper_2006_02924_amd import binding as B
from paper_2006_02924_amd import workloads as W


def check_tiles(offsets, cap=None):
    if cap is None:
        for c in (1024, 2048):
            check_tiles(offsets, c)
    cap = cap or B.tile_capacity()
    t = B.plan_tiles(offsets, cap)
    offsets = np.asarray(offsets, dtype=np.int64)
    N = int(offsets[-1])
    # cover [0, N) exactly, in order, without overlap
    if N == 0:
        assert len(t) == 0
        return t
    ends = t["start"] + t["len"]
    assert t["start"][0] == 0 and ends[-1] == N
    assert np.array_equal(t["start"][1:], ends[:-1])
    assert t["len"].min() >= 1 and t["len"].max() <= cap
    # never cross a layer boundary; layer ids are right
    lo = offsets[t["layer"]]
    hi = offsets[t["layer"] + 1]
    assert np.all(t["start"] >= lo) and np.all(ends <= hi)
    # interior boundaries fall on global multiples of the capacity or on layer boundaries
    inner = t["start"][1:]
    assert np.all((inner % cap == 0) | np.isin(inner, offsets))
    # full tiles are aligned to the capacity
    full = t["len"] == cap
    assert np.all(t["start"][full] % cap == 0)
    return t


def test_tiles_config1():
    t = check_tiles([0, 1000, 5096, 70632])
    assert list(t["layer"][:3]) == [0, 1, 2]


def test_tiles_ragged_and_empty_layers():
    cap = B.tile_capacity()
    check_tiles([0])
    check_tiles([0, 0, 0])
    check_tiles([0, 1])
    check_tiles([0, 1, 2, 3, 3, 3 + cap, 4 + 2 * cap, 4 + 2 * cap, 5 * cap + 17])
    rng = np.random.default_rng(0)
    sizes = rng.integers(0, 3 * cap, size=200)
    check_tiles(np.concatenate([[0], np.cumsum(sizes)]))


def test_tiles_bert_large():
    offs = W.offsets_from_sizes(W.bert_large_layer_sizes())
    t = check_tiles(offs)
    cap = B.tile_capacity()
    assert len(t) <= offs[-1] // cap + 2 * 391


def test_levels():
    assert B.plan_levels(1) == []
    assert B.plan_levels(2) == [2]
    assert B.plan_levels(64) == [16, 4]
    assert B.plan_levels(64, 2) == [2] * 6
    assert B.plan_levels(64, 8) == [8, 8]
    assert B.plan_levels(64, 4) == [4, 4, 4]
    assert B.plan_levels(128, 8) == [8, 8, 2]
    assert B.plan_levels(32, 8) == [8, 4]
    assert B.plan_levels(4, 8) == [4]
    assert B.plan_levels(64, 16) == [16, 4]
    assert B.plan_levels(128, 16) == [16, 8]
    assert B.plan_levels(8, 16) == [8]
    for K in (2, 4, 8, 16, 32, 64, 128, 256):
        for r in (2, 4, 8, 16):
            assert int(np.prod(B.plan_levels(K, r))) == K
    # any K: the first pass takes the sub-trees of the shallowest depth that fit the radix
    assert B.plan_levels(12) == [16]
    assert B.plan_levels(12, 8) == [8, 2]
    assert B.plan_levels(3, 2) == [2, 2]
    assert B.plan_levels(5, 2) == [2, 2, 2]
    assert B.plan_levels(6, 4) == [4, 2]
    assert B.plan_levels(33) == [16, 4]
    assert B.plan_levels(100, 8) == [8, 8, 2]
    with pytest.raises(B.AdasumError):
        B.plan_levels(8, 3)
    with pytest.raises(B.AdasumError):
        B.plan_levels(0)


def halving_tree(lo, hi, depth):
    """Nodes of the given depth of the Section 3.4 recursion, the left part taking
    floor(count / 2) workers: written as the recursion itself."""
    if depth == 0:
        return [(lo, hi)]
    mid = lo + (hi - lo) // 2
    return halving_tree(lo, mid, depth - 1) + halving_tree(mid, hi, depth - 1)


def test_first_pass_groups_are_sub_trees():
    for K in list(range(1, 70)) + [100, 127, 128, 129, 1000]:
        for radix in (2, 4, 8, 16):
            levels = B.plan_levels(K, radix)
            bounds = B.plan_groups(K, radix)
            G = len(bounds) - 1
            if K == 1:
                assert levels == [] and bounds == [0, 1]
                continue
            assert G * levels[0] == int(np.prod(levels))
            depth = int(np.log2(G))
            assert (1 << depth) == G
            want = halving_tree(0, K, depth)
            assert [(a, b) for a, b in zip(bounds[:-1], bounds[1:])] == want
            sizes = np.diff(bounds)
            assert sizes.min() >= 1 and sizes.max() <= levels[0] <= radix
            assert sizes.max() > levels[0] // 2 or levels[0] == 2, (K, radix, sizes, levels)
            # one level shallower would not fit the radix
            if depth > 0:
                assert max(b - a for a, b in halving_tree(0, K, depth - 1)) > radix


def test_linear_passes_cover_all_workers():
    import ctypes as C
    lib = B.load()
    # the schedule is visible through the workspace size only; check the arithmetic of the pass list here
    def passes(K, radix):
        first = radix
        while first > K:
            first //= 2
        out, rest = [first], K - first
        while rest > 0:
            r = radix
            while r - 1 > rest:
                r //= 2
            out.append(r)
            rest -= r - 1
        return out
    assert passes(64, 16) == [16, 16, 16, 16, 4]
    for K in (2, 3, 4, 5, 7, 8, 16, 21, 32, 64, 100, 128):
        for r in (2, 4, 8, 16):
            p = passes(K, r)
            assert p[0] + sum(x - 1 for x in p[1:]) == K
    # linear order needs one fp32 slot (the running result) whatever K and the radix are
    offs = [0, 1000, 5096, 70632]
    a = B.adasum_workspace_bytes(64, offs, B.BF16, radix=16)
    o = B.Options(); o.struct_bytes = C.sizeof(B.Options); o.out_dtype = -1; o.radix = 16; o.order = B.ORDER_LINEAR
    n = C.c_size_t(0)
    arr = (C.c_int64 * 4)(*offs)
    assert lib.adasum_workspace_bytes(64, arr, 3, B.BF16, C.byref(o), C.byref(n)) == B.OK
    assert 70656 * 4 <= n.value < 70656 * 4 + (1 << 20)
    assert n.value < a      # the tree order keeps K / radix = 4 nodes alive
