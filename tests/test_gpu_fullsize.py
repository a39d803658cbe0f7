"""Full-size parity: the configuration bench.py times (K = 64 workers,
BERT-Large shapes, bf16 gradients, 42.9 GB of input), checked against the CPU
oracle on sampled layers -- one per size class plus the 31 M-element embedding,
the first and the last layer -- and by properties that hold at any size.
"""
import numpy as np
import pytest
import torch

from paper_2006_02924_amd import binding as B
from paper_2006_02924_amd import workloads as W
from tests.gpu_util import (assert_bf16_rounding, assert_parity, oracle_after_optimizer, oracle_reduce, to_f64)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def config4():
    free, _ = torch.cuda.mem_get_info()
    if free < 150e9:
        pytest.skip("needs ~150 GB of free HBM")
    say("generating config 4 at full size")
    w = W.config4(DEV)
    torch.cuda.synchronize()
    yield w
    del w
    B.shutdown()
    torch.cuda.empty_cache()


def sampled_layers(w):
    sizes = np.diff(np.asarray(w.layer_offsets))
    picks = {0, w.n_layers - 1}
    for s in sorted(set(sizes.tolist())):
        picks.add(int(np.flatnonzero(sizes == s)[len(np.flatnonzero(sizes == s)) // 2]))
    return sorted(picks)


def test_config4_full_size_sampled_layers(config4):
    w = config4
    layers = sampled_layers(w)
    sizes = np.diff(np.asarray(w.layer_offsets))
    say(f"oracle on layers {layers} (sizes {[int(sizes[l]) for l in layers]})")
    ref = oracle_reduce(w.grads, w.layer_offsets, layers=layers)
    say("oracle done")
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    outs = {}
    # (radix, output, fuse_siblings, separate_passes): the default path (passes feed the next one), the same
    # with every pass reducing its own operands, the wide first passes (radix 64: a single pass; radix 32:
    # passes [32, 2]; Gram matrix from the matrix cores), and the three radix-2 schedules
    variants = ((0, torch.bfloat16, False, False), (0, torch.float32, False, False), (0, torch.bfloat16, False, True),
                (64, torch.bfloat16, False, False), (64, torch.float32, False, False), (32, torch.bfloat16, False, False),
                (2, torch.bfloat16, False, True), (2, torch.bfloat16, False, False), (2, torch.bfloat16, True, False))
    for radix, out_dtype, fuse, separate in variants:
        what = f"radix={radix} -> {out_dtype}{' (sibling-fused)' if fuse else ''}{' (separate passes)' if separate else ''}"
        say(f"adasum_reduce {what}")
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix, fuse_siblings=fuse,
                              separate_passes=separate,
                              layer_stats=stats if (radix == 0 and out_dtype == torch.float32) else None)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, layers=layers, what=f"config4 {what}")
        say(f"  max rel-L2 on sampled layers {err.max():.3e}")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, w.layer_offsets, layers=layers)
        assert bool(torch.isfinite(out).all())
        key = (radix, out_dtype, fuse, separate)
        outs[key] = out
        if radix == 2:
            B.shutdown()   # a radix-2 plan holds 43 GB of nodes
    # the same tree on every schedule: the bf16 results differ only in the few elements whose rounding the
    # last bits of the scalars decide
    base = outs[(0, torch.bfloat16, False, False)].float()
    for key, out in outs.items():
        if key[1] == torch.bfloat16 and key != (0, torch.bfloat16, False, False):
            differ = float((out.float() != base).float().mean())
            say(f"  {key}: bf16 output differs from the default path's in {differ:.2e} of the elements")
            assert differ < 1e-2
    # properties that hold for every layer: finite output; |Adasum(g1,g2)|^2 <= |g1|^2 + |g2|^2 at every
    # node, so the Section 3.6 metric is at most 1 (and positive here: the workers are positively
    # correlated); the default path rerun gives identical bits
    full = outs[(0, torch.float32, False, False)]
    assert bool(torch.isfinite(full).all())
    s = stats.cpu().numpy()
    metric = s[:, 0] / s[:, 1]
    assert np.all(metric <= 1.0 + 1e-5) and np.all(metric > 0.0), (metric.min(), metric.max())
    say(f"  orthogonality metric over layers: min {metric.min():.4f} max {metric.max():.4f}")
    again = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(again, outs[(0, torch.bfloat16, False, False)])
    # a single wide pass keeps no intermediate nodes, so even this workload fits the entry point that
    # allocates nothing (tables and 24 KB per span in the 64 MiB static array): the same bits
    quiet = torch.empty_like(again)
    B.adasum_reduce(w.grads, w.layer_offsets, out=quiet, radix=64, noalloc=True)
    torch.cuda.synchronize()
    assert torch.equal(quiet, outs[(64, torch.bfloat16, False, False)])
    B.shutdown()   # the cached plans' workspaces (43 GB at radix 2) go back before the next test


def test_config4_full_size_left_to_right_order(config4):
    """The left-to-right order (Section 3.4, first recursion) at full size: the kernels that take
    the running fp32 result next to fifteen bf16 leaves, on long Gram tiles."""
    w = config4
    layers = sampled_layers(w)
    say(f"oracle (left-to-right) on layers {layers}")
    ref = oracle_reduce(w.grads, w.layer_offsets, layers=layers, order="linear")
    say("oracle done")
    for out_dtype in (torch.bfloat16, torch.float32):
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, order=B.ORDER_LINEAR)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, layers=layers, what=f"config4 left-to-right {out_dtype}")
        say(f"  {out_dtype}: max rel-L2 on sampled layers {err.max():.3e}")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, w.layer_offsets, layers=layers)
        assert bool(torch.isfinite(out).all())
        again = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, order=B.ORDER_LINEAR)
        torch.cuda.synchronize()
        assert torch.equal(again, out)
        del out, again
    B.shutdown()


def test_config4_full_size_after_optimizer_form(config4):
    """Section 4.1's delta form at full size.  Starting parameters start = s_l N(0,1) per layer;
    worker k's parameters after its local step are start - 0.25 g_k (g_k: config 4's gradients),
    rounded to bf16.  The library subtracts start on the fly and adds it back at the root, also
    in place on the starting parameters."""
    w = config4
    free, _ = torch.cuda.mem_get_info()
    if free < 80e9:
        pytest.skip("needs ~80 GB of free HBM beside config 4")
    layers = sampled_layers(w)
    offs = w.layer_offsets
    gen = torch.Generator(device=DEV).manual_seed(404)
    reps = torch.tensor(np.diff(np.asarray(offs)), dtype=torch.int64)
    scale = torch.repeat_interleave(torch.tensor(w.meta["scale"], dtype=torch.float32), reps).to(DEV)
    start32 = torch.randn(w.N, generator=gen, device=DEV, dtype=torch.float32) * scale
    del scale
    start = start32.to(torch.bfloat16)
    start32 = start.float()
    currents = [(start32 - 0.25 * g.float()).to(torch.bfloat16) for g in w.grads]
    del start32
    torch.cuda.synchronize()
    say(f"oracle (after-optimizer form) on layers {layers}")
    ref = oracle_after_optimizer(start, currents, offs, layers)
    say("oracle done")
    out = B.adasum_reduce(currents, offs, delta_start=start)
    torch.cuda.synchronize()
    err = assert_parity(out, ref, offs, layers=layers, what="config4 delta form")
    say(f"  max rel-L2 of the new parameters on sampled layers {err.max():.3e}")
    assert_bf16_rounding(out, ref, offs, layers=layers)
    assert bool(torch.isfinite(out).all())
    param = start.clone()
    same = B.adasum_reduce(currents, offs, param, delta_start=param)
    torch.cuda.synchronize()
    assert same.data_ptr() == param.data_ptr() and torch.equal(param, out)
    del currents, out, param, start
    B.shutdown()
    torch.cuda.empty_cache()


def test_config3_full_size_sampled_layers():
    """K = 16 workers, fp32, BERT-Large shapes (21.4 GB of input): one radix-16 pass on long Gram
    tiles, fp32 and bf16 results, against the oracle on one layer per size class, the
    31 M-element embedding, the first and the last layer."""
    free, _ = torch.cuda.mem_get_info()
    if free < 60e9:
        pytest.skip("needs ~60 GB of free HBM")
    say("generating config 3 at full size")
    w = W.config3(DEV)
    torch.cuda.synchronize()
    layers = sampled_layers(w)
    say(f"oracle on layers {layers}")
    ref = oracle_reduce(w.grads, w.layer_offsets, layers=layers)
    say("oracle done")
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    for radix, out_dtype in ((0, torch.float32), (0, torch.bfloat16), (2, torch.float32)):
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix,
                              layer_stats=stats if (radix == 0 and out_dtype == torch.float32) else None)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, layers=layers, what=f"config3 radix {radix} {out_dtype}")
        say(f"  radix {radix} {out_dtype}: max rel-L2 on sampled layers {err.max():.3e}")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, w.layer_offsets, layers=layers)
        assert bool(torch.isfinite(out).all())
        if radix == 0 and out_dtype == torch.float32:
            again = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype)
            torch.cuda.synchronize()
            assert torch.equal(again, out)
            del again
        del out
    s = stats.cpu().numpy()
    metric = s[:, 0] / s[:, 1]
    assert np.all(metric <= 1.0 + 1e-5) and np.all(metric > 0.0), (metric.min(), metric.max())
    lin = B.adasum_reduce(w.grads, w.layer_offsets, order=B.ORDER_LINEAR)
    torch.cuda.synchronize()
    small = [l for l in layers if w.layer_offsets[l + 1] - w.layer_offsets[l] <= (1 << 22)]
    assert_parity(lin, oracle_reduce(w.grads, w.layer_offsets, layers=small, order="linear"), w.layer_offsets,
                  layers=small, what="config3 left-to-right")
    del w, lin
    B.shutdown()
    torch.cuda.empty_cache()


# Layers of 2^26 elements: more than 2048 long Gram tiles in all, which is what makes the planner
# choose them (a smaller table is cut into short tiles and runs other kernel instantiations).
LONG_TILE_SIZES = [7, 1 << 26, 4096, (1 << 26) + 3, 1 << 20, 1000]


@pytest.mark.parametrize("storage", ["fp16", "fp64"])
def test_other_storage_types_on_long_tiles(storage):
    """IEEE binary16 (K = 32: a radix-16 pass into fp32 nodes, then a pair pass) and fp64
    (K = 16: radix 8, then a pair pass, fp64 throughout) on a table big enough for the long
    Gram tiles that the timed runs use.  Checked against the oracle on every layer but one of
    the two 67 M-element ones; that one must be finite and repeat bit for bit."""
    from tests.gpu_util import TOL_F64
    free, _ = torch.cuda.mem_get_info()
    if free < 60e9:
        pytest.skip("needs ~60 GB of free HBM")
    sizes = LONG_TILE_SIZES
    assert sum(s // B.tile_capacity() for s in sizes) >= 2048
    if storage == "fp16":
        K = 32
        scales = W.log_uniform_scales(len(sizes), 78, lo_exp=-2.0, hi_exp=0.0)
        w = W.correlated_gaussian(sizes, K, dtype=torch.float16, device=DEV, seed=901, scale=scales)
        outs = (torch.float16, torch.float32)
    else:
        K = 16
        w = W.correlated_gaussian(sizes, K, dtype=torch.float32, device=DEV, seed=902)
        w.grads = [g.double() for g in w.grads]
        w.dtype = torch.float64
        outs = (torch.float64,)
    torch.cuda.synchronize()
    layers = [0, 1, 2, 4, 5]
    say(f"{storage}: K={K}, N={w.N}; oracle on layers {layers}")
    ref = oracle_reduce(w.grads, w.layer_offsets, layers=layers)
    say("oracle done")
    for out_dtype in outs:
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, layers=layers, what=f"{storage} -> {out_dtype}",
                            tol=TOL_F64 if storage == "fp64" else None)
        say(f"  {out_dtype}: max rel-L2 {err.max():.3e}")
        if out_dtype == torch.float16:
            assert_bf16_rounding(out, ref, w.layer_offsets, layers=layers)
        assert bool(torch.isfinite(out).all())
        again = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert torch.equal(again, out)
        del out, again
    small = [0, 2, 4, 5]
    lin = B.adasum_reduce(w.grads, w.layer_offsets, order=B.ORDER_LINEAR)
    torch.cuda.synchronize()
    assert_parity(lin, oracle_reduce(w.grads, w.layer_offsets, layers=small, order="linear"), w.layer_offsets,
                  layers=small, what=f"{storage} left-to-right", tol=TOL_F64 if storage == "fp64" else None)
    del w, lin
    B.shutdown()
    torch.cuda.empty_cache()


def test_config5_full_size_edge_layers():
    """K = 128 workers, bf16, BERT-Large shapes plus 16 one-element tensors and the
    degenerate layer kinds: every special layer (near-parallel, orthogonal pairs,
    all-orthogonal, zero, one-element) and one plain layer per size class is
    checked against the oracle; the 31 M-element embedding is left to the K = 64 test."""
    free, _ = torch.cuda.mem_get_info()
    if free < 200e9:
        pytest.skip("needs ~200 GB of free HBM")
    say("generating config 5 at full size")
    w = W.config5(DEV)
    torch.cuda.synchronize()
    offs = w.layer_offsets
    sizes = np.diff(np.asarray(offs))
    kinds = w.meta["kind"]
    layers = set()
    per_kind = {}
    for l, k in enumerate(kinds):
        if sizes[l] == 1:
            layers.add(l)
        elif k != "gauss" and sizes[l] <= (1 << 20):
            per_kind.setdefault((k, int(sizes[l])), []).append(l)
    for ls in per_kind.values():
        layers.update(ls[:2])
    for s in sorted(set(sizes.tolist())):
        if s <= (1 << 22):
            layers.add(int(np.flatnonzero((sizes == s) & (np.array(kinds) == "gauss"))[0])
                       if np.any((sizes == s) & (np.array(kinds) == "gauss")) else int(np.flatnonzero(sizes == s)[0]))
    layers = sorted(layers)
    say(f"oracle on {len(layers)} layers, {int(sizes[layers].sum())} elements x K={w.K}")
    ref = oracle_reduce(w.grads, offs, layers=layers)
    say("oracle done")
    # the default path (the first pass leaves the second one's 8 x 8 Gram matrix), and every pass on its own
    for radix, out_dtype, separate in ((0, torch.bfloat16, True), (0, torch.bfloat16, False), (0, torch.float32, False),
                                       (64, torch.bfloat16, False), (64, torch.float32, False)):
        out = B.adasum_reduce(w.grads, offs, out_dtype=out_dtype, radix=radix, separate_passes=separate)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, offs, layers=layers, what=f"config5 radix {radix} {out_dtype}")
        worst = int(np.argmax(err))
        say(f"  {out_dtype}{' (separate passes)' if separate else ''}: max rel-L2 {err.max():.3e} at layer {worst} "
            f"({kinds[worst]}, size {int(sizes[worst])})")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, offs, layers=layers)
    got = to_f64(out)
    for l, mode in w.meta["zero_modes"]:
        if mode == 0:
            assert np.all(got[offs[l]:offs[l + 1]] == 0.0)
    assert bool(torch.isfinite(out).all())
    del w
    B.shutdown()
    torch.cuda.empty_cache()


def test_buffers_longer_than_2_31_elements():
    """Element indices and byte offsets beyond 32 bits: K = 4 workers of 2^31 + 2^20 + 82 bf16
    elements each (4.3 GB per buffer).  Checked against the oracle: the first layer, the layer
    that straddles element 2^31, and every layer that starts beyond it; elsewhere the stored
    values must be finite and the rerun identical."""
    from oracle import adasum_oracle as O
    from tests.gpu_util import TOL_BF16, TOL_BF16_TINY, TINY_LAYER

    free, _ = torch.cuda.mem_get_info()
    if free < 60e9:
        pytest.skip("needs ~60 GB of free HBM")
    K = 4
    sizes = [(1 << 26) + 5] + [1 << 26] * 31 + [1 << 20, 77]
    offs = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    N = offs[-1]
    assert N > (1 << 31) and offs[32] > (1 << 31) > offs[31]
    gen = torch.Generator(device=DEV).manual_seed(77)
    say(f"generating K={K} x N={N} bf16")
    grads = []
    common = None
    for k in range(K + 1):
        g = torch.empty(N, dtype=torch.bfloat16, device=DEV)
        for l in range(len(sizes)):
            g[offs[l]:offs[l + 1]].normal_(generator=gen)
        if k == 0:
            common = g
        else:
            g.mul_(0.8).add_(common, alpha=0.6)    # positively correlated workers
            grads.append(g)
    del common
    torch.cuda.synchronize()
    outs = {}
    for out_dtype in (torch.bfloat16, torch.float32):
        say(f"adasum_reduce -> {out_dtype}")
        outs[out_dtype] = B.adasum_reduce(grads, offs, out_dtype=out_dtype)
        torch.cuda.synchronize()
    again = B.adasum_reduce(grads, offs, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(again, outs[torch.bfloat16])
    del again
    layers = [0, 31, 32, 33]
    for l in layers:
        lo, hi = offs[l], offs[l + 1]
        ref = O.adasum_tree([to_f64(g[lo:hi]) for g in grads])
        for out_dtype, out in outs.items():
            err = float(O.rel_l2_per_layer(to_f64(out[lo:hi]), ref, [0, hi - lo])[0])
            tol = 1e-5 if out_dtype == torch.float32 else (TOL_BF16 if hi - lo >= TINY_LAYER else TOL_BF16_TINY)
            say(f"  layer {l} [{lo}, {hi}) {out_dtype}: rel-L2 {err:.3e}")
            assert err <= tol, (l, out_dtype, err)
    for out in outs.values():
        for l in range(len(sizes)):
            assert bool(torch.isfinite(out[offs[l]:offs[l + 1]]).all()), l
    # the fp32 and bf16 outputs are one rounding apart everywhere, also in the layers without an oracle value
    for l in range(len(sizes)):
        a = outs[torch.float32][offs[l]:offs[l + 1]]
        b = outs[torch.bfloat16][offs[l]:offs[l + 1]].float()
        assert bool(((a - b).abs() <= a.abs() * 2.0 ** -8 + 1e-30).all()), l
    del grads, outs
    B.shutdown()
    torch.cuda.empty_cache()


def test_wide_first_pass_on_a_buffer_with_more_parts_than_workgroup_slots():
    """K = 32 workers of 2^30 + 4133 bf16 elements (2 GB per buffer, 69 GB in all), radix 32: the
    wide Gram pass keeps a part to 2^20 elements, so this buffer has 1024 parts -- more workgroups
    than the chip holds at once -- and one layer of 2^30 elements spans all of them.  The small layers
    against the oracle; the long one against the default schedule (the same tree: equal to the
    rounding of the scalars) and on a slice against the oracle's operator applied with the weights
    that the step entry points return."""
    from oracle import adasum_oracle as O

    free, _ = torch.cuda.mem_get_info()
    if free < 90e9:
        pytest.skip("needs ~90 GB of free HBM")
    K = 32
    sizes = [4096, 1 << 30, 37]
    offs = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    N = offs[-1]
    gen = torch.Generator(device=DEV).manual_seed(79)
    say(f"generating K={K} x N={N} bf16")
    common = torch.empty(N, dtype=torch.bfloat16, device=DEV).normal_(generator=gen)
    grads = []
    for k in range(K):
        g = torch.empty(N, dtype=torch.bfloat16, device=DEV).normal_(generator=gen)
        g.mul_(0.8).add_(common, alpha=0.6)    # positively correlated workers
        grads.append(g)
    del common
    torch.cuda.synchronize()
    assert B.plan_levels(K, 32) == [32]
    stats = torch.zeros(len(sizes), 2, dtype=torch.float64, device=DEV)
    wide = B.adasum_reduce(grads, offs, out_dtype=torch.float32, radix=32, layer_stats=stats)
    torch.cuda.synchronize()
    B.shutdown()
    base = B.adasum_reduce(grads, offs, out_dtype=torch.float32)
    torch.cuda.synchronize()
    B.shutdown()
    for l in (0, 2):
        lo, hi = offs[l], offs[l + 1]
        ref = O.adasum_tree([to_f64(g[lo:hi]) for g in grads])
        err = float(O.rel_l2_per_layer(to_f64(wide[lo:hi]), ref, [0, hi - lo])[0])
        say(f"  layer {l} [{lo}, {hi}): rel-L2 {err:.3e}")
        assert err <= 1e-5, (l, err)
    lo, hi = offs[1], offs[2]
    # the long layer: both schedules are the same linear combination of the leaves; compare on slices
    for a in (lo, lo + (1 << 29) - 1000, hi - 70000):
        x, y = to_f64(wide[a:a + 70000]), to_f64(base[a:a + 70000])
        d = float(np.linalg.norm(x - y) / np.linalg.norm(y))
        say(f"  long layer, slice at {a}: wide against default {d:.3e}")
        assert d <= 2e-6, (a, d)
    # its squared-norm statistics against a direct sum over the stored bits of one worker pair
    s = stats.cpu().numpy()
    leaves = sum(float((g[lo:hi].float() ** 2).sum(dtype=torch.float64)) for g in grads)
    assert abs(s[1, 1] - leaves) <= 2e-6 * leaves, (s[1, 1], leaves)
    root = float((wide[lo:hi].double() ** 2).sum())
    assert abs(s[1, 0] - root) <= 1e-5 * root, (s[1, 0], root)
    del wide, base, grads
    B.shutdown()
    torch.cuda.empty_cache()
