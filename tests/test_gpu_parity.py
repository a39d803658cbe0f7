"""GPU parity: the HIP library (through the C-ABI) against the fp64 CPU oracle,
element by element on the same stored inputs.

Tolerances (per layer, relative L2): 1e-5 for fp32 output, 2e-3 for bf16 output.
"""
import numpy as np
import pytest
import torch

from oracle import adasum_oracle as O
from paper_2006_02924_amd import binding as B
from paper_2006_02924_amd import workloads as W
from tests.gpu_util import (TOL_BF16, TOL_F32, assert_parity, assert_bf16_rounding, mark_ill_posed, oracle_reduce,
                            to_f64)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------
# step level
# ---------------------------------------------------------------------------

RAGGED = [0, 1, 2, 9, 9, 40, 41, 1064, 1064 + 16384, 1064 + 16384 + 33000, 60000, 60001]


# (32 and 64 operands: the wide first pass, 16-bit storage only, Gram blocks from the matrix cores)
_STEP_CASES = ([(R, dt) for R in (2, 4, 8, 16) for dt in (torch.float32, torch.bfloat16)] +
               [(R, dt) for R in (32, 64) for dt in (torch.bfloat16, torch.float16)])


@pytest.mark.parametrize("R,dtype", _STEP_CASES)
def test_group_gram_matches_dot_products(R, dtype):
    say(f"group_gram R={R} {dtype}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), R, dtype=dtype, device=DEV, seed=11)
    gram = B.adasum_group_gram(w.grads, w.layer_offsets)
    torch.cuda.synchronize()
    got = gram.cpu().numpy()
    X = np.stack([to_f64(g) for g in w.grads])
    for l in range(w.n_layers):
        lo, hi = RAGGED[l], RAGGED[l + 1]
        want = X[:, lo:hi] @ X[:, lo:hi].T
        scale = np.sqrt(np.outer(np.diag(want), np.diag(want))) + 1e-300
        assert np.max(np.abs(got[l] - want) / scale) < 2e-6, (l, got[l], want)
        if hi == lo:
            assert np.all(got[l] == 0.0)
    if R == 2:
        # Algorithm 1's triple [a.b, a.a, b.b] per layer
        lo, hi = RAGGED[-3], RAGGED[-2]
        d, n1, n2 = O.pair_scalars(X[0, lo:hi], X[1, lo:hi])
        np.testing.assert_allclose([got[-2][0, 1], got[-2][0, 0], got[-2][1, 1]], [d, n1, n2], rtol=2e-6)


@pytest.mark.parametrize("R", [2, 4, 8, 16, 32, 64])
def test_group_weights_reproduce_the_tree(R):
    say(f"group_weights R={R}")
    rng = np.random.default_rng(R)
    L, n = 12, 50
    X = rng.standard_normal((L, R, n))
    X[3, 1] = 0.0                      # a zero leaf
    X[4] = 0.0                         # an all-zero layer
    X[5, : R // 2] = 0.0               # a zero subtree
    X[6, 1] = -X[6, 0]                 # exactly cancelling siblings
    X[7] = X[7, 0]                     # all leaves identical
    G = np.einsum("lri,lsi->lrs", X, X)
    wt = B.adasum_group_weights(torch.from_numpy(G).to(DEV))
    torch.cuda.synchronize()
    wt = wt.cpu().numpy()
    assert wt.dtype == np.float64
    for l in range(L):
        want = O.adasum_tree([X[l, r] for r in range(R)])
        got = wt[l] @ X[l]
        den = np.linalg.norm(want)
        if den == 0:
            # weights that cancel in exact arithmetic; the host-side product rounds
            assert np.linalg.norm(got) <= 1e-12 * (1.0 + np.abs(wt[l]) @ np.linalg.norm(X[l], axis=1))
        else:
            assert np.linalg.norm(got - want) / den < 1e-6, l
    if R == 2:
        for l in (0, 1, 2):
            a, b = O.pair_coefficients(G[l, 0, 1], G[l, 0, 0], G[l, 1, 1])
            np.testing.assert_allclose(wt[l], [a, b], rtol=1e-13)
    # left-to-right order (Section 3.4, first recursion)
    wl = B.adasum_group_weights(torch.from_numpy(G).to(DEV), order=B.ORDER_LINEAR)
    torch.cuda.synchronize()
    wl = wl.cpu().numpy().astype(np.float64)
    for l in (0, 1, 2, 3, 5):
        want = O.adasum_linear([X[l, r] for r in range(R)])
        assert np.linalg.norm(wl[l] @ X[l] - want) / np.linalg.norm(want) < 1e-6


@pytest.mark.parametrize("R,dtype,out_dtype", [(R, dt, od) for R, dt in _STEP_CASES
                                               for od in ((torch.float32, dt) if dt != torch.float32
                                                          else (torch.float32, torch.bfloat16))])
def test_group_combine_matches_weighted_sum(R, dtype, out_dtype):
    say(f"group_combine R={R} {dtype}->{out_dtype}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), R, dtype=dtype, device=DEV, seed=12)
    L = w.n_layers
    wt = torch.randn(L, R, generator=torch.Generator().manual_seed(5), dtype=torch.float64).to(DEV)
    before = [g.clone() for g in w.grads]
    out, sq = B.adasum_group_combine(w.grads, w.layer_offsets, wt, out_dtype=out_dtype)
    torch.cuda.synchronize()
    for g, b in zip(w.grads, before):
        assert torch.equal(g, b), "inputs must not be modified"
    X = np.stack([to_f64(g) for g in w.grads])
    wt64 = wt.cpu().numpy().astype(np.float64)
    ref = np.zeros(w.N)
    for l in range(L):
        lo, hi = RAGGED[l], RAGGED[l + 1]
        ref[lo:hi] = wt64[l] @ X[:, lo:hi]
    assert_parity(out, ref, w.layer_offsets, tol=2e-6 if out_dtype == torch.float32 else
                  (1e-3 if out_dtype == torch.float16 else TOL_BF16))
    want_sq = np.array([np.dot(ref[RAGGED[l]:RAGGED[l + 1]], ref[RAGGED[l]:RAGGED[l + 1]]) for l in range(L)])
    np.testing.assert_allclose(sq.cpu().numpy(), want_sq, rtol=1e-5, atol=0)
    if out_dtype in (torch.bfloat16, torch.float16):
        assert_bf16_rounding(out, ref, w.layer_offsets)


def test_group_combine_in_place_on_first_operand():
    say("group_combine in place")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), 4, dtype=torch.float32, device=DEV, seed=13)
    wt = torch.rand(w.n_layers, 4, generator=torch.Generator().manual_seed(6), dtype=torch.float64).to(DEV)
    ref, _ = B.adasum_group_combine(w.grads, w.layer_offsets, wt)
    got, _ = B.adasum_group_combine(w.grads, w.layer_offsets, wt, out=w.grads[0])
    torch.cuda.synchronize()
    assert got.data_ptr() == w.grads[0].data_ptr()
    assert torch.equal(got, ref)
    # 64 operands, sixteen at a time: a lane still reads all of its element before it writes it
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), 64, dtype=torch.bfloat16, device=DEV, seed=14)
    wt = torch.rand(w.n_layers, 64, generator=torch.Generator().manual_seed(7), dtype=torch.float64).to(DEV)
    ref, _ = B.adasum_group_combine(w.grads, w.layer_offsets, wt)
    got, _ = B.adasum_group_combine(w.grads, w.layer_offsets, wt, out=w.grads[0])
    torch.cuda.synchronize()
    assert got.data_ptr() == w.grads[0].data_ptr()
    assert torch.equal(got, ref)


# ---------------------------------------------------------------------------
# whole tree
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("radix", [0, 2, 4, 8, 16])
def test_config1(radix):
    say(f"config1 radix={radix}")
    w = W.config1(DEV)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix)
    torch.cuda.synchronize()
    err = assert_parity(out, ref, w.layer_offsets, what=f"config1 radix {radix}")
    say(f"  max rel-L2 {err.max():.2e}")


def _k_radix(Ks, radices, lone):
    """Every (K, radix) pair, except that K = 1 (a copy: no passes, the radix plays no part) comes
    once, with radix `lone`."""
    return [(K, r) for K in Ks for r in radices if K > 1 or r == lone]


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K,radix", _k_radix([1, 2, 4, 8, 16, 32, 64], [2, 4, 8, 16], 2))
def test_ragged_tables(K, dtype, out_dtype, radix):
    say(f"ragged K={K} {dtype}->{out_dtype} radix={radix}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), K, dtype=dtype, device=DEV, seed=100 + K)
    before = [g.clone() for g in w.grads]
    ref = oracle_reduce(w.grads, w.layer_offsets)
    out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix)
    torch.cuda.synchronize()
    for g, b in zip(w.grads, before):
        assert torch.equal(g, b), "inputs must not be modified"
    assert_parity(out, ref, w.layer_offsets, what="ragged")
    if out_dtype == torch.bfloat16:
        assert_bf16_rounding(out, ref, w.layer_offsets)


# Layer sizes around the 256-element tiles of the 16-operand combine of 16-bit inputs (two operands per load
# instruction): tiles of 1 .. 32 granules, ragged heads and tails of 1 .. 7 elements on either side of a tile
# boundary, and layers that start at odd global offsets.
PAIR_EDGES = [255, 256, 257, 1, 7, 8, 9, 15, 16, 17, 511, 512, 513, 31, 33, 248, 264, 3, 1024, 2, 777, 4096 + 5]


@pytest.mark.parametrize("order", ["tree", "linear"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K", [16, 21, 64])
def test_tile_edges_of_the_paired_combine(K, dtype, order):
    say(f"pair edges K={K} {dtype} {order}")
    w = W.correlated_gaussian(PAIR_EDGES, K, dtype=dtype, device=DEV, seed=900 + K)
    ref = oracle_reduce(w.grads, w.layer_offsets, order=order)
    kw = dict(order=B.ORDER_LINEAR) if order == "linear" else {}
    out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.float32, radix=16, **kw)
    torch.cuda.synchronize()
    assert_parity(out, ref, w.layer_offsets, what=f"pair edges K={K} {order}")
    if order == "tree" and K == 64:
        # every pass on its own: the plain 16-operand combine instead of the one that feeds the next pass
        sep = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.float32, radix=16, separate_passes=True)
        torch.cuda.synchronize()
        assert_parity(sep, ref, w.layer_offsets, what=f"pair edges K={K} separate passes")
    # the result in the input's own type: one rounding of the same values
    low = B.adasum_reduce(w.grads, w.layer_offsets, radix=16, **kw)
    torch.cuda.synchronize()
    assert_parity(low, ref, w.layer_offsets, what=f"pair edges K={K} {order} -> {dtype}")


def test_empty_and_degenerate_tables():
    say("empty tables")
    for offs in ([0], [0, 0], [0, 0, 0, 5, 5], [0, 1], [0, 7, 7, 8]):
        N = offs[-1]
        g = [torch.randn(max(N, 1), device=DEV)[:N].contiguous() for _ in range(4)]
        if N == 0:
            g = [torch.empty(0, device=DEV) for _ in range(4)]
        out = B.adasum_reduce(g, offs)
        torch.cuda.synchronize()
        if N:
            assert_parity(out, oracle_reduce(g, offs), offs, what=str(offs))


@pytest.mark.parametrize("K,radix,dtype", [(K, radix, dt) for K, radix in [(8, 0), (8, 2), (64, 0), (5, 0)]
                                           for dt in (torch.float32, torch.bfloat16)] +
                         [(64, 64, torch.bfloat16), (40, 64, torch.bfloat16), (128, 32, torch.bfloat16)])
def test_nan_and_inf_stay_inside_their_layer(K, radix, dtype):
    """IEEE propagation: a NaN or an infinity in one worker's layer makes that layer's result
    NaN in every element (the scalars of the first node that sees it are NaN or Inf - Inf), in the
    oracle and in the library alike; every other layer is reduced as if nothing had happened."""
    say(f"non-finite inputs K={K} radix={radix} {dtype}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), K, dtype=dtype, device=DEV, seed=900 + K)
    offs = list(w.layer_offsets)
    poisoned = {2: (K - 1, 3, float("nan")),          # 7 elements: the small-layer path
                6: (min(3, K - 1), 500, float("nan")),
                7: (0, 16000, float("inf")),
                8: (K // 2, 0, float("-inf"))}
    for l, (k, e, v) in poisoned.items():
        assert offs[l + 1] - offs[l] > e
        w.grads[k][offs[l] + e] = v
    with np.errstate(all="ignore"):
        ref = O.adasum_reduce([to_f64(g) for g in w.grads], offs)
    for out_dtype in (dtype, torch.float32):
        out = B.adasum_reduce(w.grads, offs, out_dtype=out_dtype, radix=radix)
        torch.cuda.synchronize()
        got = to_f64(out)
        tol = TOL_BF16 if out_dtype == torch.bfloat16 else TOL_F32
        for l in range(len(offs) - 1):
            lo, hi = offs[l], offs[l + 1]
            if l in poisoned:
                assert np.isnan(ref[lo:hi]).all(), l
                assert np.isnan(got[lo:hi]).all(), (l, got[lo:hi][:8])
            elif hi > lo:
                assert np.isfinite(got[lo:hi]).all(), l
                err = O.rel_l2_per_layer(got[lo:hi], ref[lo:hi], [0, hi - lo])[0]
                assert err <= (tol if hi - lo >= 256 else max(tol, 2.0 ** -8 * 1.001 if out_dtype == torch.bfloat16 else tol)), (l, err)


def test_deterministic_and_workspace_from_caller():
    say("determinism")
    sizes = W.scaled_down(W.resnet50_layer_sizes(), 16, floor=3)
    w = W.correlated_gaussian(sizes, 8, dtype=torch.bfloat16, device=DEV, seed=21)
    a = B.adasum_reduce(w.grads, w.layer_offsets, radix=2)
    b = B.adasum_reduce(w.grads, w.layer_offsets, radix=2)
    nbytes = B.adasum_workspace_bytes(8, w.layer_offsets, B.BF16, radix=2)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    assert ws.data_ptr() % 256 == 0
    c = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)
    small = torch.empty(nbytes - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(w.grads, w.layer_offsets, radix=2, workspace=small)
    assert e.value.code == B.ERR_WORKSPACE


def test_layer_stats_orthogonality_metric():
    say("layer stats")
    # Section 3.6: |Adasum|^2 / sum |g_i|^2 is 1 for orthogonal and 1/K for identical gradients
    K, n = 8, 4096
    q, _ = torch.linalg.qr(torch.randn(n, K, dtype=torch.float64, generator=torch.Generator().manual_seed(1)))
    base = torch.randn(n, generator=torch.Generator().manual_seed(2))
    rnd = W.correlated_gaussian([3000], K, device="cpu", seed=3, corr=0.5)
    grads = []
    for i in range(K):
        grads.append(torch.cat([q[:, i].float() * (i + 1), base, rnd.grads[i]]).to(DEV))
    offs = [0, n, 2 * n, 2 * n + 3000]
    for radix in (2, 8, 16):
        stats = torch.zeros(3, 2, dtype=torch.float64, device=DEV)
        out = B.adasum_reduce(grads, offs, radix=radix, layer_stats=stats)
        torch.cuda.synchronize()
        s = stats.cpu().numpy()
        metric = s[:, 0] / s[:, 1]
        want = O.orthogonality([to_f64(g) for g in grads], offs)
        np.testing.assert_allclose(metric, want, rtol=1e-5)
        assert abs(metric[0] - 1.0) < 1e-5 and abs(metric[1] - 1.0 / K) < 1e-5
        got = to_f64(out)
        np.testing.assert_allclose(s[:, 0], [got[offs[l]:offs[l + 1]] @ got[offs[l]:offs[l + 1]] for l in range(3)],
                                   rtol=1e-5)


def test_config2_resnet50_full():
    say("config2 (K=8, fp32, ResNet-50 shapes, full size)")
    w = W.config2(DEV)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    for radix in (2, 8, 16):
        out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, what=f"config2 radix {radix}")
        say(f"  radix {radix}: max rel-L2 {err.max():.2e}")


def test_config3_bert_fp32_scaled():
    say("config3 (K=16, fp32, BERT-Large shapes / 16)")
    sizes = W.scaled_down(W.bert_large_layer_sizes(), 16, floor=64)
    w = W.config3(DEV, sizes=sizes)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    for radix in (2, 4, 8, 16):
        out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, what=f"config3 radix {radix}")
        say(f"  radix {radix}: max rel-L2 {err.max():.2e}")


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_config4_bert_bf16_scaled(out_dtype):
    say(f"config4 (K=64, bf16->{out_dtype}, BERT-Large shapes / 32)")
    sizes = W.scaled_down(W.bert_large_layer_sizes(), 32, floor=32)
    w = W.config4(DEV, sizes=sizes)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    for radix in (2, 4, 8, 16):
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, what=f"config4 radix {radix}")
        say(f"  radix {radix}: max rel-L2 {err.max():.2e}")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, w.layer_offsets)


def test_config5_edge_cases_scaled():
    say("config5 (K=128, bf16, degenerate layers, BERT-Large shapes / 64)")
    sizes = W.scaled_down(W.bert_large_layer_sizes(), 64, floor=16)
    w = W.config5(DEV, sizes=sizes)
    offs = w.layer_offsets
    ref = oracle_reduce(w.grads, offs)
    kinds = w.meta["kind"]
    for radix in (2, 8, 16):
        for out_dtype in (torch.bfloat16, torch.float32):
            out = B.adasum_reduce(w.grads, offs, out_dtype=out_dtype, radix=radix)
            torch.cuda.synchronize()
            err = assert_parity(out, ref, offs, what=f"config5 radix {radix} {out_dtype}")
            say(f"  radix {radix} {out_dtype}: max rel-L2 {err.max():.2e} at layer {int(err.argmax())} "
                f"({kinds[int(err.argmax())]}, size {offs[int(err.argmax()) + 1] - offs[int(err.argmax())]})")
    got = to_f64(out)
    for l, k in enumerate(kinds):
        lo, hi = offs[l], offs[l + 1]
        if hi - lo == 1:
            # one-element layer: collinear operands everywhere => arithmetic mean of the K scalars
            vals = np.array([float(g[lo]) for g in w.grads])
            if np.all(vals != 0):
                assert abs(got[lo] - ref[lo]) <= 1e-5 * abs(ref[lo])
    for l, mode in w.meta["zero_modes"]:
        if mode == 0:
            assert np.all(got[offs[l]:offs[l + 1]] == 0.0)


def test_graph_replay_matches_eager():
    say("hipGraph replay vs eager launches")
    sizes = W.scaled_down(W.resnet50_layer_sizes(), 16, floor=3)
    # floor=3 leaves many layers of 3..16 elements: the small-layer kernels are part of the graph;
    # K = 6 and 100 have short first-pass groups; fp64 uses its own node type
    for K, dtype, radix in ((8, torch.bfloat16, 0), (64, torch.float32, 16), (4, torch.float32, 2), (1, torch.bfloat16, 0),
                            (6, torch.bfloat16, 4), (100, torch.float16, 0), (16, torch.float64, 0)):
        w = W.correlated_gaussian(sizes, K, dtype=torch.float32 if dtype == torch.float64 else dtype, device=DEV,
                                  seed=31 + K)
        if dtype == torch.float64:
            w.grads = [g.double() for g in w.grads]
        stats_e = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
        stats_g = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
        out_e = torch.empty(w.N, dtype=dtype, device=DEV)
        out_g = torch.empty(w.N, dtype=dtype, device=DEV)
        for rep in range(4):
            # eager work between replays: new values in the same buffers
            for i, g in enumerate(w.grads):
                g.mul_(1.0 + 0.25 * ((i + rep) % 3)).add_(0.01 * rep)
            torch.cuda.synchronize()
            B.adasum_reduce(w.grads, w.layer_offsets, out_e, radix=radix, layer_stats=stats_e)
            B.adasum_reduce(w.grads, w.layer_offsets, out_g, radix=radix, layer_stats=stats_g, use_graph=True)
            torch.cuda.synchronize()
            assert torch.equal(out_e, out_g), (K, dtype, rep)
            assert torch.equal(stats_e, stats_g), (K, dtype, rep)
        # other buffers: a second graph is captured, the first one stays valid
        other = [g.clone() for g in w.grads]
        out_o = torch.empty_like(out_g)
        B.adasum_reduce(other, w.layer_offsets, out_o, radix=radix, use_graph=True)
        B.adasum_reduce(w.grads, w.layer_offsets, out_g, radix=radix, layer_stats=stats_g, use_graph=True)
        torch.cuda.synchronize()
        assert torch.equal(out_o, out_e) and torch.equal(out_g, out_e)
        ref = oracle_reduce(w.grads, w.layer_offsets)
        assert_parity(out_g, ref, w.layer_offsets, what=f"graph K={K}")


@pytest.mark.parametrize("K,radix", _k_radix([1, 2, 16, 64], [2, 8, 16], 2))
def test_fp16_storage(K, radix):
    """IEEE binary16 gradients (the low-precision format of Section 4.4.1), fp16 and fp32 results."""
    say(f"fp16 K={K} radix={radix}")
    sizes = np.diff(RAGGED).tolist()
    scales = W.log_uniform_scales(len(sizes), 77, lo_exp=-2.0, hi_exp=0.0)
    w = W.correlated_gaussian(sizes, K, dtype=torch.float16, device=DEV, seed=300 + K, scale=scales)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    for out_dtype in (torch.float16, torch.float32):
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix)
        torch.cuda.synchronize()
        assert out.dtype == out_dtype
        assert_parity(out, ref, w.layer_offsets, what=f"fp16->{out_dtype}")
        if out_dtype == torch.float16:
            assert_bf16_rounding(out, ref, w.layer_offsets)
    # fp32 gradients stored to fp16
    w32 = W.correlated_gaussian(sizes, K, dtype=torch.float32, device=DEV, seed=300 + K, scale=scales)
    out = B.adasum_reduce(w32.grads, w32.layer_offsets, out_dtype=torch.float16, radix=radix)
    torch.cuda.synchronize()
    ref32 = oracle_reduce(w32.grads, w32.layer_offsets)
    assert_parity(out, ref32, w32.layer_offsets, what="f32->fp16")
    assert_bf16_rounding(out, ref32, w32.layer_offsets)


def test_unsupported_dtype_pairs():
    g = [torch.zeros(64, dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(g, [0, 64], out_dtype=torch.float16)
    assert e.value.code == B.ERR_UNSUPPORTED


def test_fp16_step_entry_points():
    say("fp16 group steps")
    sizes = np.diff(RAGGED).tolist()
    w = W.correlated_gaussian(sizes, 16, dtype=torch.float16, device=DEV, seed=41)
    gram = B.adasum_group_gram(w.grads, w.layer_offsets)
    torch.cuda.synchronize()
    X = np.stack([to_f64(g) for g in w.grads])
    got = gram.cpu().numpy()
    for l in range(w.n_layers):
        lo, hi = RAGGED[l], RAGGED[l + 1]
        want = X[:, lo:hi] @ X[:, lo:hi].T
        scale = np.sqrt(np.outer(np.diag(want), np.diag(want))) + 1e-300
        assert np.max(np.abs(got[l] - want) / scale) < 2e-6, l


@pytest.mark.parametrize("radix", [2, 4, 16])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K", [2, 4, 8, 32, 64])
def test_linear_order(K, dtype, radix):
    """Left-to-right application (Section 3.4, first recursion): a different result from the tree."""
    say(f"linear order K={K} {dtype} radix={radix}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), K, dtype=dtype, device=DEV, seed=500 + K)
    host = [to_f64(g) for g in w.grads]
    ref = mark_ill_posed(O.adasum_reduce(host, w.layer_offsets, order="linear"), host, list(w.layer_offsets),
                         "linear")
    before = [g.clone() for g in w.grads]
    out = B.adasum_reduce(w.grads, w.layer_offsets, order=B.ORDER_LINEAR, radix=radix)
    torch.cuda.synchronize()
    for g, b in zip(w.grads, before):
        assert torch.equal(g, b)
    assert_parity(out, ref, w.layer_offsets, what="linear")
    if K > 2:
        tree = O.adasum_reduce(host, w.layer_offsets)
        big = len(RAGGED) - 4   # a layer of thousands of elements
        lo, hi = RAGGED[big], RAGGED[big + 1]
        assert np.linalg.norm(tree[lo:hi] - ref[lo:hi]) > 1e-3 * np.linalg.norm(ref[lo:hi])
    out32 = B.adasum_reduce(w.grads, w.layer_offsets, order=B.ORDER_LINEAR, radix=radix, out_dtype=torch.float32,
                            use_graph=True)
    torch.cuda.synchronize()
    assert_parity(out32, ref, w.layer_offsets, what="linear f32 out, graph")
    # the statistics of Section 3.6 in this order: the fold's squared norm and every leaf's, once
    stats = torch.full((w.n_layers, 2), -1.0, dtype=torch.float64, device=DEV)
    again = B.adasum_reduce(w.grads, w.layer_offsets, order=B.ORDER_LINEAR, radix=radix, layer_stats=stats)
    torch.cuda.synchronize()
    assert torch.equal(again, out)
    s = stats.cpu().numpy()
    offs = w.layer_offsets
    for l in range(w.n_layers):
        lo, hi = offs[l], offs[l + 1]
        if hi == lo:
            continue
        leaves = sum(float(np.dot(g[lo:hi], g[lo:hi])) for g in host)
        assert s[l, 1] == pytest.approx(leaves, rel=2e-6)
        if not np.isnan(ref[lo:hi]).any():
            assert s[l, 0] == pytest.approx(float(np.dot(ref[lo:hi], ref[lo:hi])), rel=1e-2 if dtype != torch.float32 else 1e-4,
                                            abs=1e-30)


# ---------------------------------------------------------------------------
# Adasum applied after the optimizer (Section 4.1): effective gradients formed on the fly
# ---------------------------------------------------------------------------

def _check_after_optimizer(out, start, currents, offs, what):
    """`out` against the oracle's new parameters, and -- sharper -- the step it took,
    out - start, against the oracle's combined effective gradient."""
    w0 = to_f64(start)
    cur = [to_f64(c) for c in currents]
    ref = mark_ill_posed(O.adasum_after_optimizer(w0, cur, offs), [c - w0 for c in cur], list(offs))
    assert_parity(out, ref, offs, what=what)
    if out.dtype != torch.float32:
        assert_bf16_rounding(out, ref, offs)
        return ref
    got = to_f64(out)
    for l in range(len(offs) - 1):
        lo, hi = offs[l], offs[l + 1]
        if hi == lo:
            continue
        if np.isnan(ref[lo:hi]).all():
            continue
        step_ref = ref[lo:hi] - w0[lo:hi]
        err = np.linalg.norm((got[lo:hi] - w0[lo:hi]) - step_ref)
        # the combined step to the fp32 bar, plus one fp32 rounding of the stored sum
        bound = TOL_F32 * np.linalg.norm(step_ref) + 2.0 ** -24 * np.linalg.norm(ref[lo:hi])
        assert err <= bound, f"{what}: layer {l} step error {err:.3e} > {bound:.3e}"
    return ref


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K,radix", _k_radix([1, 2, 8, 16, 64], [0, 2, 4, 16], 0))
def test_after_optimizer_delta_form(K, dtype, radix):
    say(f"delta form K={K} {dtype} radix={radix}")
    sizes = np.diff(RAGGED).tolist()
    scales = W.log_uniform_scales(len(sizes), 5, lo_exp=-2.0, hi_exp=0.0)
    w = W.after_local_step(sizes, K, dtype=dtype, device=DEV, seed=400 + K, scale=scales, step=0.25)
    start = w.meta["start"]
    before = [g.clone() for g in w.grads] + [start.clone()]
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, delta_start=start)
    torch.cuda.synchronize()
    for g, b in zip(w.grads + [start], before):
        assert torch.equal(g, b), "inputs must not be modified"
    _check_after_optimizer(out, start, w.grads, w.layer_offsets, f"delta K={K} {dtype} radix={radix}")


def test_after_optimizer_in_place_stats_and_graph():
    """`out` may be the starting parameters themselves; layer_stats describe the
    effective gradients; a graph replay gives the eager bits."""
    sizes = W.scaled_down(W.bert_large_layer_sizes(), 64, floor=1)
    K = 16
    w = W.after_local_step(sizes, K, dtype=torch.float32, device=DEV, seed=9, step=0.1)
    start = w.meta["start"]
    offs = w.layer_offsets
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    out = B.adasum_reduce(w.grads, offs, delta_start=start, layer_stats=stats)
    torch.cuda.synchronize()
    _check_after_optimizer(out, start, w.grads, offs, "delta bert/64")
    w0 = to_f64(start)
    deltas = [to_f64(c) - w0 for c in w.grads]
    metric = O.orthogonality(deltas, offs)
    s = stats.cpu().numpy()
    np.testing.assert_allclose(s[:, 0] / s[:, 1], metric, rtol=2e-5)
    np.testing.assert_allclose(s[:, 1], [sum(float(np.dot(d[a:b], d[a:b])) for d in deltas)
                                         for a, b in zip(offs[:-1], offs[1:])], rtol=1e-6)
    for _ in range(3):
        again = B.adasum_reduce(w.grads, offs, delta_start=start, use_graph=True)
        torch.cuda.synchronize()
        assert torch.equal(again, out)
    params = start.clone()
    same = B.adasum_reduce(w.grads, offs, params, delta_start=params)
    torch.cuda.synchronize()
    assert same.data_ptr() == params.data_ptr()
    assert torch.equal(params, out)
    # refused: another output type, the left-to-right order
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(w.grads, offs, delta_start=start, out_dtype=torch.bfloat16)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(w.grads, offs, delta_start=start, order=B.ORDER_LINEAR)
    assert e.value.code == B.ERR_UNSUPPORTED


# ---------------------------------------------------------------------------
# worker counts that are not a power of two (Section 3.4's recursion, the left
# part taking floor(K/2) workers): short first-pass groups
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("radix", [0, 2, 4, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K", [3, 5, 6, 7, 9, 12, 17, 33, 48, 100])
def test_any_worker_count(K, dtype, radix):
    say(f"K={K} {dtype} radix={radix} levels={B.plan_levels(K, radix)} groups={B.plan_groups(K, radix)}")
    w = W.correlated_gaussian(np.diff(RAGGED).tolist(), K, dtype=dtype, device=DEV, seed=500 + K)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, layer_stats=stats)
    torch.cuda.synchronize()
    assert_parity(out, ref, w.layer_offsets, what=f"K={K}")
    if dtype == torch.bfloat16:
        assert_bf16_rounding(out, ref, w.layer_offsets)
        out32 = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert_parity(out32, ref, w.layer_offsets, what=f"K={K} -> f32")
    # the statistics count every worker once (padding operands are not workers)
    f64 = [to_f64(g) for g in w.grads]
    offs = w.layer_offsets
    s = stats.cpu().numpy()
    for l in range(w.n_layers):
        lo, hi = offs[l], offs[l + 1]
        if hi > lo:
            assert s[l, 1] == pytest.approx(sum(float(np.dot(g[lo:hi], g[lo:hi])) for g in f64), rel=1e-6)
        if hi > lo and not np.isnan(ref[lo:hi]).any():
            assert s[l, 0] == pytest.approx(float(np.dot(ref[lo:hi], ref[lo:hi])), rel=1e-3, abs=1e-30)


@pytest.mark.parametrize("K", [3, 6, 21])
def test_any_worker_count_linear_and_delta(K):
    sizes = np.diff(RAGGED).tolist()
    w = W.correlated_gaussian(sizes, K, dtype=torch.bfloat16, device=DEV, seed=600 + K)
    for radix in (2, 4, 16):
        say(f"K={K} linear radix={radix}")
        ref = oracle_reduce(w.grads, w.layer_offsets, order="linear")
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.float32, radix=radix, order=B.ORDER_LINEAR)
        torch.cuda.synchronize()
        assert_parity(out, ref, w.layer_offsets, what=f"K={K} linear")
    say(f"K={K} delta form")
    scales = W.log_uniform_scales(len(sizes), 5, lo_exp=-2.0, hi_exp=0.0)
    d = W.after_local_step(sizes, K, dtype=torch.float32, device=DEV, seed=700 + K, scale=scales, step=0.25)
    for radix in (0, 2):
        out = B.adasum_reduce(d.grads, d.layer_offsets, radix=radix, delta_start=d.meta["start"])
        torch.cuda.synchronize()
        _check_after_optimizer(out, d.meta["start"], d.grads, d.layer_offsets, f"delta K={K} radix={radix}")


@pytest.mark.parametrize("order", ["tree", "linear"])
@pytest.mark.parametrize("K", [2, 7, 16, 64, 200])
def test_small_layers_follow_the_definition_in_fp64(K, order):
    """Layers of at most 16 elements are reduced pair by pair in fp64 (nothing stored in
    between), so even workers that nearly cancel at every tree node -- where an fp32 node
    would lose 1/eps digits -- come out to fp32 rounding."""
    say(f"small layers K={K} {order}")
    sizes = [1, 1, 2, 3, 16, 4096, 5, 1]
    offs = W.offsets_from_sizes(sizes)
    g = torch.Generator().manual_seed(900 + K)
    base = torch.randn(offs[-1], generator=g, dtype=torch.float64)
    grads = []
    for k in range(K):
        x = base * (1.0 + 1e-4 * torch.randn(offs[-1], generator=g, dtype=torch.float64))
        if k % 2:                       # odd workers point the other way: every pair nearly cancels
            x = -x
        x[offs[5]:offs[6]] = torch.randn(sizes[5], generator=g, dtype=torch.float64)   # the large layer: ordinary
        grads.append(x.float().to(DEV))
    f64 = [to_f64(t) for t in grads]
    ref = mark_ill_posed(O.adasum_reduce(f64, offs, order=order), f64, offs, order)
    code = B.ORDER_TREE if order == "tree" else B.ORDER_LINEAR
    for radix in (2, 16):
        out = B.adasum_reduce(grads, offs, radix=radix, order=code)
        torch.cuda.synchronize()
        got = to_f64(out)
        for l, n in enumerate(sizes):
            lo, hi = offs[l], offs[l + 1]
            if np.isnan(ref[lo:hi]).any():
                continue
            err = np.linalg.norm(got[lo:hi] - ref[lo:hi]) / np.linalg.norm(ref[lo:hi])
            # fp32 store (6e-8) plus fp64 noise amplified by the cancellations
            assert err <= (1e-6 if n <= 16 else TOL_F32), f"layer {l} (size {n}) radix {radix}: {err:.3e}"


# ---------------------------------------------------------------------------
# fp64 storage (the paper's dtype list: Section 4.4.1 names fp16, fp32 and fp64): reduced in fp64
# ---------------------------------------------------------------------------

def _fp64_workload(sizes, K, seed):
    """The correlated-Gaussian recipe drawn in fp32 and widened, plus an fp64 perturbation so
    that the values use the whole fp64 significand."""
    w = W.correlated_gaussian(sizes, K, dtype=torch.float32, device=DEV, seed=seed)
    g = torch.Generator(device=DEV).manual_seed(seed + 17)
    grads = [x.double() * (1.0 + 1e-9 * torch.randn(w.N, generator=g, device=DEV, dtype=torch.float64))
             for x in w.grads]
    return W.Workload("fp64", K, torch.float64, w.layer_offsets, grads, w.meta)


@pytest.mark.parametrize("K,radix", _k_radix([1, 2, 5, 16, 64], [0, 2, 4, 8], 0))
def test_fp64_storage(K, radix):
    say(f"fp64 K={K} radix={radix}")
    w = _fp64_workload(np.diff(RAGGED).tolist(), K, 800 + K)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, layer_stats=stats)
    torch.cuda.synchronize()
    assert out.dtype == torch.float64
    err = assert_parity(out, ref, w.layer_offsets, what=f"fp64 K={K}")
    say(f"  max rel-L2 {err.max():.2e}")
    if K > 1:
        lin = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, order=B.ORDER_LINEAR)
        torch.cuda.synchronize()
        assert_parity(lin, oracle_reduce(w.grads, w.layer_offsets, order="linear"), w.layer_offsets,
                      what=f"fp64 linear K={K}")
    metric = O.orthogonality([to_f64(g) for g in w.grads], w.layer_offsets)
    s = stats.cpu().numpy()
    ok = ~np.isnan(metric) & ~np.isnan([ref[a] if b > a else np.nan
                                        for a, b in zip(w.layer_offsets[:-1], w.layer_offsets[1:])])
    with np.errstate(invalid="ignore"):
        got_metric = s[:, 0] / s[:, 1]
    np.testing.assert_allclose(got_metric[ok], metric[ok], rtol=1e-9)


def test_fp64_delta_form_and_limits():
    sizes = np.diff(RAGGED).tolist()
    d = W.after_local_step(sizes, 8, dtype=torch.float32, device=DEV, seed=41, step=0.25)
    start = d.meta["start"].double()
    cur = [c.double() for c in d.grads]
    out = B.adasum_reduce(cur, d.layer_offsets, delta_start=start)
    torch.cuda.synchronize()
    w0 = to_f64(start)
    cur64 = [to_f64(c) for c in cur]
    ref = mark_ill_posed(O.adasum_after_optimizer(w0, cur64, d.layer_offsets), [c - w0 for c in cur64],
                         list(d.layer_offsets))
    assert_parity(out, ref, d.layer_offsets, what="fp64 delta")
    # fp64 goes only to fp64, and at most 8 workers per pass
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(cur, d.layer_offsets, out_dtype=torch.float32)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(cur, d.layer_offsets, radix=16)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce([c.float() for c in cur], d.layer_offsets, out_dtype=torch.float64)
    assert e.value.code == B.ERR_UNSUPPORTED


def test_plan_cache_is_bounded_and_evicts_safely():
    """More distinct layer tables than the library keeps plans for: old plans are dropped
    (their device memory freed) while results stay right, also for a table seen again."""
    g = torch.Generator().manual_seed(5)
    a = torch.randn(4000, generator=g).to(DEV)
    b = torch.randn(4000, generator=g).to(DEV)
    ref_of = {}
    for rep in range(2):
        for n in range(100, 100 + 80):
            offs = [0, n, 2 * n + 7, 4000]
            out = B.adasum_reduce([a, b], offs)
            if n not in ref_of:
                ref_of[n] = oracle_reduce([a, b], offs)
            torch.cuda.synchronize()
            assert_parity(out, ref_of[n], offs, what=f"table {n}")


@pytest.mark.parametrize("radix", [0, 2])
@pytest.mark.parametrize("K", [129, 257, 1000, 1024])
def test_many_workers(K, radix):
    """More workers than one launch carries operand pointers for (128): batched launches, deep trees."""
    say(f"many workers K={K} radix={radix} levels={B.plan_levels(K, radix)}")
    sizes = [1, 40, 3000, 7, 20000]
    w = W.correlated_gaussian(sizes, K, dtype=torch.float32, device=DEV, seed=1000 + K, corr=0.3)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, layer_stats=stats)
    torch.cuda.synchronize()
    err = assert_parity(out, ref, w.layer_offsets, what=f"K={K}")
    say(f"  max rel-L2 {err.max():.2e}")
    f64 = [to_f64(g) for g in w.grads]
    s = stats.cpu().numpy()
    offs = w.layer_offsets
    for l in range(w.n_layers):
        assert s[l, 1] == pytest.approx(sum(float(np.dot(g[offs[l]:offs[l + 1]], g[offs[l]:offs[l + 1]]))
                                            for g in f64), rel=1e-6)
    lin = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, order=B.ORDER_LINEAR)
    torch.cuda.synchronize()
    assert_parity(lin, oracle_reduce(w.grads, w.layer_offsets, order="linear"), w.layer_offsets, what=f"K={K} linear")


def test_caller_owned_plans():
    """adasum_plan_create / execute / destroy give the bits of adasum_reduce_ex, execute after
    execute, with new values in the same buffers, the plan's own or a caller's workspace,
    statistics per execute, the delta form, and graph replay."""
    sizes = np.diff(RAGGED).tolist()
    for K, dtype, radix, order in ((8, torch.bfloat16, 0, B.ORDER_TREE), (5, torch.float32, 4, B.ORDER_TREE),
                                   (16, torch.float16, 0, B.ORDER_LINEAR), (64, torch.float64, 0, B.ORDER_TREE)):
        say(f"plan K={K} {dtype} radix={radix} order={order}")
        w = W.correlated_gaussian(sizes, K, dtype=torch.float32 if dtype == torch.float64 else dtype, device=DEV,
                                  seed=40 + K)
        if dtype == torch.float64:
            w.grads = [g.double() for g in w.grads]
        plan = B.Plan(K, w.layer_offsets, dtype, radix=radix, order=order)
        assert plan.workspace_bytes() == B.adasum_workspace_bytes(K, w.layer_offsets, B._code_of(dtype), radix=radix,
                                                                  order=order)
        ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=DEV)
        ws = ws[(-ws.data_ptr()) % 256:][:plan.workspace_bytes()]
        plan_ws = B.Plan(K, w.layer_offsets, dtype, radix=radix, order=order, workspace=ws, use_graph=True)
        for rep in range(3):
            for i, g in enumerate(w.grads):
                g.mul_(1.0 + 0.5 * ((i + rep) % 2))
            want = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, order=order)
            got = plan.execute(w.grads)
            got_ws = plan_ws.execute(w.grads)
            torch.cuda.synchronize()
            assert torch.equal(got, want) and torch.equal(got_ws, want), (K, dtype, rep)
        if order == B.ORDER_TREE:
            stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
            stats_want = torch.zeros_like(stats)
            B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, layer_stats=stats_want)
            plan.execute(w.grads, layer_stats=stats)
            torch.cuda.synchronize()
            assert torch.equal(stats, stats_want)
        with pytest.raises(B.AdasumError):
            plan.execute(w.grads, delta_start=w.grads[0].clone())
        plan.destroy()
        plan_ws.destroy()
    d = W.after_local_step(sizes, 8, dtype=torch.float32, device=DEV, seed=77, step=0.25)
    plan = B.Plan(8, d.layer_offsets, torch.float32, delta=True)
    want = B.adasum_reduce(d.grads, d.layer_offsets, delta_start=d.meta["start"])
    got = plan.execute(d.grads, delta_start=d.meta["start"])
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    with pytest.raises(B.AdasumError):
        plan.execute(d.grads)
    plan.destroy()


@pytest.mark.parametrize("K,dtype,order", [(64, torch.bfloat16, B.ORDER_TREE), (6, torch.float32, B.ORDER_TREE),
                                            (20, torch.bfloat16, B.ORDER_LINEAR)])
def test_plan_execute_inside_the_callers_graph(K, dtype, order):
    """adasum_plan_execute only launches kernels (tables and workspace exist since plan creation), so
    a caller can record it into a graph of its own; every replay, with new values in the same
    buffers and eager work in between, gives the bits of an eager call."""
    say(f"execute under the caller's capture: K={K} {dtype} order={order}")
    sizes = np.diff(RAGGED).tolist()
    w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=60 + K)
    plan = B.Plan(K, w.layer_offsets, dtype, order=order)
    out = torch.zeros(w.N, dtype=dtype, device=DEV)
    stats = torch.zeros(w.n_layers, 2, dtype=torch.float64, device=DEV)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        plan.execute(w.grads, out, layer_stats=stats)
    torch.cuda.synchronize()
    for rep in range(3):
        for i, g in enumerate(w.grads):
            g.mul_(1.0 + 0.25 * ((i + rep) % 3))
        want_stats = torch.zeros_like(stats)
        want = B.adasum_reduce(w.grads, w.layer_offsets, order=order, layer_stats=want_stats)
        out.zero_()
        stats.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), (K, dtype, rep)
        assert torch.equal(stats, want_stats), (K, dtype, rep)
    del graph
    plan.destroy()


def test_two_host_threads_on_their_own_streams():
    """Calls from two host threads (ctypes releases the GIL), each with its own shape -- hence its
    own plan and workspace -- and its own stream: results stay right and deterministic."""
    import threading
    jobs = []
    for K, seed in ((8, 1), (5, 2)):
        w = W.correlated_gaussian(np.diff(RAGGED).tolist()[: 8 + K % 3], K, dtype=torch.bfloat16, device=DEV, seed=70 + seed)
        jobs.append((w, oracle_reduce(w.grads, w.layer_offsets), torch.cuda.Stream(device=DEV)))
    torch.cuda.synchronize()
    errors = []

    def work(job):
        w, ref, stream = job
        try:
            first = None
            for _ in range(25):
                out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.float32, stream=stream)
                stream.synchronize()
                if first is None:
                    first = out.clone()
                    assert_parity(out, ref, w.layer_offsets, what=f"thread K={w.K}")
                else:
                    assert torch.equal(out, first)
        except Exception as exc:   # surfaced in the main thread
            errors.append(exc)

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_same_shape_from_several_streams_and_threads():
    """The common case: several host threads reduce the SAME model shape, each on its own stream
    with its own values.  They share one cached plan and its workspace; the library orders
    their launches on the device (a call on another stream than the previous one waits for
    it), so every result is right -- against the oracle and bit-identical on every repeat.
    One thread also switches between bf16 and fp32 results and the delta form on the same
    table (plans of their own)."""
    import threading
    sizes = [3, 40000, 1, 70000, 16384 * 3 + 5]
    K = 16
    jobs = []
    for seed in (1, 2, 3):
        w = W.correlated_gaussian(sizes, K, dtype=torch.bfloat16, device=DEV, seed=90 + seed)
        jobs.append((w, oracle_reduce(w.grads, w.layer_offsets), torch.cuda.Stream(device=DEV)))
    torch.cuda.synchronize()
    errors = []

    def work(i, job):
        w, ref, stream = job
        try:
            first = {}
            # output buffers made up front: a buffer torch frees while a side stream still writes
            # it could be handed to another thread
            bufs = {od: torch.empty(w.N, dtype=od, device=DEV) for od in (torch.float32, torch.bfloat16)}
            torch.cuda.synchronize()
            for rep in range(40):
                od = torch.float32 if (i == 0 and rep % 2) else torch.bfloat16
                # no synchronisation between the calls of a thread: launches of the threads interleave
                out = B.adasum_reduce(w.grads, w.layer_offsets, bufs[od], out_dtype=od, stream=stream)
                if rep % 8 == 7 or rep < 2:
                    stream.synchronize()
                    if od not in first:
                        first[od] = out.clone()
                        assert_parity(out, ref, w.layer_offsets, what=f"thread {i} {od}")
                    else:
                        assert torch.equal(out, first[od]), (i, rep)
            stream.synchronize()
        except Exception as exc:   # surfaced in the main thread
            errors.append(exc)

    threads = [threading.Thread(target=work, args=(i, j)) for i, j in enumerate(jobs)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    # one host thread, two streams, same plan, no host synchronisation in between
    (w0, ref0, s0), (w1, ref1, s1) = jobs[0], jobs[1]
    outs = [torch.empty(w0.N, dtype=torch.bfloat16, device=DEV) for _ in range(6)]
    torch.cuda.synchronize()
    for rep in range(6):
        w, s = (w0, s0) if rep % 2 == 0 else (w1, s1)
        B.adasum_reduce(w.grads, w.layer_offsets, outs[rep], stream=s)
    torch.cuda.synchronize()
    for rep, out in enumerate(outs):
        assert_parity(out, ref0 if rep % 2 == 0 else ref1, w0.layer_offsets, what=f"alternating streams, call {rep}")


def test_binding_rejects_buffers_the_kernels_would_overrun():
    """A caller-owned plan's execute checks what the library itself cannot see from a pointer:
    a layer_stats tensor shorter than n_layers x 2 doubles (the statistics kernels would write
    past it), one on the host, and a delta_start of another dtype."""
    sizes = [100, 5000, 7]
    w = W.correlated_gaussian(sizes, 4, dtype=torch.bfloat16, device=DEV, seed=3)
    plan = B.Plan(4, w.layer_offsets, torch.bfloat16)
    short = torch.zeros(2 * len(sizes) - 2, dtype=torch.float64, device=DEV)
    with pytest.raises(ValueError):
        plan.execute(w.grads, layer_stats=short)
    with pytest.raises(ValueError):
        plan.execute(w.grads, layer_stats=torch.zeros(len(sizes), 2, dtype=torch.float64))
    with pytest.raises(ValueError):
        plan.execute(w.grads, layer_stats=torch.zeros(len(sizes), 2, dtype=torch.float32, device=DEV))
    ok = torch.zeros(len(sizes), 2, dtype=torch.float64, device=DEV)
    out = plan.execute(w.grads, layer_stats=ok)
    torch.cuda.synchronize()
    assert bool((ok[:, 1] > 0).all()) and bool(torch.isfinite(out.float()).all())
    plan.destroy()
    dplan = B.Plan(4, w.layer_offsets, torch.bfloat16, delta=True)
    with pytest.raises(ValueError):
        dplan.execute(w.grads, delta_start=torch.zeros(w.N, dtype=torch.float32, device=DEV))
    dplan.destroy()
    with pytest.raises(ValueError):
        B.adasum_reduce(w.grads, w.layer_offsets, layer_stats=torch.zeros(len(sizes), 2, dtype=torch.float64))


@pytest.mark.parametrize("K,radix,dtype", [(K, radix, dt) for K, radix in [(8, 0), (64, 0), (16, 2)]
                                           for dt in (torch.float32, torch.bfloat16)] +
                         [(64, 64, torch.bfloat16), (32, 32, torch.bfloat16)])   # (the wide first pass: fp32 sums too)
def test_supported_magnitude_range(K, radix, dtype):
    """Layers at the ends of the documented magnitude range (rms 1e-15 and 1e+15) beside ordinary
    ones: products are formed in fp32 lanes, so the squares (1e-30, 1e+30) must stay inside fp32.
    A layer far outside (1e-25: its squares underflow; 1e+25: they overflow) does not have the
    operator's result but leaves its neighbours alone."""
    say(f"magnitude range K={K} radix={radix} {dtype}")
    sizes = [5000, 70000, 300, 20000]
    w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=600 + K, scale=[1e-15, 1e15, 1.0, 1e-15])
    ref = oracle_reduce(w.grads, w.layer_offsets)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, out_dtype=torch.float32)
    torch.cuda.synchronize()
    err = assert_parity(out, ref, w.layer_offsets, what="in range")
    say(f"  rel-L2 per layer {err}")
    w2 = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=700 + K, scale=[1e-25, 1.0, 1e25, 1.0])
    ref2 = oracle_reduce(w2.grads, w2.layer_offsets)
    out2 = B.adasum_reduce(w2.grads, w2.layer_offsets, radix=radix, out_dtype=torch.float32)
    torch.cuda.synchronize()
    offs = w2.layer_offsets
    for l in (1, 3):
        lo, hi = offs[l], offs[l + 1]
        e = float(O.rel_l2_per_layer(to_f64(out2[lo:hi]), ref2[lo:hi], [0, hi - lo])[0])
        assert e <= TOL_F32, (l, e)
    # the underflowing layer stays finite (it falls on the zero-norm convention)
    assert np.all(np.isfinite(to_f64(out2[offs[0]:offs[1]])))


# ---------------------------------------------------------------------------
# radix 2 with sibling pairs combined together (the recursion of Section 3.4 taken one level ahead)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float64])
@pytest.mark.parametrize("K", [2, 3, 4, 5, 8, 13, 16, 64, 100, 256])
def test_sibling_fused_radix2(K, dtype):
    """fuse_siblings: from the second level on, the dot product of a pair comes from the combine that
    wrote its two nodes instead of from a pass of its own.  Same tree: checked against the oracle,
    against plain radix 2 (equal up to the rounding of the dot products), with statistics, and for
    identical bits on a rerun."""
    say(f"sibling-fused radix 2 K={K} {dtype}")
    sizes = np.diff(RAGGED).tolist()
    if dtype == torch.float64:
        w = _fp64_workload(sizes, K, 950 + K)
    elif dtype == torch.float16:
        w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=950 + K,
                                  scale=W.log_uniform_scales(len(sizes), 79, lo_exp=-2.0, hi_exp=0.0))
    else:
        w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=950 + K)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    before = [g.clone() for g in w.grads]
    wide = torch.float64 if dtype == torch.float64 else torch.float32
    stats = torch.full((w.n_layers, 2), -1.0, dtype=torch.float64, device=DEV)
    out = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True, out_dtype=wide, layer_stats=stats)
    plain_stats = torch.full((w.n_layers, 2), -1.0, dtype=torch.float64, device=DEV)
    plain = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, out_dtype=wide, layer_stats=plain_stats)
    torch.cuda.synchronize()
    for g, b in zip(w.grads, before):
        assert torch.equal(g, b), "inputs must not be modified"
    assert_parity(out, ref, w.layer_offsets, what="sibling-fused")
    # against the schedule it replaces: the two differ only in how the dot products were summed
    got, want = to_f64(out), to_f64(plain)
    offs = w.layer_offsets
    for l in range(w.n_layers):
        lo, hi = offs[l], offs[l + 1]
        if hi > lo and not np.isnan(ref[lo:hi]).any():
            den = np.linalg.norm(want[lo:hi])
            assert np.linalg.norm(got[lo:hi] - want[lo:hi]) <= (1e-12 if dtype == torch.float64 else 2e-6) * den, l
    np.testing.assert_allclose(stats.cpu().numpy()[:, 1], plain_stats.cpu().numpy()[:, 1], rtol=1e-12)
    np.testing.assert_allclose(stats.cpu().numpy()[:, 0], plain_stats.cpu().numpy()[:, 0], rtol=1e-5, atol=1e-300)
    if dtype != wide:
        narrow = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True)
        torch.cuda.synchronize()
        assert_parity(narrow, ref, w.layer_offsets, what="sibling-fused, narrow result")
        assert_bf16_rounding(narrow, ref, w.layer_offsets)
    again = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True, out_dtype=wide)
    torch.cuda.synchronize()
    assert torch.equal(again, out)


def test_sibling_fused_options():
    """Only with radix 2, the tree order and no delta form; caller-owned plans, graph replay and the
    entry point without allocation take the option as well."""
    w = W.correlated_gaussian([3, 5000, 70001, 1], 16, dtype=torch.bfloat16, device=DEV, seed=77)
    for kw in ({"radix": 0}, {"radix": 16}, {"radix": 2, "order": B.ORDER_LINEAR}):
        with pytest.raises(B.AdasumError) as e:
            B.adasum_reduce(w.grads, w.layer_offsets, fuse_siblings=True, **kw)
        assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True, delta_start=w.grads[0])
    assert e.value.code == B.ERR_UNSUPPORTED
    want = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True)
    torch.cuda.synchronize()
    assert_parity(want, oracle_reduce(w.grads, w.layer_offsets), w.layer_offsets)
    plan = B.Plan(16, w.layer_offsets, torch.bfloat16, radix=2, fuse_siblings=True)
    assert plan.workspace_bytes() == B.adasum_workspace_bytes(16, w.layer_offsets, B.BF16, radix=2, fuse_siblings=True)
    assert plan.workspace_bytes() != B.adasum_workspace_bytes(16, w.layer_offsets, B.BF16, radix=2)
    got = plan.execute(w.grads)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    plan.destroy()
    out = torch.empty_like(want)
    B.adasum_reduce(w.grads, w.layer_offsets, out, radix=2, fuse_siblings=True, noalloc=True)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    for _ in range(3):
        g = B.adasum_reduce(w.grads, w.layer_offsets, radix=2, fuse_siblings=True, use_graph=True)
        torch.cuda.synchronize()
        assert torch.equal(g, want)


# ---------------------------------------------------------------------------
# passes that feed the next one (default) against separate reduce passes
# ---------------------------------------------------------------------------

_FEED_CASES = [(K, radix, dtype)
               for K, radix in [(4, 2), (8, 2), (7, 4), (16, 4), (64, 4), (64, 8), (32, 0), (64, 0), (100, 0), (128, 0),
                                (256, 0), (512, 8), (1024, 0)]
               for dtype in (torch.float32, torch.bfloat16, torch.float16, torch.float64)
               # (fp64 passes take at most 8 workers: its wide cases are the radix-8 ones)
               if not (dtype == torch.float64 and radix == 0 and K > 64)]


@pytest.mark.parametrize("K,radix,dtype", _FEED_CASES)
def test_passes_that_feed_the_next_one(K, radix, dtype):
    """In the tree order the combine of a pass leaves the Gram matrix of the next pass's group
    (sibling groups of a tile in one workgroup, one wave each), unless separate_passes asks every
    pass to reduce its own operands.  Both are the same tree: each against the oracle, and against
    each other to the rounding of the dot products; statistics alike; reruns identical."""
    say(f"feeding passes K={K} radix={radix} {dtype}; passes {B.plan_levels(K, radix if radix else (8 if dtype == torch.float64 else 0))}")
    sizes = np.diff(RAGGED).tolist()
    if dtype == torch.float64:
        w = _fp64_workload(sizes, K, 1200 + K)
    elif dtype == torch.float16:
        w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=1200 + K,
                                  scale=W.log_uniform_scales(len(sizes), 80, lo_exp=-2.0, hi_exp=0.0))
    else:
        w = W.correlated_gaussian(sizes, K, dtype=dtype, device=DEV, seed=1200 + K)
    ref = oracle_reduce(w.grads, w.layer_offsets)
    wide = torch.float64 if dtype == torch.float64 else torch.float32
    s_feed = torch.full((w.n_layers, 2), -1.0, dtype=torch.float64, device=DEV)
    s_sep = torch.full((w.n_layers, 2), -1.0, dtype=torch.float64, device=DEV)
    feed = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, out_dtype=wide, layer_stats=s_feed)
    sep = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, out_dtype=wide, layer_stats=s_sep, separate_passes=True)
    torch.cuda.synchronize()
    assert_parity(feed, ref, w.layer_offsets, what="feeding passes")
    assert_parity(sep, ref, w.layer_offsets, what="separate passes")
    a, b = to_f64(feed), to_f64(sep)
    offs = w.layer_offsets
    for l in range(w.n_layers):
        lo, hi = offs[l], offs[l + 1]
        if hi > lo and not np.isnan(ref[lo:hi]).any():
            assert np.linalg.norm(a[lo:hi] - b[lo:hi]) <= (1e-12 if dtype == torch.float64 else 2e-6) * np.linalg.norm(b[lo:hi]), l
    np.testing.assert_allclose(s_feed.cpu().numpy()[:, 1], s_sep.cpu().numpy()[:, 1], rtol=1e-12)
    np.testing.assert_allclose(s_feed.cpu().numpy()[:, 0], s_sep.cpu().numpy()[:, 0], rtol=1e-5, atol=1e-300)
    again = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix, out_dtype=wide)
    torch.cuda.synchronize()
    assert torch.equal(again, feed)
    if dtype != wide:
        narrow = B.adasum_reduce(w.grads, w.layer_offsets, radix=radix)
        torch.cuda.synchronize()
        assert_parity(narrow, ref, w.layer_offsets, what="feeding passes, narrow result")
        assert_bf16_rounding(narrow, ref, w.layer_offsets)
