"""adasum_reduce_noalloc (tile tables and workspace in the library's static device array,
no allocation) against adasum_reduce_ex on the same inputs: the two run the same kernels on
the same tables, so the outputs must be identical bit for bit.  Every case makes two calls
in a row, the second on a smaller problem, so that the second finds the first one's
leftovers in the array."""
import numpy as np
import pytest
import torch

from paper_2006_02924_amd import binding as B
from paper_2006_02924_amd import workloads as W
from tests.gpu_util import assert_parity, oracle_reduce

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

RAGGED = [0, 1, 2, 9, 9, 40, 41, 1064, 1064 + 16384, 1064 + 16384 + 33000, 60000, 60001]
SMALLER = [0, 3, 3, 700, 701, 9000]


def say(msg):
    print(msg, flush=True)


def both(w, **kw):
    """The same reduction through adasum_reduce_ex and adasum_reduce_noalloc."""
    out_dtype = kw.get("out_dtype") or w.dtype
    stats = kw.pop("stats", False)
    L = w.n_layers
    s_ref = torch.zeros(L, 2, dtype=torch.float64, device=DEV) if stats else None
    s_got = torch.full((L, 2), -1.0, dtype=torch.float64, device=DEV) if stats else None
    ref = B.adasum_reduce(w.grads, w.layer_offsets, layer_stats=s_ref, **kw)
    out = torch.full((w.N,), float("nan"), dtype=out_dtype, device=DEV)
    got = B.adasum_reduce(w.grads, w.layer_offsets, out, layer_stats=s_got, noalloc=True, **kw)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), "outputs differ"
    if stats:
        assert torch.equal(s_got, s_ref)
    return got


CASES = [
    # (K, dtype, options of the first call, K and options of the second, smaller call)
    (8, torch.float32, {}, 4, {}),
    (64, torch.bfloat16, {"stats": True}, 16, {"out_dtype": torch.float32}),
    (64, torch.bfloat16, {"radix": 2}, 5, {"radix": 4}),
    (16, torch.float16, {"order": B.ORDER_LINEAR, "radix": 4}, 3, {"order": B.ORDER_LINEAR}),
    (12, torch.float64, {}, 1, {}),
    (1, torch.bfloat16, {"out_dtype": torch.float32, "stats": True}, 2, {"stats": True}),
]


@pytest.mark.parametrize("K,dtype,kw,K2,kw2", CASES)
def test_noalloc_matches_reduce_ex_twice(K, dtype, kw, K2, kw2):
    say(f"noalloc K={K} {dtype} {kw} then K={K2} {kw2}")
    if dtype == torch.float64:
        gen = lambda sizes, k, seed: _as(W.correlated_gaussian(sizes, k, dtype=torch.float32, device=DEV, seed=seed),
                                         torch.float64)
    else:
        gen = lambda sizes, k, seed: W.correlated_gaussian(sizes, k, dtype=dtype, device=DEV, seed=seed)
    w = gen(np.diff(RAGGED).tolist(), K, 31)
    got = both(w, **dict(kw))
    # and against the oracle once per case, so that "identical" cannot mean "identically wrong"
    order = "linear" if kw.get("order") == B.ORDER_LINEAR else "tree"
    assert_parity(got, oracle_reduce(w.grads, w.layer_offsets, order=order), w.layer_offsets, what="first call")
    w2 = gen(np.diff(SMALLER).tolist(), K2, 32)
    got2 = both(w2, **dict(kw2))
    order2 = "linear" if kw2.get("order") == B.ORDER_LINEAR else "tree"
    assert_parity(got2, oracle_reduce(w2.grads, w2.layer_offsets, order=order2), w2.layer_offsets,
                  what="second, smaller call")


def _as(w, dtype):
    w.grads = [g.to(dtype) for g in w.grads]
    w.dtype = dtype
    return w


def test_noalloc_delta_form_in_place_then_smaller():
    say("noalloc delta form")
    for sizes, K, seed in ((np.diff(RAGGED).tolist(), 16, 41), (np.diff(SMALLER).tolist(), 4, 42)):
        w = W.after_local_step(sizes, K, dtype=torch.bfloat16, device=DEV, seed=seed)
        start, currents, offs = w.meta["start"], w.grads, w.layer_offsets
        ref = B.adasum_reduce(currents, offs, delta_start=start)
        param = start.clone()
        got = B.adasum_reduce(currents, offs, param, delta_start=param, noalloc=True)   # in place
        torch.cuda.synchronize()
        assert got.data_ptr() == param.data_ptr()
        assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8))


def test_noalloc_many_layers_then_few():
    """More layers than one workgroup of the table builders has threads (runs of several layers
    per thread) and more boundaries than one launch carries; then three layers."""
    say("noalloc 5000 layers")
    rng = np.random.default_rng(7)
    sizes = rng.integers(0, 40, 5000)
    sizes[::97] = rng.integers(2000, 40000, len(sizes[::97]))
    for sz, K, seed in ((sizes.tolist(), 8, 51), ([5, 70000, 1], 8, 52)):
        w = W.correlated_gaussian(sz, K, dtype=torch.bfloat16, device=DEV, seed=seed)
        both(w, out_dtype=torch.float32, stats=True)


def test_noalloc_resnet50_shape_fits_and_repeats():
    """ResNet-50's table (161 tensors, 25.6 M elements), K = 8, fp32: inside the limit; the same
    call twice gives the same bits, and a small call in between does not disturb it."""
    say("noalloc config 2")
    w = W.config2(DEV)
    a = both(w).clone()
    small = W.correlated_gaussian([100, 3000], 4, dtype=torch.float32, device=DEV, seed=61)
    both(small)
    out = torch.empty_like(a)
    B.adasum_reduce(w.grads, w.layer_offsets, out, noalloc=True)
    torch.cuda.synchronize()
    assert torch.equal(out, a)


def test_noalloc_allocates_no_device_memory():
    """torch's allocator cannot see hipMalloc calls made by the library, but the driver's
    free-memory figure can: it does not move across calls on shapes the library has never seen."""
    say("noalloc leaves free device memory alone")
    ws = [W.correlated_gaussian([s, 4 * s + 3, 9], K, dtype=torch.bfloat16, device=DEV, seed=70 + K)
          for K, s in ((4, 30000), (32, 50000), (7, 11111))]
    outs = [torch.empty(w.N, dtype=torch.bfloat16, device=DEV) for w in ws]
    B.adasum_reduce(ws[0].grads, ws[0].layer_offsets, outs[0], noalloc=True)   # first use: symbol look-up
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for w, out in zip(ws, outs):
        B.adasum_reduce(w.grads, w.layer_offsets, out, noalloc=True)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, (free0, free1)


def test_noalloc_rejects_what_does_not_fit():
    say("noalloc limit")
    # 3 M elements x K = 64 fits (4 fp32 nodes = 48 MB); 4.2 M does not
    w = W.correlated_gaussian([1 << 20, (1 << 21) - 5], 64, dtype=torch.bfloat16, device=DEV, seed=81)
    both(w)
    g = [torch.zeros(4_200_000, dtype=torch.bfloat16, device=DEV)] * 64
    out = torch.empty(4_200_000, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(g, [0, 4_200_000], out, noalloc=True)
    assert e.value.code == B.ERR_TOO_LARGE
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.AdasumError) as e:
        B.adasum_reduce(w.grads, w.layer_offsets, out[: w.N], noalloc=True, workspace=ws)
    assert e.value.code == B.ERR_INVALID_ARG
