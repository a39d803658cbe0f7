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
from tests.gpu_util import assert_bf16_rounding, assert_parity, oracle_reduce, to_f64

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
    for radix, out_dtype in ((0, torch.bfloat16), (0, torch.float32), (2, torch.bfloat16)):
        say(f"adasum_reduce radix={radix} -> {out_dtype}")
        out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=radix,
                              layer_stats=stats if (radix == 0 and out_dtype == torch.float32) else None)
        torch.cuda.synchronize()
        err = assert_parity(out, ref, w.layer_offsets, layers=layers, what=f"config4 radix {radix} {out_dtype}")
        say(f"  max rel-L2 on sampled layers {err.max():.3e}")
        if out_dtype == torch.bfloat16:
            assert_bf16_rounding(out, ref, w.layer_offsets, layers=layers)
        outs[(radix, out_dtype)] = out
    # properties that hold for every layer: finite output; |Adasum(g1,g2)|^2 <= |g1|^2 + |g2|^2 at every
    # node, so the Section 3.6 metric is at most 1 (and positive here: the workers are positively
    # correlated); the default path rerun gives identical bits
    full = outs[(0, torch.float32)]
    assert bool(torch.isfinite(full).all())
    s = stats.cpu().numpy()
    metric = s[:, 0] / s[:, 1]
    assert np.all(metric <= 1.0 + 1e-5) and np.all(metric > 0.0), (metric.min(), metric.max())
    say(f"  orthogonality metric over layers: min {metric.min():.4f} max {metric.max():.4f}")
    again = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(again, outs[(0, torch.bfloat16)])
    # the two radices agree with each other on every layer far inside the bf16 tolerance
    a = outs[(0, torch.bfloat16)].float()
    b = outs[(2, torch.bfloat16)].float()
    differ = float((a != b).float().mean())
    say(f"  radix 8 vs radix 2 bf16 outputs differ in {differ:.2e} of the elements")
    assert differ < 1e-2
