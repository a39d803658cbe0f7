"""The synthetic-input recipe: layer tables and seeded generators (CPU)."""
import numpy as np
import torch

from paper_2006_02924_amd import workloads as W


def test_resnet50_table():
    s = W.resnet50_layer_sizes()
    assert len(s) == 161 and sum(s) == 25_557_032
    assert min(s) == 64 and max(s) == 2_359_296
    assert sum(1 for x in s if x <= 2048) == 107


def test_bert_large_table():
    s = W.bert_large_layer_sizes()
    assert len(s) == 391 and sum(s) == 335_141_888
    hist = {}
    for x in s:
        hist[x] = hist.get(x, 0) + 1
    assert hist == {1024: 219, 4096: 24, 2048: 1, 524_288: 1, 1_048_576: 97,
                    4_194_304: 48, 31_254_528: 1}


def test_config1_recipe_and_seed():
    a = W.config1()
    b = W.config1()
    assert a.K == 4 and a.layer_offsets == [0, 1000, 5096, 70632]
    for x, y in zip(a.grads, b.grads):
        assert torch.equal(x, y)
    # correlation between two workers is a^2 = 0.36, variance 1
    g0, g1 = a.grads[0][5096:].double(), a.grads[1][5096:].double()
    assert abs(float(g0.var()) - 1.0) < 0.03
    assert abs(float((g0 * g1).mean()) - 0.36) < 0.03


def test_config5_degenerate_cases_small():
    sizes = W.scaled_down(W.bert_large_layer_sizes(), 4096, floor=8)
    w = W.config5(K=8, sizes=sizes)
    kinds = w.meta["kind"]
    assert w.n_layers == len(sizes) + 16
    assert sum(1 for l in range(w.n_layers)
               if w.layer_offsets[l + 1] - w.layer_offsets[l] == 1) >= 16
    for k in ("parallel", "orth_pairs", "zero", "orth_all"):
        assert k in kinds, k
    offs = w.layer_offsets
    for l, k in enumerate(kinds):
        lo, hi = offs[l], offs[l + 1]
        if k == "orth_pairs" and hi - lo > 64:
            g0, g1 = w.grads[0][lo:hi].double(), w.grads[1][lo:hi].double()
            cos = float(g0 @ g1) / float(g0.norm() * g1.norm())
            assert abs(cos) < 0.02
        if k == "orth_all":
            X = torch.stack([g[lo:hi].double() for g in w.grads])
            G = (X @ X.T).numpy()
            off = G - np.diag(np.diag(G))
            assert np.abs(off).max() < 0.02 * np.diag(G).min()
    modes = {m for _, m in w.meta["zero_modes"]}
    assert modes == {0, 1, 2}
    l0 = [l for l, m in w.meta["zero_modes"] if m == 0][0]
    assert all(float(g[offs[l0]:offs[l0 + 1]].abs().sum()) == 0.0 for g in w.grads)
