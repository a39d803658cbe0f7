"""Helpers for the GPU parity tests: feed the same stored values to the HIP
library (through the C-ABI binding) and to the CPU oracle."""
import numpy as np
import torch

from oracle import adasum_oracle as O

TOL_F32 = 1e-5    # per-layer relative L2 error, fp32 output
TOL_BF16 = 2e-3   # per-layer relative L2 error, bf16 output


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Stored device values widened exactly to fp64 on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_reduce(grads, layer_offsets, layers=None) -> np.ndarray:
    """fp64 oracle result for the whole buffer, or only for `layers` (other
    positions are left at 0)."""
    offs = list(layer_offsets)
    if layers is None:
        return O.adasum_reduce([to_f64(g) for g in grads], offs)
    out = np.zeros(offs[-1], dtype=np.float64)
    for l in layers:
        lo, hi = offs[l], offs[l + 1]
        if hi > lo:
            out[lo:hi] = O.adasum_tree([to_f64(g[lo:hi]) for g in grads])
    return out


def tol_for(dtype: torch.dtype) -> float:
    return TOL_BF16 if dtype == torch.bfloat16 else TOL_F32


def assert_parity(out: torch.Tensor, ref: np.ndarray, layer_offsets, layers=None, tol=None, what=""):
    tol = tol_for(out.dtype) if tol is None else tol
    offs = list(layer_offsets)
    got = to_f64(out)
    if layers is None:
        err = O.rel_l2_per_layer(got, ref, offs)
    else:
        err = np.zeros(len(offs) - 1)
        for l in layers:
            lo, hi = offs[l], offs[l + 1]
            err[l] = O.rel_l2_per_layer(got[lo:hi], ref[lo:hi], [0, hi - lo])[0]
    worst = int(np.argmax(err))
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    assert err[worst] <= tol, (f"{what}: layer {worst} (size {offs[worst + 1] - offs[worst]}) "
                               f"rel-L2 {err[worst]:.3e} > {tol:.1e}")
    return err


def bf16_ulp_distance(out_bf16: torch.Tensor, ref: np.ndarray) -> np.ndarray:
    """|out - RNE_bf16(ref)| in units of bf16 ulps of the reference value."""
    r = torch.from_numpy(ref).to(torch.float32).to(torch.bfloat16)
    a = out_bf16.detach().cpu().view(torch.int16).to(torch.int32)
    b = r.view(torch.int16).to(torch.int32)
    # sign-magnitude -> monotone integer line
    a = torch.where(a < 0, -(a & 0x7FFF), a)
    b = torch.where(b < 0, -(b & 0x7FFF), b)
    return (a - b).abs().numpy()
