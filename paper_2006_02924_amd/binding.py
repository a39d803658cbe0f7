"""ctypes binding over the C-ABI of ``libadasum.so`` (see ``include/adasum.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (``tensor.data_ptr()``) and the current
HIP stream.  There is no fallback: if the library has not been built,
``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# ADASUM_LIB overrides the library file (e.g. a build with other tuning knobs)
LIB_PATH = os.environ.get("ADASUM_LIB") or os.path.join(HERE, "libadasum.so")

F32, BF16, F16, F64 = 0, 1, 2, 3
ORDER_TREE, ORDER_LINEAR = 0, 1

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_MISALIGNED = -1, -2, -3
ERR_OUT_OF_MEMORY, ERR_HIP, ERR_WORKSPACE, ERR_ALIAS, ERR_TOO_LARGE = -4, -5, -6, -7, -8
NOALLOC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "adasum_reduce", "adasum_reduce_ex", "adasum_reduce_noalloc", "adasum_workspace_bytes",
    "adasum_plan_create", "adasum_plan_execute", "adasum_plan_workspace_bytes", "adasum_plan_destroy",
    "adasum_group_gram", "adasum_group_weights", "adasum_group_combine",
    "adasum_tile_capacity", "adasum_plan_tiles", "adasum_plan_levels", "adasum_plan_groups",
    "adasum_profile_enable", "adasum_profile_collect",
    "adasum_strerror", "adasum_last_hip_error", "adasum_version", "adasum_shutdown",
]


class AdasumError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libadasum error {code}: {msg}")
        self.code = code


class Options(C.Structure):
    _fields_ = [
        ("struct_bytes", C.c_uint32),
        ("out_dtype", C.c_int32),
        ("radix", C.c_int32),
        ("order", C.c_int32),
        ("use_graph", C.c_int32),
        ("fuse_siblings", C.c_int32),
        ("workspace", C.c_void_p),
        ("workspace_bytes", C.c_size_t),
        ("layer_stats", C.c_void_p),
        ("delta_start", C.c_void_p),
        ("separate_passes", C.c_int32),
        ("reserved1", C.c_int32),
    ]


class Tile(C.Structure):
    _fields_ = [("start", C.c_int64), ("len", C.c_int32), ("layer", C.c_int32)]


class KernelProfile(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64),
                ("total_ms", C.c_double), ("bytes", C.c_double)]


_lib = None


def load() -> C.CDLL:
    """Loads the built library (once).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built; run `python -m paper_2006_02924_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    pp = C.POINTER(C.c_void_p)
    i64p = C.POINTER(C.c_int64)
    lib.adasum_reduce.argtypes = [pp, C.c_int, i64p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.adasum_reduce_ex.argtypes = [pp, C.c_int, i64p, C.c_int, C.c_int, C.c_void_p,
                                     C.POINTER(Options), C.c_void_p]
    lib.adasum_reduce_noalloc.argtypes = lib.adasum_reduce_ex.argtypes
    lib.adasum_workspace_bytes.argtypes = [C.c_int, i64p, C.c_int, C.c_int, C.POINTER(Options),
                                           C.POINTER(C.c_size_t)]
    lib.adasum_group_gram.argtypes = [pp, C.c_int, i64p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.adasum_group_weights.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.adasum_group_combine.argtypes = [pp, C.c_int, i64p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_int, C.c_void_p, C.c_void_p]
    lib.adasum_tile_capacity.argtypes = []
    lib.adasum_plan_tiles.argtypes = [i64p, C.c_int, C.c_int64, C.POINTER(Tile), C.c_int64, i64p]
    lib.adasum_plan_levels.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_int)]
    lib.adasum_profile_enable.argtypes = [C.c_int]
    lib.adasum_profile_collect.argtypes = [C.POINTER(KernelProfile), C.c_int, C.POINTER(C.c_int)]
    lib.adasum_strerror.argtypes = [C.c_int]
    lib.adasum_strerror.restype = C.c_char_p
    lib.adasum_last_hip_error.argtypes = []
    lib.adasum_version.argtypes = []
    lib.adasum_version.restype = C.c_char_p
    lib.adasum_shutdown.argtypes = []
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int or fn.restype is None:
            fn.restype = C.c_int
    _lib = lib
    return lib


def check(code: int) -> None:
    if code != OK:
        lib = load()
        msg = lib.adasum_strerror(code).decode()
        if code == ERR_HIP:
            msg += f" [hipError {lib.adasum_last_hip_error()}]"
        raise AdasumError(code, msg)


# ---- marshalling helpers ------------------------------------------------------

def _offsets(layer_offsets: Sequence[int]):
    arr = (C.c_int64 * len(layer_offsets))(*[int(o) for o in layer_offsets])
    return arr, len(layer_offsets) - 1


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[C.c_void_p(t.data_ptr()) for t in tensors])


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.float64:
        return F64
    raise TypeError(f"unsupported dtype {t.dtype}")


def _code_of(torch_dtype) -> int:
    import torch
    return {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16, torch.float64: F64}[torch_dtype]


def _torch_dtype(code: int):
    import torch
    return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16, F64: torch.float64}[code]


def _stream(stream) -> C.c_void_p:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check_inputs(tensors, N):
    dev = tensors[0].device
    if dev.type != "cuda":
        raise ValueError("libadasum works on device memory only (no CPU path)")
    for t in tensors:
        if t.device != dev or t.dtype != tensors[0].dtype:
            raise ValueError("all gradients must share device and dtype")
        if not t.is_contiguous() or t.dim() != 1 or t.numel() != N:
            raise ValueError("every gradient must be a contiguous 1-D buffer of layer_offsets[-1] elements")


# ---- the combiner ---------------------------------------------------------------

def adasum_reduce(grads: Sequence, layer_offsets: Sequence[int], out=None, *, out_dtype=None,
                  radix: int = 0, order: int = ORDER_TREE, layer_stats=None, workspace=None,
                  use_graph: bool = False, delta_start=None, stream=None, noalloc: bool = False,
                  fuse_siblings: bool = False, separate_passes: bool = False):
    """Per-layer Adasum tree of ``grads`` (K device tensors of N elements).
    Returns ``out`` (allocated here when None).  With ``delta_start`` (a tensor
    like one of ``grads``) the tensors in ``grads`` are parameters after a local
    optimizer step, the tree runs on ``grads[k] - delta_start`` and the result
    is ``delta_start + Adasum(...)``; ``out`` may then be ``delta_start`` itself.
    ``noalloc`` calls ``adasum_reduce_noalloc`` (tables and workspace in the library's
    static scratch; ``out`` must then be given, so that nothing here allocates either)."""
    import torch
    lib = load()
    if noalloc and out is None:
        raise ValueError("noalloc: pass `out` (this call must not allocate)")
    offs, L = _offsets(layer_offsets)
    N = int(layer_offsets[-1])
    _check_inputs(grads, N)
    in_code = _dtype_code(grads[0])
    out_code = in_code if out_dtype is None else _code_of(out_dtype)
    if out is None:
        out = torch.empty(N, dtype=_torch_dtype(out_code), device=grads[0].device)
    elif (_dtype_code(out) != out_code or out.numel() != N or not out.is_contiguous()
          or out.device != grads[0].device):
        raise ValueError("out has the wrong dtype, size, layout or device")
    ptrs = _ptr_array(grads)
    plain = (out_code == in_code and radix == 0 and order == ORDER_TREE and layer_stats is None
             and workspace is None and not use_graph and delta_start is None and not noalloc
             and not fuse_siblings and not separate_passes)
    if plain:
        check(lib.adasum_reduce(ptrs, len(grads), offs, L, in_code, C.c_void_p(out.data_ptr()), _stream(stream)))
        return out
    o = Options()
    o.struct_bytes = C.sizeof(Options)
    o.out_dtype = out_code
    o.radix = radix
    o.order = order
    o.use_graph = 1 if use_graph else 0
    o.fuse_siblings = 1 if fuse_siblings else 0
    o.separate_passes = 1 if separate_passes else 0
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    if layer_stats is not None:
        if (layer_stats.dtype != torch.float64 or layer_stats.numel() != 2 * L or not layer_stats.is_contiguous()
                or layer_stats.device != grads[0].device):
            raise ValueError("layer_stats must be a contiguous float64 tensor of n_layers x 2 on the device of grads")
        o.layer_stats = layer_stats.data_ptr()
    if delta_start is not None:
        _check_inputs([delta_start], N)
        if delta_start.dtype != grads[0].dtype or delta_start.device != grads[0].device:
            raise ValueError("delta_start must have the dtype and device of grads")
        o.delta_start = delta_start.data_ptr()
    fn = lib.adasum_reduce_noalloc if noalloc else lib.adasum_reduce_ex
    check(fn(ptrs, len(grads), offs, L, in_code, C.c_void_p(out.data_ptr()), C.byref(o), _stream(stream)))
    return out


class Plan:
    """A plan the caller owns (``adasum_plan_create`` .. ``adasum_plan_destroy``) for one
    problem shape; ``execute`` reduces K tensors of that shape."""

    def __init__(self, K: int, layer_offsets: Sequence[int], dtype, *, out_dtype=None, radix: int = 0,
                 order: int = ORDER_TREE, use_graph: bool = False, workspace=None, delta: bool = False,
                 fuse_siblings: bool = False, separate_passes: bool = False):
        lib = load()
        offs, L = _offsets(layer_offsets)
        self.K, self.N, self.n_layers = K, int(layer_offsets[-1]), L
        self.in_code = _code_of(dtype)
        self.out_code = self.in_code if out_dtype is None else _code_of(out_dtype)
        self.delta = delta
        self._workspace = workspace          # keep the tensor alive
        o = Options()
        o.struct_bytes = C.sizeof(Options)
        o.out_dtype = self.out_code
        o.radix = radix
        o.order = order
        o.use_graph = 1 if use_graph else 0
        o.fuse_siblings = 1 if fuse_siblings else 0
        o.separate_passes = 1 if separate_passes else 0
        if workspace is not None:
            o.workspace = workspace.data_ptr()
            o.workspace_bytes = workspace.numel() * workspace.element_size()
        if delta:
            o.delta_start = 0x100            # "set": the pointer itself comes with every execute
        self._h = C.c_void_p(None)
        check(lib.adasum_plan_create(K, offs, L, self.in_code, C.byref(o), C.byref(self._h)))

    def workspace_bytes(self) -> int:
        n = C.c_size_t(0)
        check(load().adasum_plan_workspace_bytes(self._h, C.byref(n)))
        return int(n.value)

    def execute(self, grads: Sequence, out=None, *, layer_stats=None, delta_start=None, stream=None):
        import torch
        if len(grads) != self.K:
            raise ValueError("the plan was made for another number of workers")
        _check_inputs(grads, self.N)
        if _dtype_code(grads[0]) != self.in_code:
            raise ValueError("the plan was made for another dtype")
        if out is None:
            out = torch.empty(self.N, dtype=_torch_dtype(self.out_code), device=grads[0].device)
        elif _dtype_code(out) != self.out_code or out.numel() != self.N or not out.is_contiguous():
            raise ValueError("out has the wrong dtype, size or layout")
        if out.device != grads[0].device:
            raise ValueError("out must be on the device of grads")
        stats_ptr = None
        if layer_stats is not None:
            # the kernels write n_layers x 2 doubles: a shorter buffer would be overrun on the device
            if (layer_stats.dtype != torch.float64 or not layer_stats.is_contiguous()
                    or layer_stats.numel() != 2 * self.n_layers or layer_stats.device != grads[0].device):
                raise ValueError("layer_stats must be a contiguous float64 tensor of n_layers x 2 on the device "
                                 "of grads")
            stats_ptr = C.c_void_p(layer_stats.data_ptr())
        start_ptr = None
        if delta_start is not None:
            _check_inputs([delta_start], self.N)
            if delta_start.dtype != grads[0].dtype or delta_start.device != grads[0].device:
                raise ValueError("delta_start must have the dtype and device of grads")
            start_ptr = C.c_void_p(delta_start.data_ptr())
        check(load().adasum_plan_execute(self._h, _ptr_array(grads), C.c_void_p(out.data_ptr()), stats_ptr,
                                         start_ptr, _stream(stream)))
        return out

    def destroy(self) -> None:
        if self._h:
            check(load().adasum_plan_destroy(self._h))
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def adasum_workspace_bytes(K: int, layer_offsets: Sequence[int], dtype_code: int, *, radix: int = 0,
                           out_dtype_code: int = -1, delta: bool = False, order: int = ORDER_TREE,
                           fuse_siblings: bool = False, separate_passes: bool = False) -> int:
    lib = load()
    offs, L = _offsets(layer_offsets)
    o = Options()
    o.struct_bytes = C.sizeof(Options)
    o.out_dtype = out_dtype_code
    o.radix = radix
    o.order = order
    o.fuse_siblings = 1 if fuse_siblings else 0
    o.separate_passes = 1 if separate_passes else 0
    if delta:
        o.delta_start = 0x100   # only "set or not" matters for the size
    n = C.c_size_t(0)
    check(lib.adasum_workspace_bytes(K, offs, L, dtype_code, C.byref(o), C.byref(n)))
    return int(n.value)


# ---- the steps of one level -----------------------------------------------------

def adasum_group_gram(xs: Sequence, layer_offsets: Sequence[int], stream=None):
    """Per-layer R x R Gram matrices of R operands -> float64 tensor [L, R, R]."""
    import torch
    lib = load()
    offs, L = _offsets(layer_offsets)
    _check_inputs(xs, int(layer_offsets[-1]))
    R = len(xs)
    gram = torch.empty((L, R, R), dtype=torch.float64, device=xs[0].device)
    check(lib.adasum_group_gram(_ptr_array(xs), R, offs, L, _dtype_code(xs[0]),
                                C.c_void_p(gram.data_ptr()), _stream(stream)))
    return gram


def adasum_group_weights(gram, order: int = ORDER_TREE, stream=None):
    """[L, R, R] float64 Gram matrices -> [L, R] float64 tree weights."""
    import torch
    lib = load()
    L, R, _ = gram.shape
    w = torch.empty((L, R), dtype=torch.float64, device=gram.device)
    check(lib.adasum_group_weights(C.c_void_p(gram.data_ptr()), R, L, order, C.c_void_p(w.data_ptr()),
                                   _stream(stream)))
    return w


def adasum_group_combine(xs: Sequence, layer_offsets: Sequence[int], weights, *, out=None, out_dtype=None,
                         want_sqnorm: bool = True, stream=None):
    """out = sum_r weights[layer, r] * xs[r]; returns (out, per-layer squared norm or None)."""
    import torch
    lib = load()
    offs, L = _offsets(layer_offsets)
    N = int(layer_offsets[-1])
    _check_inputs(xs, N)
    in_code = _dtype_code(xs[0])
    out_code = in_code if out_dtype is None else _code_of(out_dtype)
    if weights.dtype != torch.float64 or weights.numel() != L * len(xs) or not weights.is_contiguous():
        raise ValueError("weights must be a contiguous float64 tensor of n_layers x R")
    if out is None:
        out = torch.empty(N, dtype=_torch_dtype(out_code), device=xs[0].device)
    sq = torch.empty(L, dtype=torch.float64, device=xs[0].device) if want_sqnorm else None
    check(lib.adasum_group_combine(_ptr_array(xs), len(xs), offs, L, in_code, C.c_void_p(weights.data_ptr()),
                                   C.c_void_p(out.data_ptr()), out_code,
                                   C.c_void_p(sq.data_ptr()) if sq is not None else None, _stream(stream)))
    return out, sq


# ---- planning (host only) ---------------------------------------------------------

def tile_capacity() -> int:
    return int(load().adasum_tile_capacity())


def plan_tiles(layer_offsets: Sequence[int], capacity: int = 0) -> np.ndarray:
    """Tile table (capacity 0 = the Gram pass's) as a structured array with
    fields start, len, layer."""
    lib = load()
    offs, L = _offsets(layer_offsets)
    n = C.c_int64(0)
    check(lib.adasum_plan_tiles(offs, L, capacity, None, 0, C.byref(n)))
    buf = (Tile * max(1, n.value))()
    check(lib.adasum_plan_tiles(offs, L, capacity, buf, n.value, C.byref(n)))
    arr = np.frombuffer(buf, dtype=np.dtype([("start", "<i8"), ("len", "<i4"), ("layer", "<i4")]),
                        count=n.value)
    return arr.copy()


def plan_levels(K: int, radix: int = 0) -> List[int]:
    lib = load()
    buf = (C.c_int * 64)()
    n = C.c_int(0)
    check(lib.adasum_plan_levels(K, radix, buf, 64, C.byref(n)))
    return [int(buf[i]) for i in range(n.value)]


def plan_groups(K: int, radix: int = 0) -> List[int]:
    """Worker ranges of the first pass's groups: G + 1 boundaries."""
    lib = load()
    n = C.c_int(0)
    check(lib.adasum_plan_groups(K, radix, None, 0, C.byref(n)))
    buf = (C.c_int * (n.value + 1))()
    check(lib.adasum_plan_groups(K, radix, buf, n.value + 1, C.byref(n)))
    return [int(buf[i]) for i in range(n.value + 1)]


# ---- per-kernel timing --------------------------------------------------------------

def profile_enable(on: bool) -> None:
    check(load().adasum_profile_enable(1 if on else 0))


def profile_collect() -> List[dict]:
    lib = load()
    buf = (KernelProfile * 128)()
    n = C.c_int(0)
    check(lib.adasum_profile_collect(buf, 128, C.byref(n)))
    return [{"name": buf[i].name.decode(), "launches": int(buf[i].launches),
             "total_ms": float(buf[i].total_ms), "bytes": float(buf[i].bytes)}
            for i in range(min(n.value, 128))]


def version() -> str:
    return load().adasum_version().decode()


def shutdown() -> None:
    check(load().adasum_shutdown())
