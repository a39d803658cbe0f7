"""The C-ABI library loads, exports what include/adasum.h declares, and rejects
bad arguments before touching a device (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2006_02924_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "adasum.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adasum_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_version_and_strerror(lib):
    assert b"libadasum" in lib.adasum_version()
    for code in range(0, -9, -1):
        assert lib.adasum_strerror(code)
    assert lib.adasum_strerror(-99) == b"unknown error"


def _call_reduce(lib, ptrs, K, offs, dtype, out, opts=None):
    arr = (C.c_void_p * max(1, len(ptrs)))(*ptrs) if ptrs is not None else None
    o = (C.c_int64 * len(offs))(*offs) if offs is not None else None
    L = len(offs) - 1 if offs is not None else 0
    if opts is None:
        return lib.adasum_reduce(arr, K, o, L, dtype, out, None)
    return lib.adasum_reduce_ex(arr, K, o, L, dtype, out, C.byref(opts), None)


def _opts(**kw):
    o = B.Options()
    o.struct_bytes = C.sizeof(B.Options)
    o.out_dtype = -1
    for k, v in kw.items():
        setattr(o, k, v)
    return o


def test_reduce_rejects_bad_arguments(lib):
    good = [0x1000, 0x2000, 0x3000, 0x4000]
    offs = [0, 10, 30]
    assert _call_reduce(lib, None, 4, offs, B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 0, offs, B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 4, None, B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 4, [1, 10, 30], B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 4, [0, 30, 10], B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 4, offs, 7, 0x9000) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, [0x1000, 0x2004, 0x3000, 0x4000], 4, offs, B.F32, 0x9000) == B.ERR_MISALIGNED
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x9008) == B.ERR_MISALIGNED
    assert _call_reduce(lib, [0x1000, 0, 0x3000, 0x4000], 4, offs, B.F32, 0x9000) == B.ERR_INVALID_ARG
    assert _call_reduce(lib, good, 4, offs, B.F32, None) == B.ERR_INVALID_ARG
    # out overlapping worker 1's buffer (30 fp32 = 120 bytes from 0x2000)
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x2040) == B.ERR_ALIAS


def test_noalloc_entry_point_validates_before_any_device_work(lib):
    """adasum_reduce_noalloc: the checks of adasum_reduce_ex, no caller workspace or graph replay,
    and a problem whose tables and workspace exceed the static array is refused up front."""
    def call(ptrs, K, offs, dtype, out, opts=None):
        arr = (C.c_void_p * len(ptrs))(*ptrs)
        o = (C.c_int64 * len(offs))(*offs)
        return lib.adasum_reduce_noalloc(arr, K, o, len(offs) - 1, dtype, out, C.byref(opts) if opts else None, None)

    good = [0x100000 * (i + 1) for i in range(64)]
    out = 0x90000000
    assert call(good[:2], 2, [0], B.BF16, out) == B.OK                      # empty problem
    assert call(good[:2], 0, [0, 8], B.BF16, out) == B.ERR_INVALID_ARG
    assert call(good[:2], 2, [0, 8], 9, out) == B.ERR_UNSUPPORTED
    assert call(good[:2], 2, [0, 8], B.F32, out + 4) == B.ERR_MISALIGNED
    assert call(good[:2], 2, [0, 8], B.F32, good[1] + 16) == B.ERR_ALIAS
    assert call(good[:2], 2, [0, 8], B.F32, out, _opts(use_graph=1)) == B.ERR_INVALID_ARG
    assert call(good[:2], 2, [0, 8], B.F32, out, _opts(workspace=0x10000, workspace_bytes=1 << 30)) \
        == B.ERR_INVALID_ARG
    # K = 64 over 4.2 M elements needs four fp32 nodes = 67 MB: more than the 64 MiB array
    assert call(good, 64, [0, 4_200_000], B.BF16, out) == B.ERR_TOO_LARGE
    assert B.adasum_workspace_bytes(64, [0, 4_200_000], B.BF16) > B.NOALLOC_SCRATCH_BYTES
    assert b"static scratch" in lib.adasum_strerror(B.ERR_TOO_LARGE)
    header = open(os.path.join(ROOT, "include", "adasum.h")).read()
    assert re.search(r"#define\s+ADASUM_NOALLOC_SCRATCH_BYTES\s+\(64u << 20\)", header)


def test_empty_problem_is_a_no_op(lib):
    assert _call_reduce(lib, [0x1000, 0x2000], 2, [0], B.F32, 0x9000) == B.OK
    assert _call_reduce(lib, [0x1000, 0x2000], 2, [0, 0, 0], B.BF16, 0x9000) == B.OK
    assert _call_reduce(lib, [0, 0], 2, [0, 0], B.BF16, None) == B.OK


def test_options_validation(lib):
    good = [0x1000, 0x2000]
    offs = [0, 8]
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(out_dtype=5)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(radix=3)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(order=9)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(workspace=0x10010, workspace_bytes=1 << 20)) \
        == B.ERR_WORKSPACE
    bad = _opts()
    bad.struct_bytes = 8
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, bad) == B.ERR_INVALID_ARG


def test_sibling_fusion_option_validation(lib):
    """fuse_siblings goes with radix 2, the tree order and no delta form; it needs room for the
    dot products its combines leave."""
    good = [0x1000, 0x2000, 0x3000, 0x4000]
    offs = [0, 8]
    assert _call_reduce(lib, good, 4, [0], B.F32, 0x9000, _opts(radix=2, fuse_siblings=1)) == B.OK
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x9000, _opts(radix=0, fuse_siblings=1)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x9000, _opts(radix=4, fuse_siblings=1)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x9000, _opts(radix=2, fuse_siblings=1, order=B.ORDER_LINEAR)) \
        == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 4, offs, B.F32, 0x9000, _opts(radix=2, fuse_siblings=1, delta_start=0x5000)) \
        == B.ERR_UNSUPPORTED
    big = [0, 70632]
    # the delta form leaves nothing for the pass above (no such extra section): the size to compare with
    bare = B.adasum_workspace_bytes(16, big, B.F32, radix=2, delta=True)
    fused = B.adasum_workspace_bytes(16, big, B.F32, radix=2, fuse_siblings=True)
    # 4 pairs of groups x 69 combine tiles of 1024 elements, one double each
    assert bare < fused <= bare + 4 * 70 * 8 + 256
    # plain radix 2: every pass but the last leaves the next one's 2 x 2 Gram matrix (3 entries) per
    # 256-element combine tile: 4 next-pass groups x 276 tiles x 3 doubles
    plain = B.adasum_workspace_bytes(16, big, B.F32, radix=2)
    assert bare + 4 * 276 * 3 * 8 <= plain <= bare + 4 * 277 * 3 * 8 + 256
    # a single pair has no level above its first: nothing to leave
    assert B.adasum_workspace_bytes(2, big, B.F32, radix=2, fuse_siblings=True) == B.adasum_workspace_bytes(2, big, B.F32, radix=2)


def test_wide_radix_option_validation(lib):
    """Radix 32 and 64 (the first pass's Gram matrix from the matrix cores): bf16 and fp16 inputs, the
    tree order, no delta form; the passes above stay at 16 or less; the pass leaves its blocks per span."""
    good = [0x1000 * (i + 1) for i in range(64)]
    offs = [0, 8]
    for radix in (32, 64):
        assert _call_reduce(lib, good, 64, [0], B.BF16, 0x90000, _opts(radix=radix)) == B.OK
        assert _call_reduce(lib, good, 64, offs, B.F32, 0x90000, _opts(radix=radix)) == B.ERR_UNSUPPORTED
        assert _call_reduce(lib, good, 64, offs, B.F64, 0x90000, _opts(radix=radix)) == B.ERR_UNSUPPORTED
        assert _call_reduce(lib, good, 64, offs, B.BF16, 0x90000, _opts(radix=radix, order=B.ORDER_LINEAR)) \
            == B.ERR_UNSUPPORTED
        assert _call_reduce(lib, good, 64, offs, B.F16, 0x90000, _opts(radix=radix, delta_start=0x80000)) \
            == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 64, offs, B.BF16, 0x90000, _opts(radix=128)) == B.ERR_UNSUPPORTED
    assert B.plan_levels(64, 64) == [64] and B.plan_levels(64, 32) == [32, 2] and B.plan_levels(32, 64) == [32]
    assert B.plan_levels(128, 64) == [64, 2] and B.plan_levels(4096, 64) == [64, 16, 4]
    assert B.plan_levels(48, 64) == [64] and B.plan_levels(24, 64) == [32] and B.plan_levels(12, 64) == [16]
    # a single pass keeps no nodes: blocks of 3 x 1024 doubles per span (here 35 parts of 2048 elements,
    # one more span where the layer boundary cuts a part), nothing per element
    big = [0, 1000, 70632]
    n64 = B.adasum_workspace_bytes(64, big, B.BF16, radix=64)
    assert 36 * 3072 * 8 <= n64 <= 36 * 3072 * 8 + (1 << 20)
    assert n64 < B.adasum_workspace_bytes(64, big, B.BF16)
    # step entry points: 32 and 64 operands for 16-bit storage only
    x = (C.c_void_p * 64)(*good)
    o = (C.c_int64 * 2)(0, 8)
    assert lib.adasum_group_gram(x, 64, o, 1, B.F32, 0x90000, None) == B.ERR_UNSUPPORTED
    assert lib.adasum_group_gram(x, 64, o, 1, B.BF16, None, None) == B.ERR_INVALID_ARG
    assert lib.adasum_group_combine(x, 32, o, 1, B.F32, 0xa0000, 0x90000, B.F32, None, None) == B.ERR_UNSUPPORTED
    assert lib.adasum_group_weights(0x9000, 64, 0, 0, 0xa000, None) == B.OK
    assert lib.adasum_group_weights(0x9000, 128, 1, 0, 0xa000, None) == B.ERR_UNSUPPORTED


def test_fp64_storage_limits(lib):
    good = [0x1000, 0x2000]
    offs = [0, 8]
    assert _call_reduce(lib, good, 2, offs, B.F64, 0x9000, _opts(out_dtype=B.F32)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(out_dtype=B.F64)) == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F64, 0x9000, _opts(radix=16)) == B.ERR_UNSUPPORTED
    # fp64 nodes are twice as wide as fp32 ones
    big = [0, 70632]
    assert B.adasum_workspace_bytes(64, big, B.F64, radix=8) > B.adasum_workspace_bytes(64, big, B.F32, radix=8) \
        + 8 * 70632 * 4 - 4096
    x = (C.c_void_p * 2)(0x1000, 0x2000)
    o = (C.c_int64 * 2)(0, 8)
    assert lib.adasum_group_combine(x, 2, o, 1, B.F64, 0xa000, 0x9000, B.F32, None, None) == B.ERR_UNSUPPORTED


def test_delta_options_validation(lib):
    """Section 4.1's delta form: same dtype in and out, tree order, aligned, and
    `out` either is `delta_start` or does not touch it."""
    good = [0x1000, 0x2000]
    offs = [0, 8]
    assert _call_reduce(lib, good, 2, offs, B.BF16, 0x9000, _opts(delta_start=0x5000, out_dtype=B.F32)) \
        == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(delta_start=0x5000, order=B.ORDER_LINEAR)) \
        == B.ERR_UNSUPPORTED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(delta_start=0x5004)) == B.ERR_MISALIGNED
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(delta_start=0x9010)) == B.ERR_ALIAS
    # a struct that ends before delta_start (the layout without the field) never reads it
    old = _opts(delta_start=0x5004)
    old.struct_bytes = B.Options.delta_start.offset
    assert _call_reduce(lib, good, 2, [0], B.F32, 0x9000, old) == B.OK
    # ... and one that ends before separate_passes (the layout with delta_start but without it) reads it as 0
    mid = _opts(delta_start=0x5004, separate_passes=1, reserved1=7)
    mid.struct_bytes = B.Options.separate_passes.offset
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, mid) == B.ERR_MISALIGNED   # delta_start is read
    assert _call_reduce(lib, good, 2, offs, B.F32, 0x9000, _opts(reserved1=1)) == B.ERR_INVALID_ARG
    # every pass reducing its own operands needs no room for what a combine leaves the next pass
    big4 = [0, 70632]
    assert B.adasum_workspace_bytes(64, big4, B.BF16, separate_passes=True) < B.adasum_workspace_bytes(64, big4, B.BF16)
    # the delta form defaults to radix 8: K = 16 takes two passes and needs intermediate nodes
    big = [0, 70632]
    assert B.adasum_workspace_bytes(16, big, B.F32, delta=True) > B.adasum_workspace_bytes(16, big, B.F32) + 70632 * 4


def test_step_entry_points_validate(lib):
    offs = (C.c_int64 * 3)(0, 10, 30)
    x = (C.c_void_p * 2)(0x1000, 0x2000)
    assert lib.adasum_group_gram(x, 3, offs, 2, B.F32, 0x9000, None) == B.ERR_UNSUPPORTED
    assert lib.adasum_group_gram(x, 2, offs, 2, 9, 0x9000, None) == B.ERR_UNSUPPORTED
    assert lib.adasum_group_gram(x, 2, offs, 2, B.F32, None, None) == B.ERR_INVALID_ARG
    assert lib.adasum_group_gram(None, 2, offs, 2, B.F32, 0x9000, None) == B.ERR_INVALID_ARG
    assert lib.adasum_group_weights(0x9000, 5, 2, 0, 0xa000, None) == B.ERR_UNSUPPORTED
    assert lib.adasum_group_weights(None, 2, 2, 0, 0xa000, None) == B.ERR_INVALID_ARG
    assert lib.adasum_group_weights(0x9000, 2, 0, 0, 0xa000, None) == B.OK
    assert lib.adasum_group_combine(x, 2, offs, 2, B.F32, None, 0x9000, B.F32, None, None) == B.ERR_INVALID_ARG
    assert lib.adasum_group_combine(x, 2, offs, 2, B.F32, 0xa000, 0x2010, B.F32, None, None) == B.ERR_ALIAS
    assert lib.adasum_group_combine(x, 2, offs, 2, B.F32, 0xa000, 0x9000, 3, None, None) == B.ERR_UNSUPPORTED


def test_binding_refuses_cpu_tensors():
    import torch
    g = [torch.zeros(8), torch.zeros(8)]
    with pytest.raises(ValueError):
        B.adasum_reduce(g, [0, 8])


def test_workspace_bytes(lib):
    offs = [0, 1000, 5096, 70632]
    n2 = B.adasum_workspace_bytes(4, offs, B.F32, radix=2)
    # two fp32 intermediate nodes of N elements (rounded up to 64) dominate
    assert n2 >= 2 * 70656 * 4
    assert n2 < 2 * 70656 * 4 + (1 << 20)
    # one pass over all four workers needs no intermediate node
    n4 = B.adasum_workspace_bytes(4, offs, B.F32, radix=4)
    assert n4 < (1 << 20)
    n = C.c_size_t(0)
    o = (C.c_int64 * 4)(*offs)
    # K = 3: two first-pass groups (1 and 2 workers) leave two fp32 nodes for the root pass
    assert lib.adasum_workspace_bytes(3, o, 3, B.F32, None, C.byref(n)) == B.OK
    assert n.value > 0
    assert B.adasum_workspace_bytes(3, offs, B.F32, radix=2) >= 2 * 70656 * 4
    assert lib.adasum_workspace_bytes(4, o, 3, B.F32, None, None) == B.ERR_INVALID_ARG


def test_plan_entry_points_validate(lib):
    offs = (C.c_int64 * 3)(0, 10, 30)
    h = C.c_void_p(None)
    assert lib.adasum_plan_create(4, offs, 2, B.F32, None, None) == B.ERR_INVALID_ARG
    assert lib.adasum_plan_create(0, offs, 2, B.F32, None, C.byref(h)) == B.ERR_INVALID_ARG
    assert lib.adasum_plan_create(4, offs, 2, 9, None, C.byref(h)) == B.ERR_UNSUPPORTED
    assert lib.adasum_plan_create(4, offs, 2, B.F64, C.byref(_opts(radix=16)), C.byref(h)) == B.ERR_UNSUPPORTED
    assert lib.adasum_plan_create(4, offs, 2, B.F32, C.byref(_opts(layer_stats=0x9000)), C.byref(h)) \
        == B.ERR_INVALID_ARG
    assert h.value is None
    assert lib.adasum_plan_execute(None, None, None, None, None, None) == B.ERR_INVALID_ARG
    assert lib.adasum_plan_destroy(None) == B.OK
    # an empty problem needs no device: the plan exists and executes as a no-op
    empty = (C.c_int64 * 2)(0, 0)
    assert lib.adasum_plan_create(2, empty, 1, B.BF16, None, C.byref(h)) == B.OK
    n = C.c_size_t(7)
    assert lib.adasum_plan_workspace_bytes(h, C.byref(n)) == B.OK and n.value == 0
    x = (C.c_void_p * 2)(0, 0)
    assert lib.adasum_plan_execute(h, x, None, None, None, None) == B.OK
    # a plan made without the delta form refuses a delta_start, and the other way round
    assert lib.adasum_plan_execute(h, x, None, None, 0x5000, None) == B.ERR_INVALID_ARG
    assert lib.adasum_plan_destroy(h) == B.OK


def test_header_is_plain_c(tmp_path):
    """include/adasum.h compiles as C (gcc, C99, pedantic): no C++ or HIP types at the boundary."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "adasum.h"\n'
        "int main(void) {\n"
        "    adasum_options o = {0};\n"
        "    adasum_plan* p = 0;\n"
        "    o.struct_bytes = (uint32_t)sizeof o;\n"
        "    return (adasum_plan_create(0, 0, 0, ADASUM_F32, &o, &p) == ADASUM_ERR_INVALID_ARG &&\n"
        "            adasum_reduce(0, 0, 0, 0, ADASUM_BF16, 0, 0) == ADASUM_ERR_INVALID_ARG) ? 0 : 1;\n"
        "}\n")
    exe = tmp_path / "use_header"
    libdir = os.path.join(ROOT, "paper_2006_02924_amd")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-ladasum", f"-Wl,-rpath,{libdir}"], check=True)
    assert subprocess.run([str(exe)]).returncode == 0
