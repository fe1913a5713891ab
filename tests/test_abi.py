"""The C-ABI library loads without a GPU, exports every symbol spion.h declares, and rejects bad
arguments on the host before touching the device (no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2309_12578_amd as sp
from paper_2309_12578_amd import accounting as acc
from paper_2309_12578_amd.binding import _AttnParams, _PatternParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "spion.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spion_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sp.load()
    names = _declared_symbols()
    assert {"spion_pattern", "spion_attn_fwd", "spion_attn_bwd", "spion_pattern_workspace_bytes",
            "spion_attn_workspace_bytes", "spion_strerror", "spion_version"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert sp.spion_version() >= 100
    assert "workspace" in sp.spion_strerror(-4)


def test_workspace_queries():
    assert sp.spion_pattern_workspace_bytes(4096, 64) > 0
    assert sp.spion_pattern_workspace_bytes(4096, 48) == 0          # unsupported block
    assert sp.spion_pattern_workspace_bytes(100, 16) == 0           # L % block != 0
    assert sp.spion_attn_workspace_bytes(4, 4, 4096, 64, 64, sp.SPION_BF16, 215, False) == 0
    assert sp.spion_attn_workspace_bytes(4, 4, 4096, 64, 64, sp.SPION_BF16, 215, True) >= 4 * 4 * 4096 * 4
    with pytest.raises(sp.SpionError):
        sp.spion_attn_workspace_bytes(4, 4, 4096, 32, 64, sp.SPION_BF16, 215, True)   # d != 64


def test_argument_errors_are_reported_before_any_launch():
    lib = sp.load()
    fake = ctypes.c_void_p(256)         # non-NULL, never dereferenced: validation fails first
    none = ctypes.c_void_p(None)
    p = _PatternParams(256, 16, 5, sp.SPION_T_QUANTILE, 0.5, 0, 0)
    args = [fake, ctypes.byref(p)] + [fake] * 8 + [fake, 1 << 20, none]
    bad = list(args)
    bad[0] = none
    assert lib.spion_pattern(*bad) == -1                                   # NULL A_s
    for field, value, code in (("filter", 4, -5), ("filter", 33, -5), ("block", 24, -2), ("L", 250, -2),
                               ("thresh_value", 1.5, -5), ("thresh_mode", 9, -5), ("flags", 8, -5),
                               ("reserved", 1, -5)):
        q = _PatternParams(256, 16, 5, sp.SPION_T_QUANTILE, 0.5, 0, 0)
        setattr(q, field, value)
        a = list(args)
        a[1] = ctypes.byref(q)
        assert lib.spion_pattern(*a) == code, field
    small = list(args)
    small[11] = 16                                                          # workspace too small
    assert lib.spion_pattern(*small) == -4
    odd = list(args)
    odd[10] = ctypes.c_void_p(264)                                          # misaligned workspace
    assert lib.spion_pattern(*odd) == -4
    partial_bsc = list(args)
    partial_bsc[6] = none                                                   # row_idx missing, others given
    assert lib.spion_pattern(*partial_bsc) == -1

    # the variant with the built-in scratch validates the same way and refuses what does not fit
    sargs = [fake, ctypes.byref(p)] + [fake] * 8 + [none]
    nul = list(sargs)
    nul[2] = none
    assert lib.spion_pattern_static(*nul) == -1
    big = _PatternParams(8192, 16, 5, sp.SPION_T_QUANTILE, 0.5, 0, 0)            # nb = 512 > 256
    sargs[1] = ctypes.byref(big)
    assert lib.spion_pattern_static(*sargs) == -8
    even = _PatternParams(256, 16, 4, sp.SPION_T_QUANTILE, 0.5, 0, 0)
    sargs[1] = ctypes.byref(even)
    assert lib.spion_pattern_static(*sargs) == -5
    # the built-in scratch (5 MiB) holds the workspace of the largest grid the variant accepts
    lib.spion_pattern_workspace_bytes.restype = ctypes.c_size_t
    assert 0 < lib.spion_pattern_workspace_bytes(256 * 64, 64) <= 5 << 20

    ap = _AttnParams(1, 1, 256, 64, 16, sp.SPION_F32, 0.0, 0)
    fargs = [fake] * 7 + [19, ctypes.byref(ap), none, 0, none]
    nul = list(fargs)
    nul[3] = none
    assert lib.spion_attn_fwd(*nul) == -1
    for field, value, code in (("d", 128, -2), ("block", 8, -2), ("dtype", 7, -3), ("scale", -1.0, -5),
                               ("flags", 64, -5), ("B", 0, -2)):
        q = _AttnParams(1, 1, 256, 64, 16, sp.SPION_F32, 0.0, 0)
        setattr(q, field, value)
        a = list(fargs)
        a[8] = ctypes.byref(q)
        assert lib.spion_attn_fwd(*a) == code, field
    too_many = list(fargs)
    too_many[7] = 16 * 16 + 1                                               # nnzb > nb^2
    assert lib.spion_attn_fwd(*too_many) == -2
    bargs = [fake] * 14 + [19, ctypes.byref(ap), none, 0, none]
    assert lib.spion_attn_bwd(*bargs) == -4                                 # backward needs a workspace
    both = _AttnParams(1, 1, 256, 64, 16, sp.SPION_F32, 0.0, 2 | 4)
    b2 = list(bargs)
    b2[15] = ctypes.byref(both)
    assert lib.spion_attn_bwd(*b2) == -5                                    # both "only" flags at once
    status = ctypes.c_void_p(512)
    assert lib.spion_index_check(fake, fake, none, none, none, 16, 19, none, none) == -1      # no status
    assert lib.spion_index_check(fake, fake, fake, none, none, 16, 19, status, none) == -1    # partial BSC
    assert lib.spion_index_check(fake, fake, none, none, none, 2000, 19, status, none) == -2  # nb too large
    assert lib.spion_index_check(fake, fake, none, none, none, 16, 257, status, none) == -2   # nnzb > nb^2
    # forward grid fits (B H nb < 2^31) but the key side of the backward would need more workgroups
    huge = _AttnParams(1 << 10, 1 << 10, 16384, 64, 16, sp.SPION_BF16, 0.0, 0)
    b3 = list(bargs)
    b3[14] = 1024 * 1024
    b3[15] = ctypes.byref(huge)
    assert lib.spion_attn_bwd(*b3) == -2


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(4)
    with pytest.raises(ValueError):
        sp.binding._ptr(x)


def test_paper_operation_counts():
    vals = {}
    for line in open(os.path.join(GOLDEN, "op_counts.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            vals[k] = int(v)
    assert acc.paper_ops_dense(vals["L"], vals["D"]) == vals["dense"]
    assert acc.paper_ops_sparse(vals["L"], vals["D"], vals["C"]) == vals["sparse"]
    assert acc.paper_ops_sddmm(64, 10) == 10 * 127


def test_useful_flop_and_byte_accounting():
    # 6 tile products of 2 * bs^2 * d FLOP per kept block and head
    assert acc.useful_flops(215, 64, 64, 16) == 12 * 64 * 64 * 64 * 215 * 16
    assert acc.useful_flops(1, 16, 64, 1, products=2) == 4 * 16 * 16 * 64
    t = 16 * 4096 * 64 * 2
    assert acc.algorithmic_bytes("path", 16, 4096, 64, 2) == 12 * t + 2 * 16 * 4096 * 4
    assert acc.algorithmic_bytes("fwd", 16, 4096, 64, 2) == 4 * t + 16 * 4096 * 4


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_product_package_does_not_import_the_oracle():
    # the oracle is test infrastructure: nothing under the package may reach it
    pkg = os.path.join(ROOT, "paper_2309_12578_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), name
