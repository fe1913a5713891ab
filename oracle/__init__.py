"""ctypes front end of the CPU oracle (test infrastructure only).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It shares nothing with the GPU library; the product path never calls it.

The arithmetic lives in ``spion_oracle.c`` (plain C, fp64 / exact integers); this file only
builds it with gcc, marshals numpy arrays, and strings the steps of Algorithm 3 together in the
order the paper gives them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spion_oracle.c")
_LIB = os.path.join(_HERE, "libspion_oracle.so")

T_ABS, T_QUANTILE, T_MEAN_KSTD = 0, 1, 2
ATTN_PAPER_DENOM = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Thresh(ctypes.Structure):
    _fields_ = [("is_int", ctypes.c_int32), ("pad", ctypes.c_int32), ("ti", ctypes.c_int64),
                ("td", ctypes.c_double)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


# --------------------------------------------------------------------------------------------
# pattern generation, step by step
# --------------------------------------------------------------------------------------------
def quantize(A: np.ndarray) -> np.ndarray:
    A = np.ascontiguousarray(A, dtype=np.float32)
    out = np.empty(A.shape, dtype=np.int64)
    _chk(lib().oracle_quantize(_p(A), ctypes.c_int64(A.size), _p(out)), "quantize")
    return out


def conv_diag(aq: np.ndarray, F: int) -> np.ndarray:
    aq = np.ascontiguousarray(aq, dtype=np.int64)
    L = aq.shape[0]
    assert aq.shape == (L, L)
    out = np.empty((L, L), dtype=np.int64)
    _chk(lib().oracle_conv_diag(_p(aq), ctypes.c_int32(L), ctypes.c_int32(F), _p(out)), "conv_diag")
    return out


def pool_sum(conv: np.ndarray, bs: int) -> np.ndarray:
    conv = np.ascontiguousarray(conv, dtype=np.int64)
    L = conv.shape[0]
    nb = L // bs
    out = np.empty((nb, nb), dtype=np.int64)
    _chk(lib().oracle_pool_sum(_p(conv), ctypes.c_int32(L), ctypes.c_int32(bs), _p(out)), "pool_sum")
    return out


def threshold(ps: np.ndarray, bs: int, mode: int, value: float) -> _Thresh:
    ps = np.ascontiguousarray(ps, dtype=np.int64)
    t = _Thresh()
    _chk(lib().oracle_threshold(_p(ps), ctypes.c_int32(ps.shape[0]), ctypes.c_int32(bs),
                                ctypes.c_int32(mode), ctypes.c_double(value), ctypes.byref(t)),
         "threshold")
    return t


def make_thresh_int(ti: int) -> _Thresh:
    return _Thresh(1, 0, int(ti), float(ti))


def make_thresh_double(td: float) -> _Thresh:
    return _Thresh(0, 0, 0, float(td))


def fill(ps: np.ndarray, t: _Thresh, force_diag: bool = True) -> np.ndarray:
    ps = np.ascontiguousarray(ps, dtype=np.int64)
    nb = ps.shape[0]
    out = np.empty((nb, nb), dtype=np.uint8)
    rc = lib().oracle_fill(_p(ps), ctypes.c_int32(nb), ctypes.byref(t), ctypes.c_int32(int(force_diag)),
                           _p(out))
    _chk(rc, "fill")
    return out


def topk(ps: np.ndarray, t: _Thresh, force_diag: bool = True) -> np.ndarray:
    ps = np.ascontiguousarray(ps, dtype=np.int64)
    nb = ps.shape[0]
    out = np.empty((nb, nb), dtype=np.uint8)
    _chk(lib().oracle_topk(_p(ps), ctypes.c_int32(nb), ctypes.byref(t), ctypes.c_int32(int(force_diag)),
                           _p(out)), "topk")
    return out


def upsample(fl: np.ndarray, bs: int) -> np.ndarray:
    fl = np.ascontiguousarray(fl, dtype=np.uint8)
    nb = fl.shape[0]
    out = np.empty((nb * bs, nb * bs), dtype=np.uint8)
    _chk(lib().oracle_upsample(_p(fl), ctypes.c_int32(nb), ctypes.c_int32(bs), _p(out)), "upsample")
    return out


def compact(fl: np.ndarray) -> Dict[str, np.ndarray]:
    fl = np.ascontiguousarray(fl, dtype=np.uint8)
    nb = fl.shape[0]
    row_ptr = np.zeros(nb + 1, dtype=np.int32)
    col_idx = np.full(nb * nb, -1, dtype=np.int32)
    col_ptr = np.zeros(nb + 1, dtype=np.int32)
    row_idx = np.full(nb * nb, -1, dtype=np.int32)
    bsr_pos = np.full(nb * nb, -1, dtype=np.int32)
    nnzb = ctypes.c_int32(0)
    _chk(lib().oracle_compact(_p(fl), ctypes.c_int32(nb), _p(row_ptr), _p(col_idx), _p(col_ptr),
                              _p(row_idx), _p(bsr_pos), ctypes.byref(nnzb)), "compact")
    n = int(nnzb.value)
    return dict(row_ptr=row_ptr, col_idx=col_idx[:n].copy(), col_ptr=col_ptr,
                row_idx=row_idx[:n].copy(), bsr_pos=bsr_pos[:n].copy(), nnzb=n)


def generate_pattern(A: np.ndarray, bs: int, F: int, mode: int, value: float,
                     variant: str = "CF") -> Dict[str, np.ndarray]:
    """Algorithm 3 end to end.  variant "CF" = conv + fill, "F" = fill only (F forced to 1),
    "C" = conv + top blocks without fill (Section 5, "Models Compared")."""
    if variant == "F":
        F = 1
    aq = quantize(A)
    conv = conv_diag(aq, F)
    ps = pool_sum(conv, bs)
    t = threshold(ps, bs, mode, value)
    fl = topk(ps, t) if variant == "C" else fill(ps, t)
    out = compact(fl)
    out.update(pool_sum=ps, fl_out=fl, thresh=t)
    return out


# --------------------------------------------------------------------------------------------
# producers of the pattern input
# --------------------------------------------------------------------------------------------
def score_mean(maps: np.ndarray) -> np.ndarray:
    """maps: [n_maps, L, L]; element-wise mean in fp64."""
    maps = np.ascontiguousarray(maps, dtype=np.float64)
    n_maps = maps.shape[0]
    out = np.empty(maps.shape[1:], dtype=np.float64)
    _chk(lib().oracle_score_mean(_p(maps), ctypes.c_int32(n_maps), ctypes.c_int64(out.size), _p(out)),
         "score_mean")
    return out


def frobenius_distance(a: np.ndarray, b: np.ndarray):
    """Eq. 2; returns (distance, ||a||_F, ||b||_F) in fp64."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    assert a.size == b.size
    out = np.empty(3, dtype=np.float64)
    _chk(lib().oracle_frobenius_distance(_p(a), _p(b), ctypes.c_int64(a.size), _p(out)), "frobenius_distance")
    return float(out[0]), float(out[1]), float(out[2])


# --------------------------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------------------------
def _f64(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float64)


def attn_fwd(Q, K, V, P, scale: Optional[float] = None, flags: int = 0):
    """Q, K, V: [BH, L, d]; P: [L, L] uint8.  Returns (O, LSE) in fp64."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    P = np.ascontiguousarray(P, dtype=np.uint8)
    BH, L, d = Q.shape
    assert P.shape == (L, L)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    O = np.empty_like(Q)
    LSE = np.empty((BH, L), dtype=np.float64)
    _chk(lib().oracle_attn_fwd(_p(Q), _p(K), _p(V), _p(P), ctypes.c_int32(BH), ctypes.c_int32(L),
                               ctypes.c_int32(d), ctypes.c_double(scale), ctypes.c_int32(flags),
                               _p(O), _p(LSE)), "attn_fwd")
    return O, LSE


def attn_bwd(Q, K, V, dO, P, scale: Optional[float] = None, flags: int = 0):
    """Returns (dQ, dK, dV) in fp64."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    P = np.ascontiguousarray(P, dtype=np.uint8)
    BH, L, d = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    _chk(lib().oracle_attn_bwd(_p(Q), _p(K), _p(V), _p(dO), _p(P), ctypes.c_int32(BH),
                               ctypes.c_int32(L), ctypes.c_int32(d), ctypes.c_double(scale),
                               ctypes.c_int32(flags), _p(dQ), _p(dK), _p(dV)), "attn_bwd")
    return dQ, dK, dV


def attn_probs_row(Q, K, P, bh: int, i: int, scale: Optional[float] = None, flags: int = 0):
    Q, K = _f64(Q), _f64(K)
    P = np.ascontiguousarray(P, dtype=np.uint8)
    BH, L, d = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    p = np.empty(L, dtype=np.float64)
    _chk(lib().oracle_attn_probs_row(_p(Q), _p(K), _p(P), ctypes.c_int32(L), ctypes.c_int32(d),
                                     ctypes.c_double(scale), ctypes.c_int32(flags), ctypes.c_int32(bh),
                                     ctypes.c_int32(i), _p(p)), "attn_probs_row")
    return p
