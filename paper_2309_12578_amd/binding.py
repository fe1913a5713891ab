"""ctypes binding of libspion.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory (``torch.empty`` / ``data_ptr``) and the current HIP stream;
every step of the path runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspion.so")

SPION_F32, SPION_BF16 = 0, 1
SPION_T_ABS, SPION_T_QUANTILE, SPION_T_MEAN_KSTD = 0, 1, 2
SPION_PATTERN_NO_FILL = 1
SPION_PATTERN_POOL_ONLY = 2
SPION_PATTERN_FROM_POOL = 4
SPION_ATTN_PAPER_DENOM = 1
SPION_ATTN_BWD_QUERY_SIDE_ONLY = 2
SPION_ATTN_BWD_KEY_SIDE_ONLY = 4


class SpionError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {spion_strerror(code)} ({code})")


class _PatternParams(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("block", ctypes.c_int32), ("filter", ctypes.c_int32),
                ("thresh_mode", ctypes.c_int32), ("thresh_value", ctypes.c_double),
                ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class _AttnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32),
                ("d", ctypes.c_int32), ("block", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float), ("flags", ctypes.c_uint32)]


_lib: Optional[ctypes.CDLL] = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libspion.so (built in-tree by ``paper_2309_12578_amd.build``); raise if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2309_12578_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.spion_version.restype = ctypes.c_int
    lib.spion_strerror.restype = ctypes.c_char_p
    lib.spion_strerror.argtypes = [ctypes.c_int]
    lib.spion_pattern_workspace_bytes.restype = sz
    lib.spion_pattern_workspace_bytes.argtypes = [i32, i32]
    lib.spion_pattern.restype = ctypes.c_int
    lib.spion_pattern.argtypes = [vp, ctypes.POINTER(_PatternParams)] + [vp] * 8 + [vp, sz, vp]
    lib.spion_pattern_static.restype = ctypes.c_int
    lib.spion_pattern_static.argtypes = [vp, ctypes.POINTER(_PatternParams)] + [vp] * 8 + [vp]
    lib.spion_index_check.restype = ctypes.c_int
    lib.spion_index_check.argtypes = [vp] * 5 + [i32, i32, vp, vp]
    lib.spion_score_mean.restype = ctypes.c_int
    lib.spion_score_mean.argtypes = [vp, i32, i32, i32, vp, vp]
    lib.spion_frobenius_workspace_bytes.restype = sz
    lib.spion_frobenius_workspace_bytes.argtypes = []
    lib.spion_frobenius_distance.restype = ctypes.c_int
    lib.spion_frobenius_distance.argtypes = [vp, vp, ctypes.c_int64, vp, vp, sz, vp]
    lib.spion_copy_yardstick.restype = ctypes.c_int
    lib.spion_copy_yardstick.argtypes = [vp, vp, sz, vp]
    lib.spion_attn_workspace_bytes.restype = sz
    lib.spion_attn_workspace_bytes.argtypes = [ctypes.POINTER(_AttnParams), i32, i32]
    lib.spion_attn_fwd.restype = ctypes.c_int
    lib.spion_attn_fwd.argtypes = [vp] * 7 + [i32, ctypes.POINTER(_AttnParams), vp, sz, vp]
    lib.spion_attn_bwd.restype = ctypes.c_int
    lib.spion_attn_bwd.argtypes = [vp] * 14 + [i32, ctypes.POINTER(_AttnParams), vp, sz, vp]
    _lib = lib
    return lib


def spion_version() -> int:
    return int(load().spion_version())


def spion_strerror(code: int) -> str:
    return load().spion_strerror(int(code)).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libspion needs contiguous device tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SPION_F32
    if dt == torch.bfloat16:
        return SPION_BF16
    raise ValueError(f"unsupported dtype {dt}")


# ------------------------------------------------------------------------------------------------
# 1:1 wrappers of the C entry points
# ------------------------------------------------------------------------------------------------
def spion_pattern_workspace_bytes(L: int, block: int) -> int:
    return int(load().spion_pattern_workspace_bytes(L, block))


def spion_pattern(A_s, L, block, filt, thresh_mode, thresh_value, fl_out, row_ptr, col_idx, col_ptr,
                  row_idx, bsr_pos, nnzb, pool_sum, workspace, stream=None, flags: int = 0) -> None:
    p = _PatternParams(L, block, filt, thresh_mode, float(thresh_value), flags, 0)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spion_pattern(_ptr(A_s), ctypes.byref(p), _ptr(fl_out), _ptr(row_ptr), _ptr(col_idx),
                              _ptr(col_ptr), _ptr(row_idx), _ptr(bsr_pos), _ptr(nnzb), _ptr(pool_sum),
                              _ptr(workspace), ws_bytes, _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_pattern")


def spion_pattern_static(A_s, L, block, filt, thresh_mode, thresh_value, fl_out, row_ptr, col_idx, col_ptr,
                         row_idx, bsr_pos, nnzb, pool_sum, stream=None, flags: int = 0) -> None:
    p = _PatternParams(L, block, filt, thresh_mode, float(thresh_value), flags, 0)
    rc = load().spion_pattern_static(_ptr(A_s), ctypes.byref(p), _ptr(fl_out), _ptr(row_ptr), _ptr(col_idx),
                                     _ptr(col_ptr), _ptr(row_idx), _ptr(bsr_pos), _ptr(nnzb), _ptr(pool_sum),
                                     _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_pattern_static")


def spion_index_check(row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nb: int, nnzb: int, status,
                      stream=None) -> None:
    rc = load().spion_index_check(_ptr(row_ptr), _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx), _ptr(bsr_pos),
                                  int(nb), int(nnzb), _ptr(status), _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_index_check")


def spion_score_mean(A_maps, n_maps: int, L: int, dtype: int, A_s, stream=None) -> None:
    rc = load().spion_score_mean(_ptr(A_maps), int(n_maps), int(L), int(dtype), _ptr(A_s), _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_score_mean")


def spion_frobenius_workspace_bytes() -> int:
    return int(load().spion_frobenius_workspace_bytes())


def spion_frobenius_distance(A_prev, A_cur, n: int, out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spion_frobenius_distance(_ptr(A_prev), _ptr(A_cur), int(n), _ptr(out), _ptr(workspace),
                                         ws_bytes, _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_frobenius_distance")


def spion_copy_yardstick(src, dst, n_bytes: int, stream=None) -> None:
    rc = load().spion_copy_yardstick(_ptr(src), _ptr(dst), int(n_bytes), _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_copy_yardstick")


def _attn_params(B, H, L, d, block, dtype, scale, flags) -> _AttnParams:
    return _AttnParams(B, H, L, d, block, dtype, float(scale), flags)


def spion_attn_workspace_bytes(B, H, L, d, block, dtype, nnzb, is_bwd, scale=0.0, flags=0) -> int:
    p = _attn_params(B, H, L, d, block, dtype, scale, flags)
    n = int(load().spion_attn_workspace_bytes(ctypes.byref(p), nnzb, int(is_bwd)))
    if n == ctypes.c_size_t(-1).value:
        raise SpionError(-2, "spion_attn_workspace_bytes")
    return n


def spion_attn_fwd(Q, K, V, O, LSE, row_ptr, col_idx, nnzb, B, H, L, d, block, dtype, scale=0.0,
                   flags=0, workspace=None, stream=None) -> None:
    p = _attn_params(B, H, L, d, block, dtype, scale, flags)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spion_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(row_ptr),
                               _ptr(col_idx), int(nnzb), ctypes.byref(p), _ptr(workspace), ws_bytes,
                               _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_attn_fwd")


def spion_attn_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nnzb,
                   B, H, L, d, block, dtype, scale=0.0, flags=0, workspace=None, stream=None) -> None:
    p = _attn_params(B, H, L, d, block, dtype, scale, flags)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spion_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ),
                               _ptr(dK), _ptr(dV), _ptr(row_ptr), _ptr(col_idx), _ptr(col_ptr),
                               _ptr(row_idx), _ptr(bsr_pos), int(nnzb), ctypes.byref(p),
                               _ptr(workspace), ws_bytes, _stream(stream))
    if rc != 0:
        raise SpionError(rc, "spion_attn_bwd")


# ------------------------------------------------------------------------------------------------
# conveniences: allocate the outputs with torch, then call the entry points above
# ------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class Pattern:
    L: int
    block: int
    fl_out: torch.Tensor     # [nb, nb] uint8
    row_ptr: torch.Tensor    # [nb + 1] int32
    col_idx: torch.Tensor    # [nb * nb] int32, first nnzb valid
    col_ptr: torch.Tensor
    row_idx: torch.Tensor
    bsr_pos: torch.Tensor
    nnzb_dev: torch.Tensor   # [1] int32 on device
    pool_sum: torch.Tensor   # [nb, nb] int64
    nnzb: int = -1           # host copy, filled by generate_pattern(sync=True)

    @property
    def nb(self) -> int:
        return self.L // self.block


def generate_pattern(A_s: torch.Tensor, block: int, filt: int, thresh_mode: int, thresh_value: float,
                     flags: int = 0, sync: bool = True, out: Optional[Pattern] = None,
                     workspace: Optional[torch.Tensor] = None) -> Pattern:
    L = A_s.shape[0]
    nb = L // block
    dev = A_s.device
    if out is None:
        i32 = dict(dtype=torch.int32, device=dev)
        out = Pattern(L, block, torch.empty((nb, nb), dtype=torch.uint8, device=dev),
                      torch.empty(nb + 1, **i32), torch.empty(nb * nb, **i32),
                      torch.empty(nb + 1, **i32), torch.empty(nb * nb, **i32),
                      torch.empty(nb * nb, **i32), torch.empty(1, **i32),
                      torch.empty((nb, nb), dtype=torch.int64, device=dev))
    if workspace is None:
        workspace = torch.empty(max(spion_pattern_workspace_bytes(L, block), 256), dtype=torch.uint8,
                                device=dev)
    spion_pattern(A_s, L, block, filt, thresh_mode, thresh_value, out.fl_out, out.row_ptr, out.col_idx,
                  out.col_ptr, out.row_idx, out.bsr_pos, out.nnzb_dev, out.pool_sum, workspace,
                  flags=flags)
    if sync:
        out.nnzb = int(out.nnzb_dev.item())
    return out


def index_is_well_formed(pat: Pattern) -> bool:
    """Runs spion_index_check on a pattern's index (synchronises to read the verdict back)."""
    status = torch.empty(1, dtype=torch.int32, device=pat.row_ptr.device)
    spion_index_check(pat.row_ptr, pat.col_idx, pat.col_ptr, pat.row_idx, pat.bsr_pos, pat.nb, pat.nnzb,
                      status)
    return int(status.item()) == 0


def score_mean(A_maps: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """A_maps [n_maps, L, L] (fp32 or bf16) -> fp32 [L, L] mean map."""
    n_maps, L, _ = A_maps.shape
    if out is None:
        out = torch.empty((L, L), dtype=torch.float32, device=A_maps.device)
    spion_score_mean(A_maps, n_maps, L, _dtype_code(A_maps.dtype), out)
    return out


def frobenius_distance(A_prev: torch.Tensor, A_cur: torch.Tensor, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 2 on two fp32 maps; returns a device tensor {distance, ||A_prev||_F, ||A_cur||_F} (fp64)."""
    if out is None:
        out = torch.empty(3, dtype=torch.float64, device=A_prev.device)
    if workspace is None:
        workspace = torch.empty(spion_frobenius_workspace_bytes(), dtype=torch.uint8, device=A_prev.device)
    spion_frobenius_distance(A_prev, A_cur, A_prev.numel(), out, workspace)
    return out


def attn_fwd(Q, K, V, pat: Pattern, scale: float = 0.0, flags: int = 0,
             O: Optional[torch.Tensor] = None, LSE: Optional[torch.Tensor] = None
             ) -> Tuple[torch.Tensor, torch.Tensor]:
    B, H, L, d = Q.shape
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
    spion_attn_fwd(Q, K, V, O, LSE, pat.row_ptr, pat.col_idx, pat.nnzb, B, H, L, d, pat.block,
                   _dtype_code(Q.dtype), scale, flags)
    return O, LSE


def attn_bwd(Q, K, V, O, dO, LSE, pat: Pattern, scale: float = 0.0, flags: int = 0,
             dQ=None, dK=None, dV=None, workspace: Optional[torch.Tensor] = None):
    B, H, L, d = Q.shape
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    code = _dtype_code(Q.dtype)
    if workspace is None:
        n = spion_attn_workspace_bytes(B, H, L, d, pat.block, code, pat.nnzb, True, scale, flags)
        workspace = torch.empty(max(n, 256), dtype=torch.uint8, device=Q.device)
    spion_attn_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, pat.row_ptr, pat.col_idx, pat.col_ptr, pat.row_idx,
                   pat.bsr_pos, pat.nnzb, B, H, L, d, pat.block, code, scale, flags, workspace)
    return dQ, dK, dV
