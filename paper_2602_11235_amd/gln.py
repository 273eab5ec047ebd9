"""Thin ctypes binding of the group-layer-normalization entry points of libmtfm_hta.so (C ABI declared in
include/mtfm_gln.h).  Argument marshalling only; PyTorch supplies device memory and the stream.  There is no
fallback: without the built library the first call raises."""
from __future__ import annotations

import ctypes
from typing import Optional, Tuple

import torch

from . import hta

EXPORTS = ("mtfm_gln_fwd", "mtfm_gln_bwd", "mtfm_gln_bwd_workspace_bytes", "mtfm_gln_validate_host")
KERNEL_FWD, KERNEL_BWD, KERNEL_BWD_REDUCE = 4, 5, 6

_declared = False


def load_library() -> ctypes.CDLL:
    global _declared
    lib = hta.load_library()
    if not _declared:
        vp, i32, i64, f32, sz, ci = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t,
                                     ctypes.c_int)
        lib.mtfm_gln_fwd.restype = ci
        lib.mtfm_gln_fwd.argtypes = [vp] * 8 + [i64, i32, i32, f32, ci, vp]
        lib.mtfm_gln_bwd_workspace_bytes.restype = sz
        lib.mtfm_gln_bwd_workspace_bytes.argtypes = [i32, i32]
        lib.mtfm_gln_bwd.restype = ci
        lib.mtfm_gln_bwd.argtypes = [vp] * 12 + [i64, i32, i32, ci, vp, sz, vp]
        lib.mtfm_gln_validate_host.restype = ci
        lib.mtfm_gln_validate_host.argtypes = [vp, i64, i32]
        _declared = True
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return hta.BF16
    if t.dtype == torch.float32:
        return hta.FP32
    raise TypeError(f"unsupported element type {t.dtype}")


def _check(status: int) -> None:
    if status != hta.OK:
        raise hta.HtaError(status, hta.mtfm_hta_last_error())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def mtfm_gln_bwd_workspace_bytes(d_model: int, n_groups: int) -> int:
    return int(load_library().mtfm_gln_bwd_workspace_bytes(d_model, n_groups))


def mtfm_gln_validate_host(group_id: torch.Tensor, n_groups: int) -> None:
    g = group_id.detach().to("cpu", torch.int32).contiguous()
    _check(load_library().mtfm_gln_validate_host(g.data_ptr(), g.numel(), n_groups))


def mtfm_gln_fwd(x: torch.Tensor, group_id: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float,
                 gate: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None,
                 save_stats: bool = True, stats=None) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
    """y = GLN(x) (times gate); returns (y, mean, rstd), the statistics being None when save_stats is False.
    `stats` may hold preallocated (mean, rstd) tensors."""
    lib = load_library()
    n, d = x.shape
    if y is None:
        y = torch.empty_like(x)
    if stats is not None:
        mean, rstd = stats
    else:
        mean = torch.empty(n, dtype=torch.float32, device=x.device) if save_stats else None
        rstd = torch.empty(n, dtype=torch.float32, device=x.device) if save_stats else None
    _check(lib.mtfm_gln_fwd(hta._ptr(x), hta._ptr(gate), hta._ptr(group_id), hta._ptr(gamma), hta._ptr(beta),
                            hta._ptr(y), hta._ptr(mean), hta._ptr(rstd), n, d, gamma.shape[0], eps, _dtype_code(x),
                            _stream()))
    return y, mean, rstd


def mtfm_gln_bwd(dy: torch.Tensor, x: torch.Tensor, group_id: torch.Tensor, gamma: torch.Tensor,
                 beta: Optional[torch.Tensor], mean: torch.Tensor, rstd: torch.Tensor,
                 gate: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, out=None):
    """Returns (dx, dgamma, dbeta, dgate); dgate is None without a gate.  `out` may hold preallocated
    (dx, dgamma, dbeta, dgate) tensors."""
    lib = load_library()
    n, d = x.shape
    groups = gamma.shape[0]
    if out is None:
        out = (torch.empty_like(x), torch.empty_like(gamma), torch.empty_like(gamma),
               None if gate is None else torch.empty_like(x))
    dx, dgamma, dbeta, dgate = out
    need = mtfm_gln_bwd_workspace_bytes(d, groups)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _check(lib.mtfm_gln_bwd(hta._ptr(dy), hta._ptr(x), hta._ptr(gate), hta._ptr(group_id), hta._ptr(gamma),
                            hta._ptr(beta), hta._ptr(mean), hta._ptr(rstd), hta._ptr(dx), hta._ptr(dgate),
                            hta._ptr(dgamma), hta._ptr(dbeta), n, d, groups, _dtype_code(x), hta._ptr(workspace),
                            workspace.numel(), _stream()))
    return dx, dgamma, dbeta, dgate
