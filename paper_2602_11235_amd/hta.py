"""Thin ctypes binding of libmtfm_hta.so (C ABI declared in include/mtfm_hta.h; timing hooks in mtfm_hta_timing.h).

Argument marshalling only: every step of the attention runs in the library's HIP kernels.
PyTorch appears here for device memory and streams and nothing else.  If the shared library is
missing this module raises on first use -- there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

BF16, FP32 = 0, 1
LAYER_FULL, LAYER_TARGET = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = 0, -1, -2, -3, -4

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmtfm_hta.so")
EXPORTS = ("mtfm_hta_workspace_bytes", "mtfm_hta_fwd", "mtfm_hta_fwd_static", "mtfm_hta_bwd", "mtfm_hta_validate_host",
           "mtfm_hta_workspace_bytes_rt", "mtfm_hta_fwd_rt", "mtfm_hta_bwd_rt", "mtfm_hta_validate_host_rt",
           "mtfm_hta_last_error", "mtfm_hta_version", "mtfm_hta_timing_enable", "mtfm_hta_timing_read")
KERNEL_FWD, KERNEL_BWD_SELF, KERNEL_BWD_DQ, KERNEL_BWD_DKDV = 0, 1, 2, 3

_lib = None


class HtaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"mtfm_hta status {status}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library (built by paper_2602_11235_amd/build.py) and declare its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2602_11235_amd.build` "
                                "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz, ci = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t,
                                 ctypes.c_int)
    lib.mtfm_hta_workspace_bytes.restype = sz
    lib.mtfm_hta_workspace_bytes.argtypes = [ci, ci, ci, i32, i64, i64, i32, i32, i32, i32, i32]
    tail = [i32, i64, i64, i32, i32, i32, i32, i32, f32, ci, ci, vp, sz, vp]
    lib.mtfm_hta_fwd.restype = ci
    lib.mtfm_hta_fwd.argtypes = [vp] * 9 + tail
    lib.mtfm_hta_fwd_static.restype = ci
    lib.mtfm_hta_fwd_static.argtypes = [vp] * 9 + tail[:-3] + [vp]
    lib.mtfm_hta_bwd.restype = ci
    lib.mtfm_hta_bwd.argtypes = [vp] * 13 + tail
    lib.mtfm_hta_validate_host.restype = ci
    lib.mtfm_hta_validate_host.argtypes = [vp, vp, vp, vp, i32, i64, i64, i32, i32, ci]
    # samples with real-time tokens: rt_len / timestamps pointers and max_rt are extra
    lib.mtfm_hta_workspace_bytes_rt.restype = sz
    lib.mtfm_hta_workspace_bytes_rt.argtypes = [ci, ci, ci, i32, i64, i64, i32, i32, i32, i32, i32, i32]
    tail_rt = [i32, i64, i64, i32, i32, i32, i32, i32, i32, f32, ci, ci, vp, sz, vp]
    lib.mtfm_hta_fwd_rt.restype = ci
    lib.mtfm_hta_fwd_rt.argtypes = [vp] * 11 + tail_rt
    lib.mtfm_hta_bwd_rt.restype = ci
    lib.mtfm_hta_bwd_rt.argtypes = [vp] * 15 + tail_rt
    lib.mtfm_hta_validate_host_rt.restype = ci
    lib.mtfm_hta_validate_host_rt.argtypes = [vp] * 6 + [i32, i64, i64, i32, i32, i32, ci]
    lib.mtfm_hta_last_error.restype = ctypes.c_char_p
    lib.mtfm_hta_last_error.argtypes = []
    lib.mtfm_hta_version.restype = ctypes.c_char_p
    lib.mtfm_hta_version.argtypes = []
    lib.mtfm_hta_timing_enable.restype = ci
    lib.mtfm_hta_timing_enable.argtypes = [ci]
    lib.mtfm_hta_timing_read.restype = ci
    lib.mtfm_hta_timing_read.argtypes = [ci, ctypes.POINTER(f32), ci]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int):
    if status != OK:
        raise HtaError(status, load_library().mtfm_hta_last_error().decode())


def mtfm_hta_version() -> str:
    return load_library().mtfm_hta_version().decode()


def mtfm_hta_last_error() -> str:
    return load_library().mtfm_hta_last_error().decode()


def mtfm_hta_timing_enable(slots: int) -> None:
    _check(load_library().mtfm_hta_timing_enable(int(slots)))


def mtfm_hta_timing_read(kernel: int, capacity: int = 4096):
    """Durations (ms) recorded for one kernel kind since the last read, oldest first (blocks on the events)."""
    buf = (ctypes.c_float * capacity)()
    n = load_library().mtfm_hta_timing_read(int(kernel), buf, capacity)
    if n < 0:
        raise HtaError(n, "mtfm_hta_timing_read failed")
    return [float(buf[i]) for i in range(n)]


def mtfm_hta_workspace_bytes(layer, dtype, is_bwd, batch, total_q, total_kv, max_hist, max_targets, Hq, Hkv,
                             head_dim) -> int:
    n = load_library().mtfm_hta_workspace_bytes(layer, dtype, int(is_bwd), batch, total_q, total_kv, max_hist,
                                                max_targets, Hq, Hkv, head_dim)
    if n == ctypes.c_size_t(-1).value:
        raise HtaError(ERR_INVALID_ARG, mtfm_hta_last_error())
    return int(n)


def mtfm_hta_validate_host(q_offsets, kv_offsets, hist_len, n_targets, batch, total_q, total_kv, max_hist,
                           max_targets, layer) -> None:
    """Arguments are CPU int32 tensors (or NumPy arrays converted by the caller)."""
    _check(load_library().mtfm_hta_validate_host(_ptr(q_offsets), _ptr(kv_offsets), _ptr(hist_len),
                                                 _ptr(n_targets), batch, total_q, total_kv, max_hist,
                                                 max_targets, layer))


def mtfm_hta_fwd(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, n_targets, batch, total_q, total_kv,
                 max_hist, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, workspace=None,
                 workspace_bytes=0, stream=None) -> None:
    """Enqueue the forward pass; tensors are device tensors (or raw device addresses)."""
    _check(load_library().mtfm_hta_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(q_offsets),
                                       _ptr(kv_offsets), _ptr(hist_len), _ptr(n_targets), batch, total_q,
                                       total_kv, max_hist, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype,
                                       layer, _ptr(workspace), workspace_bytes, _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 8 << 20


def mtfm_hta_fwd_static(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, n_targets, batch, total_q, total_kv,
                        max_hist, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, stream=None) -> None:
    """The forward pass without a workspace argument: scratch memory built into the library, nothing allocated."""
    _check(load_library().mtfm_hta_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(q_offsets),
                                              _ptr(kv_offsets), _ptr(hist_len), _ptr(n_targets), batch, total_q,
                                              total_kv, max_hist, max_targets, Hq, Hkv, head_dim, softmax_scale,
                                              dtype, layer, _stream_handle(stream)))


def mtfm_hta_bwd(dout, q, k, v, out, lse, dq, dk, dv, q_offsets, kv_offsets, hist_len, n_targets, batch, total_q,
                 total_kv, max_hist, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, workspace=None,
                 workspace_bytes=0, stream=None) -> None:
    """Enqueue the backward pass; tensors are device tensors (or raw device addresses)."""
    _check(load_library().mtfm_hta_bwd(_ptr(dout), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dq),
                                       _ptr(dk), _ptr(dv), _ptr(q_offsets), _ptr(kv_offsets), _ptr(hist_len),
                                       _ptr(n_targets), batch, total_q, total_kv, max_hist, max_targets, Hq, Hkv,
                                       head_dim, softmax_scale, dtype, layer, _ptr(workspace), workspace_bytes,
                                       _stream_handle(stream)))


def mtfm_hta_workspace_bytes_rt(layer, dtype, is_bwd, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq,
                                Hkv, head_dim) -> int:
    n = load_library().mtfm_hta_workspace_bytes_rt(layer, dtype, int(is_bwd), batch, total_q, total_kv, max_hist,
                                                   max_rt, max_targets, Hq, Hkv, head_dim)
    if n == ctypes.c_size_t(-1).value:
        raise HtaError(ERR_INVALID_ARG, mtfm_hta_last_error())
    return int(n)


def mtfm_hta_validate_host_rt(q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch, total_q,
                              total_kv, max_hist, max_rt, max_targets, layer) -> None:
    """Arguments are CPU int32 tensors (or NumPy arrays converted by the caller)."""
    _check(load_library().mtfm_hta_validate_host_rt(_ptr(q_offsets), _ptr(kv_offsets), _ptr(hist_len), _ptr(rt_len),
                                                    _ptr(n_targets), _ptr(timestamps), batch, total_q, total_kv,
                                                    max_hist, max_rt, max_targets, layer))


def mtfm_hta_fwd_rt(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch,
                    total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer,
                    workspace=None, workspace_bytes=0, stream=None) -> None:
    """Forward pass for samples with real-time tokens (mask rule 2)."""
    _check(load_library().mtfm_hta_fwd_rt(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(q_offsets),
                                          _ptr(kv_offsets), _ptr(hist_len), _ptr(rt_len), _ptr(n_targets),
                                          _ptr(timestamps), batch, total_q, total_kv, max_hist, max_rt, max_targets,
                                          Hq, Hkv, head_dim, softmax_scale, dtype, layer, _ptr(workspace),
                                          workspace_bytes, _stream_handle(stream)))


def mtfm_hta_bwd_rt(dout, q, k, v, out, lse, dq, dk, dv, q_offsets, kv_offsets, hist_len, rt_len, n_targets,
                    timestamps, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim,
                    softmax_scale, dtype, layer, workspace=None, workspace_bytes=0, stream=None) -> None:
    """Backward pass for samples with real-time tokens (mask rule 2)."""
    _check(load_library().mtfm_hta_bwd_rt(_ptr(dout), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dq),
                                          _ptr(dk), _ptr(dv), _ptr(q_offsets), _ptr(kv_offsets), _ptr(hist_len),
                                          _ptr(rt_len), _ptr(n_targets), _ptr(timestamps), batch, total_q, total_kv,
                                          max_hist, max_rt, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype,
                                          layer, _ptr(workspace), workspace_bytes, _stream_handle(stream)))


# --------------------------------------------------------------------------- buffer plumbing
class Batch:
    """Device buffers of one jagged batch plus the host-known scalars the C ABI wants.  Allocation and
    marshalling only; ``forward`` / ``backward`` call straight into the library."""

    def __init__(self, q, k, v, q_offsets, kv_offsets, hist_len, n_targets, max_hist, max_targets, softmax_scale,
                 layer, rt_len=None, timestamps=None, max_rt=0):
        assert q.is_cuda and k.is_cuda and v.is_cuda, "HTA runs on the GPU only"
        assert q.dtype in (torch.bfloat16, torch.float32) and k.dtype == q.dtype and v.dtype == q.dtype
        assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
        for t in (q_offsets, kv_offsets, hist_len, n_targets):
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
        self.q, self.k, self.v = q, k, v
        self.q_offsets, self.kv_offsets, self.hist_len, self.n_targets = q_offsets, kv_offsets, hist_len, n_targets
        self.batch = int(hist_len.shape[0])
        self.total_q, self.Hq, self.head_dim = int(q.shape[0]), int(q.shape[1]), int(q.shape[2])
        self.total_kv, self.Hkv = int(k.shape[0]), int(k.shape[1])
        self.max_hist, self.max_targets = int(max_hist), int(max_targets)
        assert (rt_len is None) == (timestamps is None)
        self.rt_len, self.timestamps, self.max_rt = rt_len, timestamps, int(max_rt)
        if rt_len is not None:
            for t in (rt_len, timestamps):
                assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
        self.softmax_scale, self.layer = float(softmax_scale), int(layer)
        self.dtype = BF16 if q.dtype == torch.bfloat16 else FP32
        self.out = torch.empty_like(q)
        self.lse = torch.empty((self.Hq, self.total_q), dtype=torch.float32, device=q.device)
        self.dq = self.dk = self.dv = None
        self.fwd_workspace_bytes = self._workspace_bytes(False)
        self.fwd_workspace = None
        if self.fwd_workspace_bytes:
            self.fwd_workspace = torch.empty(self.fwd_workspace_bytes, dtype=torch.uint8, device=q.device)
        self.workspace = None
        self.workspace_bytes = 0

    def _sizes(self):
        if self.rt_len is None:
            return (self.batch, self.total_q, self.total_kv, self.max_hist, self.max_targets, self.Hq, self.Hkv,
                    self.head_dim)
        return (self.batch, self.total_q, self.total_kv, self.max_hist, self.max_rt, self.max_targets, self.Hq,
                self.Hkv, self.head_dim)

    def _workspace_bytes(self, is_bwd: bool) -> int:
        fn = mtfm_hta_workspace_bytes if self.rt_len is None else mtfm_hta_workspace_bytes_rt
        return fn(self.layer, self.dtype, is_bwd, *self._sizes())

    def forward(self, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
        if self.rt_len is None:
            mtfm_hta_fwd(self.q, self.k, self.v, self.out, self.lse, self.q_offsets, self.kv_offsets, self.hist_len,
                         self.n_targets, *self._sizes(), self.softmax_scale, self.dtype, self.layer,
                         self.fwd_workspace, self.fwd_workspace_bytes, stream)
        else:
            mtfm_hta_fwd_rt(self.q, self.k, self.v, self.out, self.lse, self.q_offsets, self.kv_offsets, self.hist_len,
                            self.rt_len, self.n_targets, self.timestamps, *self._sizes(), self.softmax_scale,
                            self.dtype, self.layer, self.fwd_workspace, self.fwd_workspace_bytes, stream)
        return self.out, self.lse

    def prepare_backward(self) -> None:
        if self.dq is None:
            self.dq, self.dk, self.dv = torch.empty_like(self.q), torch.empty_like(self.k), torch.empty_like(self.v)
            self.workspace_bytes = self._workspace_bytes(True)
            if self.workspace_bytes:
                self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.q.device)
                assert self.workspace.data_ptr() % 256 == 0

    def backward(self, dout, stream=None):
        assert dout.is_cuda and dout.dtype == self.q.dtype and dout.shape == self.q.shape and dout.is_contiguous()
        self.prepare_backward()
        if self.rt_len is None:
            mtfm_hta_bwd(dout, self.q, self.k, self.v, self.out, self.lse, self.dq, self.dk, self.dv, self.q_offsets,
                         self.kv_offsets, self.hist_len, self.n_targets, *self._sizes(), self.softmax_scale,
                         self.dtype, self.layer, self.workspace, self.workspace_bytes, stream)
        else:
            mtfm_hta_bwd_rt(dout, self.q, self.k, self.v, self.out, self.lse, self.dq, self.dk, self.dv,
                            self.q_offsets, self.kv_offsets, self.hist_len, self.rt_len, self.n_targets,
                            self.timestamps, *self._sizes(), self.softmax_scale, self.dtype, self.layer,
                            self.workspace, self.workspace_bytes, stream)
        return self.dq, self.dk, self.dv
