"""Thin ctypes binding of the pointwise variant of Hybrid Target Attention (C ABI declared in
include/mtfm_hta_pw.h): out_i = norm * sum over visible keys of silu(scale <q_i, k_j>) v_j.
Argument marshalling only; PyTorch supplies device memory and the stream; no fallback without the library."""
from __future__ import annotations

import ctypes

import torch

from . import hta

EXPORTS = ("mtfm_hta_pw_workspace_bytes", "mtfm_hta_pw_fwd", "mtfm_hta_pw_bwd",
           "mtfm_hta_pw_workspace_bytes_rt", "mtfm_hta_pw_fwd_rt", "mtfm_hta_pw_bwd_rt")

_declared = False


def load_library() -> ctypes.CDLL:
    global _declared
    lib = hta.load_library()
    if not _declared:
        vp, i32, i64, f32, sz, ci = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t,
                                     ctypes.c_int)
        lib.mtfm_hta_pw_workspace_bytes.restype = sz
        lib.mtfm_hta_pw_workspace_bytes.argtypes = [ci, ci, ci, i32, i64, i64, i32, i32, i32, i32, i32]
        tail = [i32, i64, i64, i32, i32, i32, i32, i32, f32, f32, ci, ci, vp, sz, vp]
        lib.mtfm_hta_pw_fwd.restype = ci
        lib.mtfm_hta_pw_fwd.argtypes = [vp] * 8 + tail
        lib.mtfm_hta_pw_bwd.restype = ci
        lib.mtfm_hta_pw_bwd.argtypes = [vp] * 11 + tail
        lib.mtfm_hta_pw_workspace_bytes_rt.restype = sz
        lib.mtfm_hta_pw_workspace_bytes_rt.argtypes = [ci, ci, ci, i32, i64, i64, i32, i32, i32, i32, i32, i32]
        tail_rt = [i32, i64, i64, i32, i32, i32, i32, i32, i32, f32, f32, ci, ci, vp, sz, vp]
        lib.mtfm_hta_pw_fwd_rt.restype = ci
        lib.mtfm_hta_pw_fwd_rt.argtypes = [vp] * 10 + tail_rt
        lib.mtfm_hta_pw_bwd_rt.restype = ci
        lib.mtfm_hta_pw_bwd_rt.argtypes = [vp] * 13 + tail_rt
        _declared = True
    return lib


def mtfm_hta_pw_workspace_bytes(layer, dtype, is_bwd, batch, total_q, total_kv, max_hist, max_targets, Hq, Hkv,
                                head_dim) -> int:
    n = load_library().mtfm_hta_pw_workspace_bytes(layer, dtype, int(is_bwd), batch, total_q, total_kv, max_hist,
                                                   max_targets, Hq, Hkv, head_dim)
    if n == ctypes.c_size_t(-1).value:
        raise hta.HtaError(hta.ERR_INVALID_ARG, hta.mtfm_hta_last_error())
    return int(n)


def mtfm_hta_pw_fwd(q, k, v, out, q_offsets, kv_offsets, hist_len, n_targets, batch, total_q, total_kv, max_hist,
                    max_targets, Hq, Hkv, head_dim, scale, norm, dtype, layer, workspace=None, workspace_bytes=0,
                    stream=None) -> None:
    P = hta._ptr
    hta._check(load_library().mtfm_hta_pw_fwd(P(q), P(k), P(v), P(out), P(q_offsets), P(kv_offsets), P(hist_len),
                                              P(n_targets), batch, total_q, total_kv, max_hist, max_targets, Hq, Hkv,
                                              head_dim, scale, norm, dtype, layer, P(workspace), workspace_bytes,
                                              hta._stream_handle(stream)))


def mtfm_hta_pw_bwd(dout, q, k, v, dq, dk, dv, q_offsets, kv_offsets, hist_len, n_targets, batch, total_q, total_kv,
                    max_hist, max_targets, Hq, Hkv, head_dim, scale, norm, dtype, layer, workspace=None,
                    workspace_bytes=0, stream=None) -> None:
    P = hta._ptr
    hta._check(load_library().mtfm_hta_pw_bwd(P(dout), P(q), P(k), P(v), P(dq), P(dk), P(dv), P(q_offsets),
                                              P(kv_offsets), P(hist_len), P(n_targets), batch, total_q, total_kv,
                                              max_hist, max_targets, Hq, Hkv, head_dim, scale, norm, dtype, layer,
                                              P(workspace), workspace_bytes, hta._stream_handle(stream)))


def mtfm_hta_pw_workspace_bytes_rt(layer, dtype, is_bwd, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq,
                                   Hkv, head_dim) -> int:
    n = load_library().mtfm_hta_pw_workspace_bytes_rt(layer, dtype, int(is_bwd), batch, total_q, total_kv, max_hist,
                                                      max_rt, max_targets, Hq, Hkv, head_dim)
    if n == ctypes.c_size_t(-1).value:
        raise hta.HtaError(hta.ERR_INVALID_ARG, hta.mtfm_hta_last_error())
    return int(n)


def mtfm_hta_pw_fwd_rt(q, k, v, out, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch, total_q,
                       total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, scale, norm, dtype, layer,
                       workspace=None, workspace_bytes=0, stream=None) -> None:
    P = hta._ptr
    hta._check(load_library().mtfm_hta_pw_fwd_rt(P(q), P(k), P(v), P(out), P(q_offsets), P(kv_offsets), P(hist_len),
                                                 P(rt_len), P(n_targets), P(timestamps), batch, total_q, total_kv,
                                                 max_hist, max_rt, max_targets, Hq, Hkv, head_dim, scale, norm, dtype,
                                                 layer, P(workspace), workspace_bytes, hta._stream_handle(stream)))


def mtfm_hta_pw_bwd_rt(dout, q, k, v, dq, dk, dv, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch,
                       total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, scale, norm, dtype, layer,
                       workspace=None, workspace_bytes=0, stream=None) -> None:
    P = hta._ptr
    hta._check(load_library().mtfm_hta_pw_bwd_rt(P(dout), P(q), P(k), P(v), P(dq), P(dk), P(dv), P(q_offsets),
                                                 P(kv_offsets), P(hist_len), P(rt_len), P(n_targets), P(timestamps),
                                                 batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv,
                                                 head_dim, scale, norm, dtype, layer, P(workspace), workspace_bytes,
                                                 hta._stream_handle(stream)))


class PointwiseBatch:
    """Device buffers of one jagged batch for the pointwise variant (allocation and marshalling only)."""

    def __init__(self, q, k, v, q_offsets, kv_offsets, hist_len, n_targets, max_hist, max_targets, scale, norm, layer,
                 rt_len=None, timestamps=None, max_rt=0):
        assert q.is_cuda and q.dtype in (torch.bfloat16, torch.float32) and k.dtype == q.dtype and v.dtype == q.dtype
        assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
        self.q, self.k, self.v = q, k, v
        assert (rt_len is None) == (timestamps is None)
        self.rt = rt_len is not None
        if self.rt:   # samples with real-time tokens: the *_rt entry points
            self.ints = (q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps)
            self.sizes = (int(hist_len.shape[0]), int(q.shape[0]), int(k.shape[0]), int(max_hist), int(max_rt),
                          int(max_targets), int(q.shape[1]), int(k.shape[1]), int(q.shape[2]))
        else:
            self.ints = (q_offsets, kv_offsets, hist_len, n_targets)
            self.sizes = (int(hist_len.shape[0]), int(q.shape[0]), int(k.shape[0]), int(max_hist), int(max_targets),
                          int(q.shape[1]), int(k.shape[1]), int(q.shape[2]))
        for t in self.ints:
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
        self.scale, self.norm, self.layer = float(scale), float(norm), int(layer)
        self.dtype = hta.BF16 if q.dtype == torch.bfloat16 else hta.FP32
        self.out = torch.empty_like(q)
        self.dq = self.dk = self.dv = None
        self.fwd_ws = self._workspace(False)
        self.bwd_ws = None

    def _workspace(self, is_bwd):
        fn = mtfm_hta_pw_workspace_bytes_rt if self.rt else mtfm_hta_pw_workspace_bytes
        n = fn(self.layer, self.dtype, is_bwd, *self.sizes)
        return torch.empty(n, dtype=torch.uint8, device=self.q.device) if n else None

    def forward(self, stream=None):
        ws = self.fwd_ws
        fn = mtfm_hta_pw_fwd_rt if self.rt else mtfm_hta_pw_fwd
        fn(self.q, self.k, self.v, self.out, *self.ints, *self.sizes, self.scale, self.norm, self.dtype, self.layer, ws,
           0 if ws is None else ws.numel(), stream)
        return self.out

    def prepare_backward(self):
        if self.dq is None:
            self.dq, self.dk, self.dv = torch.empty_like(self.q), torch.empty_like(self.k), torch.empty_like(self.v)
            self.bwd_ws = self._workspace(True)

    def backward(self, dout, stream=None):
        assert dout.is_cuda and dout.dtype == self.q.dtype and dout.shape == self.q.shape and dout.is_contiguous()
        self.prepare_backward()
        ws = self.bwd_ws
        fn = mtfm_hta_pw_bwd_rt if self.rt else mtfm_hta_pw_bwd
        fn(dout, self.q, self.k, self.v, self.dq, self.dk, self.dv, *self.ints, *self.sizes, self.scale, self.norm,
           self.dtype, self.layer, ws, 0 if ws is None else ws.numel(), stream)
        return self.dq, self.dk, self.dv
