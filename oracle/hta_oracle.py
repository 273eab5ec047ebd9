"""ctypes front end of the float64 C oracle (oracle/hta_oracle.c).

TEST INFRASTRUCTURE ONLY.  The functions take NumPy arrays of any float dtype, widen them
exactly to float64 and return float64 results; there is no rounding anywhere in between.
Shapes: q/out/dout/dq [total_q, Hq, d]; k/v/dk/dv [total_kv, Hkv, d]; lse [Hq, total_q].
``layer``: 0 = full attention layer (every token is a query), 1 = target attention layer
(queries are the target tokens only) -- Section 3.2.2.
A sample may carry real-time tokens between its history and its target tokens (``rt_len`` per user,
``timestamps`` one int32 per K/V row): mask rule 2 of Section 3.2.2 then applies to them.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.hta_oracle_fwd.restype = ctypes.c_int
        lib.hta_oracle_fwd.argtypes = [dp, dp, dp, dp, dp, ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int64,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                       ctypes.c_int32]
        lib.hta_oracle_bwd.restype = ctypes.c_int
        lib.hta_oracle_bwd.argtypes = [dp] * 9 + [ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int64,
                                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_double, ctypes.c_int32]
        lib.hta_oracle_probs.restype = ctypes.c_int
        lib.hta_oracle_probs.argtypes = [dp, dp, dp] + [ctypes.c_int32] * 8 + [ctypes.c_double, ctypes.c_int32]
        lib.hta_oracle_fwd_rt.restype = ctypes.c_int
        lib.hta_oracle_fwd_rt.argtypes = [dp, dp, dp, dp, dp, ip, ip, ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int64,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                          ctypes.c_int32]
        lib.hta_oracle_bwd_rt.restype = ctypes.c_int
        lib.hta_oracle_bwd_rt.argtypes = [dp] * 9 + [ip, ip, ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int64,
                                                     ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                     ctypes.c_double, ctypes.c_int32]
        lib.hta_oracle_probs_rt.restype = ctypes.c_int
        lib.hta_oracle_probs_rt.argtypes = ([dp, dp, dp] + [ctypes.c_int32] * 5 + [ip] + [ctypes.c_int32] * 4 +
                                            [ctypes.c_double, ctypes.c_int32])
        lib.hta_oracle_pw_fwd_rt.restype = ctypes.c_int
        lib.hta_oracle_pw_fwd_rt.argtypes = [dp, dp, dp, dp, ip, ip, ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int32,
                                             ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                             ctypes.c_int32]
        lib.hta_oracle_pw_bwd_rt.restype = ctypes.c_int
        lib.hta_oracle_pw_bwd_rt.argtypes = [dp] * 7 + [ip, ip, ip, ip, ip, ip, ctypes.c_int32, ctypes.c_int32,
                                                        ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                                        ctypes.c_int32]
        lib.hta_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def num_threads() -> int:
    return int(_load().hta_oracle_num_threads())


def _check_shapes(q, k, v, q_start, kv_start, hist_len, n_targets, layer, rt_len=None, timestamps=None):
    assert q.ndim == 3 and k.ndim == 3 and k.shape == v.shape and q.shape[2] == k.shape[2]
    B = hist_len.shape[0]
    assert n_targets.shape[0] == B and q_start.shape[0] >= B and kv_start.shape[0] >= B
    assert (rt_len is None) == (timestamps is None)
    if rt_len is not None:
        assert rt_len.shape[0] == B and timestamps.shape[0] == k.shape[0]
    for b in range(B):
        L, T = int(hist_len[b]), int(n_targets[b])
        R = int(rt_len[b]) if rt_len is not None else 0
        assert L >= 0 and T >= 0 and R >= 0
        rows = L + R + T if layer == 0 else T
        assert 0 <= q_start[b] and q_start[b] + rows <= q.shape[0]
        assert 0 <= kv_start[b] and kv_start[b] + L + R + T <= k.shape[0]


def forward(q, k, v, q_offsets, kv_offsets, hist_len, n_targets, scale, layer, rt_len=None, timestamps=None):
    """Returns (out [total_q,Hq,d], lse [Hq,total_q]) in float64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    qs, ks, hl, nt = _i32(q_offsets), _i32(kv_offsets), _i32(hist_len), _i32(n_targets)
    rl = _i32(rt_len) if rt_len is not None else None
    ts = _i32(timestamps) if timestamps is not None else None
    _check_shapes(q, k, v, qs, ks, hl, nt, layer, rl, ts)
    tq, Hq, d = q.shape
    out = np.zeros_like(q)
    lse = np.zeros((Hq, tq), dtype=np.float64)
    if rl is None:
        rc = _load().hta_oracle_fwd(_dp(q), _dp(k), _dp(v), _dp(out), _dp(lse), _ip(qs), _ip(ks), _ip(hl), _ip(nt),
                                    hl.shape[0], tq, Hq, k.shape[1], d, float(scale), int(layer))
    else:
        rc = _load().hta_oracle_fwd_rt(_dp(q), _dp(k), _dp(v), _dp(out), _dp(lse), _ip(qs), _ip(ks), _ip(hl), _ip(rl),
                                       _ip(nt), _ip(ts), hl.shape[0], tq, Hq, k.shape[1], d, float(scale), int(layer))
    if rc != 0:
        raise ValueError("hta_oracle_fwd: invalid arguments")
    return out, lse


def backward(dout, q, k, v, out, lse, q_offsets, kv_offsets, hist_len, n_targets, scale, layer, rt_len=None,
             timestamps=None):
    """Returns (dq, dk, dv) in float64 for the upstream gradient ``dout``."""
    dout, q, k, v, out, lse = _f64(dout), _f64(q), _f64(k), _f64(v), _f64(out), _f64(lse)
    qs, ks, hl, nt = _i32(q_offsets), _i32(kv_offsets), _i32(hist_len), _i32(n_targets)
    rl = _i32(rt_len) if rt_len is not None else None
    ts = _i32(timestamps) if timestamps is not None else None
    _check_shapes(q, k, v, qs, ks, hl, nt, layer, rl, ts)
    assert dout.shape == q.shape and out.shape == q.shape and lse.shape == (q.shape[1], q.shape[0])
    tq, Hq, d = q.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    if rl is None:
        rc = _load().hta_oracle_bwd(_dp(dout), _dp(q), _dp(k), _dp(v), _dp(out), _dp(lse), _dp(dq), _dp(dk), _dp(dv),
                                    _ip(qs), _ip(ks), _ip(hl), _ip(nt), hl.shape[0], tq, Hq, k.shape[1], d,
                                    float(scale), int(layer))
    else:
        rc = _load().hta_oracle_bwd_rt(_dp(dout), _dp(q), _dp(k), _dp(v), _dp(out), _dp(lse), _dp(dq), _dp(dk),
                                       _dp(dv), _ip(qs), _ip(ks), _ip(hl), _ip(rl), _ip(nt), _ip(ts), hl.shape[0], tq,
                                       Hq, k.shape[1], d, float(scale), int(layer))
    if rc != 0:
        raise ValueError("hta_oracle_bwd: invalid arguments")
    return dq, dk, dv


def probs(q, k, q_start, kv_start, hist_len, n_targets, head, scale, layer, rt_len=0, timestamps=None):
    """Dense attention probabilities [n_rows, L+R+T] of one user and one query head (0 where masked)."""
    q, k = _f64(q), _f64(k)
    N = int(hist_len) + int(rt_len) + int(n_targets)
    rows = N if layer == 0 else int(n_targets)
    assert q_start + rows <= q.shape[0] and kv_start + N <= k.shape[0]
    p = np.zeros((rows, N), dtype=np.float64)
    if timestamps is None:
        assert rt_len == 0
        rc = _load().hta_oracle_probs(_dp(q), _dp(k), _dp(p), int(q_start), int(kv_start), int(hist_len),
                                      int(n_targets), int(head), q.shape[1], k.shape[1], q.shape[2], float(scale),
                                      int(layer))
    else:
        ts = _i32(timestamps)
        assert ts.shape[0] == k.shape[0]
        rc = _load().hta_oracle_probs_rt(_dp(q), _dp(k), _dp(p), int(q_start), int(kv_start), int(hist_len),
                                         int(rt_len), int(n_targets), _ip(ts), int(head), q.shape[1], k.shape[1],
                                         q.shape[2], float(scale), int(layer))
    if rc != 0:
        raise ValueError("hta_oracle_probs: invalid arguments")
    return p


def _ip_or_null(a):
    return _ip(a) if a is not None else None


def forward_pointwise(q, k, v, q_offsets, kv_offsets, hist_len, n_targets, scale, norm, layer, rt_len=None,
                      timestamps=None):
    """The pointwise reading of phi2: out_i = norm * sum over visible j of silu(scale <q_i, k_j>) v_j, float64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    qs, ks, hl, nt = _i32(q_offsets), _i32(kv_offsets), _i32(hist_len), _i32(n_targets)
    rl = _i32(rt_len) if rt_len is not None else None
    ts = _i32(timestamps) if timestamps is not None else None
    _check_shapes(q, k, v, qs, ks, hl, nt, layer, rl, ts)
    out = np.zeros_like(q)
    rc = _load().hta_oracle_pw_fwd_rt(_dp(q), _dp(k), _dp(v), _dp(out), _ip(qs), _ip(ks), _ip(hl), _ip_or_null(rl),
                                      _ip(nt), _ip_or_null(ts), hl.shape[0], q.shape[1], k.shape[1], q.shape[2],
                                      float(scale), float(norm), int(layer))
    if rc != 0:
        raise ValueError("hta_oracle_pw_fwd: invalid arguments")
    return out


def backward_pointwise(dout, q, k, v, q_offsets, kv_offsets, hist_len, n_targets, scale, norm, layer, rt_len=None,
                       timestamps=None):
    """Returns (dq, dk, dv) of forward_pointwise for the upstream gradient ``dout``, float64."""
    dout, q, k, v = _f64(dout), _f64(q), _f64(k), _f64(v)
    qs, ks, hl, nt = _i32(q_offsets), _i32(kv_offsets), _i32(hist_len), _i32(n_targets)
    rl = _i32(rt_len) if rt_len is not None else None
    ts = _i32(timestamps) if timestamps is not None else None
    _check_shapes(q, k, v, qs, ks, hl, nt, layer, rl, ts)
    assert dout.shape == q.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    rc = _load().hta_oracle_pw_bwd_rt(_dp(dout), _dp(q), _dp(k), _dp(v), _dp(dq), _dp(dk), _dp(dv), _ip(qs), _ip(ks),
                                      _ip(hl), _ip_or_null(rl), _ip(nt), _ip_or_null(ts), hl.shape[0], q.shape[1],
                                      k.shape[1], q.shape[2], float(scale), float(norm), int(layer))
    if rc != 0:
        raise ValueError("hta_oracle_pw_bwd: invalid arguments")
    return dq, dk, dv
