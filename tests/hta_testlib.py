"""Helpers of the GPU parity tests: move a seeded case to the device, run the library through the
C-ABI binding, run the float64 oracle on the same bits, compare element by element."""
from __future__ import annotations

import sys

import numpy as np
import torch

from oracle import hta_oracle as O
from paper_2602_11235_amd import hta, inputs

# |gpu - ref| <= ATOL + RTOL * |ref|, per element
TOL = {"bf16": (2e-2, 2e-2), "fp32": (1e-4, 1e-4)}


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def to_torch(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t  # exact: values are bf16-representable


def device_batch(case: inputs.Case) -> hta.Batch:
    dt = case.cfg.dtype
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda")
    max_hist = int(case.hist_len.max()) if case.batch else 0
    max_tgt = int(case.n_targets.max()) if case.batch else 0
    rt = {}
    if case.rt_len is not None:   # samples with real-time tokens (mask rule 2)
        rt = dict(rt_len=dev(case.rt_len), timestamps=dev(case.timestamps),
                  max_rt=int(case.rt_len.max()) if case.batch else 0)
    return hta.Batch(to_torch(case.q, dt), to_torch(case.k, dt), to_torch(case.v, dt), dev(case.q_offsets),
                     dev(case.kv_offsets), dev(case.hist_len), dev(case.n_targets), max_hist, max_tgt, case.scale,
                     case.cfg.layer, **rt)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def oracle_all(case: inputs.Case, with_bwd: bool, per_head: bool = False):
    """The oracle's results for `case`.

    per_head: for users whose history is so long that one (user, kv head) unit of the oracle's backward pass -- it runs
    one thread per such unit -- would take minutes.  The oracle is then run on the equivalent multi-head problem, every
    query head with a copy of its kv head (grouped-query attention equals multi-head attention on consecutively
    repeated K/V: one of the oracle's pins), which gives it r times as many units to run side by side; out, lse and dq
    are the same, and dk/dv of a kv head are the sums of the per-head results over its r query heads."""
    layer = case.cfg.layer
    run = inputs.repeat_kv_heads(case) if per_head else case
    rt = dict(rt_len=run.rt_len, timestamps=run.timestamps)
    out, lse = O.forward(run.q, run.k, run.v, run.q_offsets, run.kv_offsets, run.hist_len, run.n_targets,
                         run.scale, layer, **rt)
    if not with_bwd:
        return out, lse
    # the backward is fed the *oracle's* forward results: the GPU backward is checked against the exact
    # gradient, not against a gradient contaminated by its own forward rounding
    dq, dk, dv = O.backward(run.dout, run.q, run.k, run.v, out, lse, run.q_offsets, run.kv_offsets,
                            run.hist_len, run.n_targets, run.scale, layer, **rt)
    if per_head:
        dk, dv = sum_over_group(dk, case.cfg.Hkv), sum_over_group(dv, case.cfg.Hkv)
    return out, lse, dq, dk, dv


def sum_over_group(per_head: np.ndarray, Hkv: int) -> np.ndarray:
    """[rows, Hq, d] per-query-head gradients of repeated K/V -> [rows, Hkv, d]: summed over each kv head's query heads."""
    rows, Hq, d = per_head.shape
    return per_head.reshape(rows, Hkv, Hq // Hkv, d).sum(axis=2)


def assert_close(name: str, got: np.ndarray, ref: np.ndarray, dtype: str) -> None:
    atol, rtol = TOL[dtype]
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    if got.size == 0:
        return
    assert np.isfinite(got).all(), f"{name}: non-finite values in GPU result"
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = int(np.argmax(err - bound))
    say(f"    {name}: max abs err {err.max():.3e}  max rel err {(err / (np.abs(ref) + 1e-30)).max():.3e}  "
        f"ref absmax {np.abs(ref).max():.3e}")
    # the element-wise bound is loose where |ref| << atol, so also require the worst error to be small
    # relative to the tensor's own scale
    assert err.max() <= rtol * np.abs(ref).max() + 1e-30, (
        f"{name}: max abs err {err.max():.3e} exceeds {rtol:g} x max|ref| = {rtol * np.abs(ref).max():.3e}")
    assert (err <= bound).all(), (f"{name}: {int((err > bound).sum())} of {err.size} elements out of tolerance; worst at "
                                  f"flat index {worst}: got {got.flat[worst]!r} ref {ref.flat[worst]!r}")


def run_library(case: inputs.Case, with_bwd: bool) -> dict:
    """One forward (+ backward) call of the library on the whole case; the results stay on the device."""
    dt = case.cfg.dtype
    batch = device_batch(case)
    out, lse = batch.forward()
    g = {"out": out, "lse": lse}
    if with_bwd:
        dq, dk, dv = batch.backward(to_torch(case.dout, dt))
        g.update(dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    return g


def compare_with_oracle(case: inputs.Case, g: dict, with_bwd: bool, users=None, kv_group=None, compare=None,
                        per_head: bool = False) -> None:
    """Compare device results `g` of the whole case with the oracle run on all users (users=None) or on exactly the
    listed ones (users are independent samples) and, if kv_group is given, on that kv head and its query heads only."""
    dt = case.cfg.dtype
    compare = compare or assert_close
    if users is None:
        ref_case, qrows, kvrows = case, None, None
    else:
        ref_case = inputs.take_users(case, users)
        qrows = torch.from_numpy(inputs.user_rows(case.q_offsets, users)).to("cuda")
        kvrows = torch.from_numpy(inputs.user_rows(case.kv_offsets, users)).to("cuda")
    hs, gs = slice(None), slice(None)
    if kv_group is not None:
        r = case.cfg.Hq // case.cfg.Hkv
        hs, gs = slice(kv_group * r, (kv_group + 1) * r), slice(kv_group, kv_group + 1)
        ref_case = inputs.take_kv_group(ref_case, kv_group)
    say(f"    oracle on {ref_case.batch} users, {ref_case.cfg.Hq} heads ...")
    ref = oracle_all(ref_case, with_bwd, per_head)

    def rows_of(t, rows, heads):   # [rows, heads, d] slice, taken on the device
        t = t if rows is None else t.index_select(0, rows)
        return host(t[:, heads])

    compare("out", rows_of(g["out"], qrows, hs), ref[0], dt)
    lse = g["lse"][hs]
    compare("lse", host(lse if qrows is None else lse.index_select(1, qrows)), ref[1], dt)
    if with_bwd:
        compare("dq", rows_of(g["dq"], qrows, hs), ref[2], dt)
        compare("dk", rows_of(g["dk"], kvrows, gs), ref[3], dt)
        compare("dv", rows_of(g["dv"], kvrows, gs), ref[4], dt)


def check_case(case: inputs.Case, with_bwd: bool, users=None, kv_group=None, compare=None) -> None:
    """Run the library on the whole case; compare all users (users=None) or the listed ones against the
    oracle run on exactly those users (and, if kv_group is given, only that kv head and its query heads)."""
    say(f"  case {case.cfg.name}: layer={case.cfg.layer} B={case.batch} total_q={case.total_q} total_kv={case.total_kv} "
        f"Hq={case.cfg.Hq} Hkv={case.cfg.Hkv} d={case.cfg.head_dim} dtype={case.cfg.dtype} bwd={with_bwd}")
    compare_with_oracle(case, run_library(case, with_bwd), with_bwd, users, kv_group, compare)


def close_on_tensor_scale(name: str, got: np.ndarray, ref: np.ndarray, dtype: str) -> None:
    """max |gpu - ref| <= rtol * max |ref| over the tensor: the bound for results whose elements are differences of
    terms much larger than themselves, where an element-wise relative bound cannot hold in 8-bit mantissas."""
    rtol = TOL[dtype][1]
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values in GPU result"
    err = np.abs(got - ref).max() if got.size else 0.0
    say(f"    {name}: max abs err {err:.3e}  ref absmax {np.abs(ref).max() if ref.size else 0.0:.3e}")
    assert err <= rtol * np.abs(ref).max() + 1e-30, f"{name}: max abs err {err:.3e} exceeds {rtol:g} x max|ref|"


def close_on_row_scale(name: str, got: np.ndarray, ref: np.ndarray, dtype: str) -> None:
    """|gpu - ref| <= atol + rtol * max |ref| over the features of the element's own (token, head) row, and the tensor-scale
    bound of assert_close.  For gradients that are sums of hundreds of terms of order one -- dk/dv of a key that a whole
    batch of candidates attends to with weight 1/2 or 1/3 (a user with two or three history tokens) -- the bf16
    rounding of the weights (2^-9 relative per term, the same weights for every feature of the row) leaves an
    absolute error proportional to the row's own scale, which an element that happens to be small does not shrink; a
    missing term still moves the row by more than rtol of its scale."""
    atol, rtol = TOL[dtype]
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    if got.size == 0:
        return
    assert np.isfinite(got).all(), f"{name}: non-finite values in GPU result"
    err = np.abs(got - ref)
    scale = np.abs(ref).max(axis=-1, keepdims=True) if ref.ndim == 3 else np.abs(ref)   # lse [Hq, rows]: per element
    bound = atol + rtol * scale
    say(f"    {name}: max abs err {err.max():.3e}  ref absmax {np.abs(ref).max():.3e}  worst err / bound {(err / bound).max():.3f}")
    assert err.max() <= rtol * np.abs(ref).max() + 1e-30, (
        f"{name}: max abs err {err.max():.3e} exceeds {rtol:g} x max|ref| = {rtol * np.abs(ref).max():.3e}")
    worst = int(np.argmax(err / bound))
    assert (err <= bound).all(), (f"{name}: {int((err > bound).sum())} of {err.size} elements out of tolerance; worst at "
                                  f"flat index {worst}: got {got.flat[worst]!r} ref {ref.flat[worst]!r}")


def pick_users(case: inputs.Case, n_random: int, seed: int = 0):
    """Extremes (shortest/longest history, fewest/most targets) plus `n_random` seeded random users."""
    picks = {int(np.argmin(case.hist_len)), int(np.argmax(case.hist_len)), int(np.argmin(case.n_targets)),
             int(np.argmax(case.n_targets))}
    u = inputs.uniform01(inputs.stream_key(seed, 99), 0, 4 * n_random)
    for x in u:
        if len(picks) >= 4 + n_random:
            break
        picks.add(int(x * case.batch) % case.batch)
    return sorted(picks)
