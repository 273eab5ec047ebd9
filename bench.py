#!/usr/bin/env python3
"""Benchmark of the Hybrid Target Attention hot path on one MI355X.

A step is one forward + one backward pass of the whole jagged batch through the C-ABI library
(inputs resident in HBM).  Prints ONE JSON line: whole-job TFLOP/s (algorithmic FLOPs of the visible
pairs only: 4*d per pair forward, 10*d backward including the recomputation of S), samples/s, the
roofline of the dominant kernel from HIP events recorded around it inside the timed region, and the
float64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


# ----------------------------------------------------------------------------- algorithmic work (FLOP credit)
# Counting only: which (query, key) pairs the mask leaves visible.  Kept here (and out of the input generators) because
# it restates the mask rules; the tests pin it to hand-counted totals.
def visible_pairs(hist_len: np.ndarray, n_targets: np.ndarray, Hq: int, layer: int) -> int:
    """Number of (query, key) pairs the hybrid mask leaves visible, summed over heads: per user
    L^2 + T*L + T for a full layer and T*L + T for a target layer (the N^2 vs N*L_T terms of the
    complexity statement in Section 3.2.2)."""
    L = hist_len.astype(np.int64)
    T = n_targets.astype(np.int64)
    per = T * L + T
    if layer == 0:
        per = per + L * L
    return int(Hq * per.sum())


def visible_pairs_of(case) -> int:
    """visible_pairs for a batch that may carry real-time tokens: under rule 2 a real-time key is visible to the
    queries with a strictly later timestamp and to its own token."""
    cfg = case.cfg
    if case.rt_len is None:
        return visible_pairs(case.hist_len, case.n_targets, cfg.Hq, cfg.layer)
    total = 0
    for b in range(case.batch):
        L, R, T = int(case.hist_len[b]), int(case.rt_len[b]), int(case.n_targets[b])
        ts = case.timestamps[case.kv_offsets[b]:case.kv_offsets[b + 1]].astype(np.int64)
        first = 0 if cfg.layer == 0 else L + R
        rows_ts = ts[first:]
        total += rows_ts.shape[0] * L                                               # rule 1
        total += int(np.searchsorted(ts[L:L + R], rows_ts, side="left").sum())       # rule 2: strictly earlier keys
        total += (R if cfg.layer == 0 else 0) + T                           # own keys
    return int(cfg.Hq * total)


def history_pairs(case, inputs) -> int:
    """Visible (query, key, head) triples whose key is not the query's own target key: what the dK/dV pass owns."""
    if case.rt_len is not None:
        own = case.n_targets.astype(np.int64).sum() * case.cfg.Hq
        return visible_pairs_of(case) - int(own)
    L = case.hist_len.astype(np.int64)
    T = case.n_targets.astype(np.int64)
    rows = L + T if case.cfg.layer == 0 else T
    return int(case.cfg.Hq * (rows * L).sum())


def cpu_baseline(case, inputs, budget_s: float, pointwise: bool = False):
    """Time the float64 oracle (forward + backward) on the first users of the batch: a probe on 2 users
    sizes the sample so that the run takes about `budget_s` seconds."""
    from oracle import hta_oracle as O

    def run(users):
        sub = inputs.take_users(case, users)
        t0 = time.perf_counter()
        rt = dict(rt_len=sub.rt_len, timestamps=sub.timestamps)
        if pointwise:
            O.forward_pointwise(sub.q, sub.k, sub.v, sub.q_offsets, sub.kv_offsets, sub.hist_len, sub.n_targets,
                                sub.scale, 1e-3, sub.cfg.layer, **rt)
            O.backward_pointwise(sub.dout, sub.q, sub.k, sub.v, sub.q_offsets, sub.kv_offsets, sub.hist_len,
                                 sub.n_targets, sub.scale, 1e-3, sub.cfg.layer, **rt)
        else:
            out, lse = O.forward(sub.q, sub.k, sub.v, sub.q_offsets, sub.kv_offsets, sub.hist_len, sub.n_targets,
                                 sub.scale, sub.cfg.layer, **rt)
            O.backward(sub.dout, sub.q, sub.k, sub.v, out, lse, sub.q_offsets, sub.kv_offsets, sub.hist_len,
                       sub.n_targets, sub.scale, sub.cfg.layer, **rt)
        dt = time.perf_counter() - t0
        pairs = visible_pairs_of(sub)
        return dt, pairs, sub.batch

    O.num_threads()  # loads (and if needed builds) the oracle before timing
    probe_dt, probe_pairs, _ = run(range(min(2, case.batch)))
    per_pair = probe_dt / max(probe_pairs, 1)
    L = case.hist_len.astype(np.int64) + (0 if case.rt_len is None else case.rt_len.astype(np.int64))
    T = case.n_targets.astype(np.int64)
    per_user = case.cfg.Hq * ((L + T) * L + T if case.cfg.layer == 0 else T * L + T)  # upper bound with real-time tokens
    n = int(np.searchsorted(np.cumsum(per_user * per_pair), budget_s)) + 1
    n = max(2, min(n, case.batch))
    dt, pairs, users = run(range(n))
    d = case.cfg.head_dim
    return {
        "value": 14.0 * d * pairs / dt / 1e12, "unit": "TFLOP/s", "cores": O.num_threads(), "kind": "oracle",
        "sample": f"float64 oracle fwd+bwd on the first {users} of {case.batch} users of {case.cfg.name} "
                  f"({pairs} visible pairs, {dt:.2f} s)",
        "samples_per_s": users / dt, "seconds": dt,
    }


def recorded_traffic(workload: str, kernel: str, family: str = "hta_fwd_bwd"):
    """HBM bytes per launch of `kernel` on `workload`, as recorded by the committed rocprofv3 counter summary
    (FETCH_SIZE / WRITE_SIZE cannot be read from inside this process); None when there is no record."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"{workload.lower()}_{family}_kernels.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and parts[0] == "TRAFFIC" and parts[1] == kernel:
                    kv = dict(x.split("=") for x in parts[2:])
                    return {"read_bytes": int(kv["read_bytes"]), "write_bytes": int(kv["write_bytes"]),
                            "source": os.path.relpath(path, os.path.dirname(os.path.abspath(__file__)))}
    except (OSError, ValueError, KeyError):
        pass
    return None


def calibration_copy(torch, mib: int) -> None:
    """One plain device copy of `mib` MiB (known HBM traffic) for scaling the counters of a rocprofv3 --pmc run."""
    if mib <= 0:
        return
    src = torch.ones(mib << 20, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)  # reads and writes exactly `mib` MiB
    torch.cuda.synchronize()
    del src, dst


def bench_gln(args) -> int:
    """--op gln: one step = the gated fused group layer normalization, forward + backward, over all tokens of the
    headline batch at the model width of its heads (d_model = Hq * head_dim).  HBM-bound: the line reports GB/s of
    algorithmic bytes (each operand read once, each result written once) against the 8 TB/s peak."""
    import torch
    from paper_2602_11235_amd import gln, hta, inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    gln.load_library()
    cfg = inputs.CONFIGS[args.config]
    lens = inputs.make_case(dataclasses.replace(cfg, Hq=1, Hkv=1, head_dim=8, dtype="fp32"))  # token count only
    n, d, groups = int(lens.total_kv), cfg.Hq * cfg.head_dim, args.groups
    t0 = time.perf_counter()
    case = inputs.make_gln_case(f"{cfg.name}_gln", n, d, groups, dtype="bf16", gated=True, seed=cfg.seed)
    log(f"[bench] generated {n} tokens x {d} features, {groups} groups in {time.perf_counter() - t0:.1f} s")

    def dev(a, bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
        return t.to(torch.bfloat16) if bf16 else t

    x, u, dy = dev(case.x, True), dev(case.gate, True), dev(case.dy, True)
    gid, gamma, beta = dev(case.group_id), dev(case.gamma), dev(case.beta)
    y = torch.empty_like(x)
    out = (torch.empty_like(x), torch.empty_like(gamma), torch.empty_like(gamma), torch.empty_like(x))
    ws = torch.empty(gln.mtfm_gln_bwd_workspace_bytes(d, groups), dtype=torch.uint8, device="cuda:0")
    stats = {}

    def step():
        _, stats["mean"], stats["rstd"] = gln.mtfm_gln_fwd(x, gid, gamma, beta, case.eps, gate=u, y=y)
        gln.mtfm_gln_bwd(dy, x, gid, gamma, beta, stats["mean"], stats["rstd"], gate=u, workspace=ws, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    calibration_copy(torch, args.calibration_copy_mib)
    hta.mtfm_hta_timing_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kinds = {"gln_fwd": gln.KERNEL_FWD, "gln_bwd": gln.KERNEL_BWD, "gln_bwd_reduce": gln.KERNEL_BWD_REDUCE}
    kernel_ms = {k: hta.mtfm_hta_timing_read(v) for k, v in kinds.items()}
    hta.mtfm_hta_timing_enable(0)

    # algorithmic bytes per token: forward reads x, u and writes y (2 bytes each per feature), reads the group id
    # and writes two statistics; backward reads dy, x, u, writes dx, du, reads the id and the statistics
    bytes_fwd, bytes_bwd = n * (6 * d + 12), n * (10 * d + 12)
    alg = {"gln_fwd": bytes_fwd, "gln_bwd": bytes_bwd}
    ms_per_step = elapsed / args.steps * 1e3
    kernels = {}
    for name, ms in kernel_ms.items():
        if ms:
            kernels[name] = {"avg_ms": float(np.mean(ms)), "min_ms": float(np.min(ms)), "launches": len(ms)}
            if name in alg:
                kernels[name]["gb_per_s"] = alg[name] / (kernels[name]["avg_ms"] * 1e-3) / 1e9
                kernels[name]["frac_of_hbm_peak"] = kernels[name]["gb_per_s"] / HBM_PEAK_GBS
    dominant = max(alg, key=lambda k: kernels[k]["avg_ms"])
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": kernels[dominant]["gb_per_s"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[dominant]["gb_per_s"] / HBM_PEAK_GBS, "traffic": None,
                "avg_kernel_ms": kernels[dominant]["avg_ms"], "algorithmic_bytes_per_launch": alg[dominant]}
    measured = recorded_traffic(cfg.name, dominant, "gln")
    if measured is not None:
        roofline["traffic"] = measured["read_bytes"] + measured["write_bytes"]
        roofline["traffic_note"] = (f"HBM bytes per launch (read {measured['read_bytes']}, written "
                                    f"{measured['write_bytes']}) from the rocprofv3 counter runs recorded in "
                                    f"{measured['source']}; not measured by this run")
    value = (bytes_fwd + bytes_bwd) / (ms_per_step * 1e-3) / 1e9
    result = {
        "metric": "fused GLN(A)*U fwd+bwd GB/s of algorithmic bytes over the tokens of the headline batch; % of HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}_gln: {n} tokens (all tokens of {cfg.name}) d_model={d} n_groups={groups} "
                               "bf16 storage, gated, fwd+bwd", "seed": cfg.seed},
        "tokens_per_s": n / (ms_per_step * 1e-3), "frac_of_hbm_peak": value / HBM_PEAK_GBS,
        "kernels": kernels, "roofline": roofline,
    }
    if args.cpu_seconds > 0:
        from oracle import gln_oracle as G
        log("[bench] timing the float64 oracle on a bounded sample ...")
        m = min(n, 2000)
        t0 = time.perf_counter()
        G.forward(case.x[:m], case.group_id[:m], case.gamma, case.beta, case.eps, case.gate[:m])
        G.backward(case.dy[:m], case.x[:m], case.group_id[:m], case.gamma, case.beta, case.eps, case.gate[:m])
        per_tok = (time.perf_counter() - t0) / m
        m = int(max(m, min(n, args.cpu_seconds / per_tok)))
        t0 = time.perf_counter()
        G.forward(case.x[:m], case.group_id[:m], case.gamma, case.beta, case.eps, case.gate[:m])
        G.backward(case.dy[:m], case.x[:m], case.group_id[:m], case.gamma, case.beta, case.eps, case.gate[:m])
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": m * (16 * d + 24) / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"float64 NumPy oracle fwd+bwd on the first {m} of {n} tokens ({dt:.2f} s)",
                                  "tokens_per_s": m / dt, "seconds": dt}
    print(json.dumps(result), flush=True)
    return 0


def bench_infer(args) -> int:
    """--op infer: one step = one forward call of the target layer over a handful of requests (inference shape:
    request-level aggregation, forward only).  The batch is far too small to fill the chip with (user, kv head) groups,
    so the library splits the keys of each group over workgroups; the figure of merit is the latency of a call."""
    import torch
    from paper_2602_11235_amd import hta, inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    hta.load_library()
    cfg = inputs.CONFIGS[args.config if args.config.startswith("I") else "I2"]
    case = inputs.make_case(cfg)

    def dev(x):
        t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
        return t.to(torch.bfloat16) if cfg.dtype == "bf16" and t.dtype == torch.float32 else t

    rt = {}
    if case.rt_len is not None:
        rt = dict(rt_len=dev(case.rt_len), timestamps=dev(case.timestamps), max_rt=int(case.rt_len.max()))
    batch = hta.Batch(dev(case.q), dev(case.k), dev(case.v), dev(case.q_offsets), dev(case.kv_offsets),
                      dev(case.hist_len), dev(case.n_targets), int(case.hist_len.max()), int(case.n_targets.max()),
                      case.scale, cfg.layer, **rt)
    for _ in range(args.warmup):
        batch.forward()
    torch.cuda.synchronize()
    calibration_copy(torch, args.calibration_copy_mib)
    # latency of a single call: enqueue, then wait for the result
    lat = []
    for _ in range(args.steps):
        t0 = time.perf_counter()
        batch.forward()
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t0)
    # the same call replayed from a HIP graph (the library only enqueues kernels, so a caller can capture it)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        batch.forward()
    torch.cuda.synchronize()
    glat = []
    for _ in range(args.steps):
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        glat.append(time.perf_counter() - t0)
    # back-to-back calls (the stream never drains): the timed region of the JSON line
    hta.mtfm_hta_timing_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        batch.forward()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = hta.mtfm_hta_timing_read(hta.KERNEL_FWD)
    hta.mtfm_hta_timing_enable(0)

    d = cfg.head_dim
    pairs = visible_pairs_of(case)
    ms_per_step = elapsed / args.steps * 1e3
    avg = float(np.mean(ms))
    flops = 4.0 * d * pairs
    tflops = flops / (avg * 1e-3) / 1e12
    # operands a call has to read at least once: Q rows, K and V rows, and the output it writes
    io_bytes = 2 * (2 * case.total_q * cfg.Hq * d + 2 * case.total_kv * cfg.Hkv * d)
    result = {
        "metric": "HTA target-layer forward at inference shape (few requests): requests/s, latency per call",
        "value": case.batch / (ms_per_step * 1e-3), "unit": "requests/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.batch} hist={cfg.hist}{'' if cfg.rt is None else f' realtime={cfg.rt}'} targets={cfg.targets} "
                               f"Hq={cfg.Hq} Hkv={cfg.Hkv} head_dim={d} layer=target fwd only",
                   "seed": cfg.seed, "visible_pairs": pairs, "total_tokens": case.total_kv},
        "latency_us": {"median": float(np.median(lat) * 1e6), "min": float(np.min(lat) * 1e6),
                       "note": "host enqueue + device + synchronize, one call at a time",
                       "graph_replay_median": float(np.median(glat) * 1e6), "graph_replay_min": float(np.min(glat) * 1e6)},
        "candidates_per_s": int(case.n_targets.sum()) / (ms_per_step * 1e-3),
        "kernels": {"fwd": {"avg_ms": avg, "min_ms": float(np.min(ms)), "launches": len(ms), "tflops": tflops,
                            "note": "split-key forward kernel + merge kernel (one event pair around both)"}},
        "roofline": {"bound": "mfma", "kernel": "fwd", "achieved": tflops, "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / BF16_MFMA_PEAK_TFLOPS, "traffic": None,
                     "avg_kernel_ms": avg, "algorithmic_flops_per_launch": flops,
                     "note": f"latency-bound: a call has {flops / 1e9:.2f} GFLOP and {io_bytes / 1e6:.1f} MB of operands, "
                             "microseconds of work for the whole chip; what is measured is the critical path of one call"},
    }
    if args.cpu_seconds > 0:
        log("[bench] timing the float64 oracle on a bounded sample ...")
        from oracle import hta_oracle as O
        O.num_threads()
        users = list(range(min(case.batch, 2)))
        sub = inputs.take_users(case, users)
        t0 = time.perf_counter()
        O.forward(sub.q, sub.k, sub.v, sub.q_offsets, sub.kv_offsets, sub.hist_len, sub.n_targets, sub.scale,
                  sub.cfg.layer, rt_len=sub.rt_len, timestamps=sub.timestamps)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": len(users) / dt, "unit": "requests/s", "cores": O.num_threads(),
                                  "kind": "oracle", "seconds": dt,
                                  "sample": f"float64 oracle forward on the first {len(users)} of {case.batch} requests of {cfg.name}"}
    print(json.dumps(result), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--op", default="hta", choices=["hta", "pointwise", "gln", "infer"],
                    help="hta: the attention hot path (the headline metric); pointwise: the same path with the "
                         "pointwise (SiLU) reading of phi2; gln: the fused group layer normalization; "
                         "infer: forward-only target layer on a few requests (--config I1 | I2 | I3 | I2_RT)")
    ap.add_argument("--groups", type=int, default=8, help="--op gln: number of normalization groups")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C3", help="workload name in paper_2602_11235_amd.inputs.CONFIGS")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU time budget of the oracle baseline (0: skip)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the timed region (known HBM "
                         "traffic, to scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus {args.gpus} is not "
              "supported. Users are independent samples, so a multi-GPU run would be data parallel with no exchange.",
              file=sys.stderr)
        return 2
    if args.op == "gln":
        return bench_gln(args)
    if args.op == "infer":
        return bench_infer(args)

    import torch
    from paper_2602_11235_amd import hta, hta_pw, inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    hta.load_library()  # fail loudly if the HIP library is missing
    pointwise = args.op == "pointwise"

    cfg = inputs.CONFIGS[args.config]
    t0 = time.perf_counter()
    case = inputs.make_case(cfg)
    log(f"[bench] generated {cfg.name}: B={case.batch} total_q={case.total_q} total_kv={case.total_kv} "
        f"in {time.perf_counter() - t0:.1f} s")

    def dev(x):
        t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
        return t.to(torch.bfloat16) if cfg.dtype == "bf16" and t.dtype == torch.float32 else t

    rt = {}
    if case.rt_len is not None:  # samples with real-time tokens: the *_rt entry points
        rt = dict(rt_len=dev(case.rt_len), timestamps=dev(case.timestamps), max_rt=int(case.rt_len.max()))
    if pointwise:  # weights norm * silu(scale s); norm = 1 / longest sample, as HSTU divides by the sequence length
        longest = case.hist_len + case.n_targets + (0 if case.rt_len is None else case.rt_len)
        batch = hta_pw.PointwiseBatch(dev(case.q), dev(case.k), dev(case.v), dev(case.q_offsets), dev(case.kv_offsets),
                                      dev(case.hist_len), dev(case.n_targets), int(case.hist_len.max()),
                                      int(case.n_targets.max()), case.scale, 1.0 / float(longest.max()), cfg.layer, **rt)
    else:
        batch = hta.Batch(dev(case.q), dev(case.k), dev(case.v), dev(case.q_offsets), dev(case.kv_offsets),
                          dev(case.hist_len), dev(case.n_targets), int(case.hist_len.max()), int(case.n_targets.max()),
                          case.scale, cfg.layer, **rt)
    dout = dev(case.dout)
    batch.prepare_backward()
    torch.cuda.synchronize()

    def step():
        batch.forward()
        batch.backward(dout)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    calibration_copy(torch, args.calibration_copy_mib)
    hta.mtfm_hta_timing_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kinds = {"fwd": hta.KERNEL_FWD, "bwd_self": hta.KERNEL_BWD_SELF, "bwd_dq": hta.KERNEL_BWD_DQ,
             "bwd_dkdv": hta.KERNEL_BWD_DKDV}
    kernel_ms = {name: hta.mtfm_hta_timing_read(kind) for name, kind in kinds.items()}
    hta.mtfm_hta_timing_enable(0)

    d = cfg.head_dim
    pairs = visible_pairs_of(case)
    hist_pairs = history_pairs(case, inputs)
    ms_per_step = elapsed / args.steps * 1e3
    flops_step = 14.0 * d * pairs
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # Algorithmic FLOPs per launch (what the method needs, not what the kernel executes): forward 4*d per
    # visible pair; backward 10*d per pair, split between the two passes by the products they own -- dQ
    # (S, dP, dQ = 6*d, of which S and dP are shared work credited once) and dK/dV (dV, dK = 4*d).
    flops = {"fwd": 4.0 * d * pairs, "bwd_dq": 6.0 * d * pairs, "bwd_dkdv": 4.0 * d * hist_pairs}
    kernels = {}
    for name, ms in kernel_ms.items():
        if not ms:
            continue
        avg = float(np.mean(ms))
        kernels[name] = {"avg_ms": avg, "min_ms": float(np.min(ms)), "launches": len(ms)}
        if name in flops:
            kernels[name]["tflops"] = flops[name] / (avg * 1e-3) / 1e12
            kernels[name]["frac_of_bf16_mfma_peak"] = kernels[name]["tflops"] / BF16_MFMA_PEAK_TFLOPS
    dominant = max(kernels, key=lambda n: kernels[n]["avg_ms"]) if kernels else None
    roofline = None
    if dominant in flops:
        ach = kernels[dominant]["tflops"]
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": ach, "peak": BF16_MFMA_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / BF16_MFMA_PEAK_TFLOPS, "traffic": None,
                    "avg_kernel_ms": kernels[dominant]["avg_ms"],
                    "algorithmic_flops_per_launch": flops[dominant]}
        measured = None if pointwise else recorded_traffic(cfg.name, dominant)
        if measured is not None:
            roofline["traffic"] = measured["read_bytes"] + measured["write_bytes"]
            roofline["traffic_note"] = (f"HBM bytes per launch (read {measured['read_bytes']}, written "
                                        f"{measured['write_bytes']}) from the rocprofv3 counter runs recorded in "
                                        f"{measured['source']}; not measured by this run")

    result = {
        "metric": ("HTA fwd+bwd TFLOP/s & samples/s at B=256,L=1024,T=64; % of bf16 MFMA peak" if not pointwise else
                   "HTA with pointwise (SiLU) weights, fwd+bwd TFLOP/s & samples/s; % of bf16 MFMA peak"),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.batch} hist={cfg.hist}{'' if cfg.rt is None else f' realtime={cfg.rt}'} targets={cfg.targets} Hq={cfg.Hq} "
                               f"Hkv={cfg.Hkv} head_dim={d} layer={'full' if cfg.layer == 0 else 'target'} fwd+bwd",
                   "seed": cfg.seed, "visible_pairs": pairs, "total_tokens": case.total_kv},
        "samples_per_s": case.batch / (ms_per_step * 1e-3),
        "frac_of_bf16_mfma_peak": value / BF16_MFMA_PEAK_TFLOPS,
        "tflops_no_recompute_credit": 12.0 * d * pairs / (ms_per_step * 1e-3) / 1e12,
        "kernels": kernels, "roofline": roofline,
        "cache_note": "no flush between steps: the step's working set (>1 GB) exceeds L2 + the 256 MB memory-side cache",
    }
    if args.cpu_seconds > 0:
        log("[bench] timing the float64 oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(case, inputs, args.cpu_seconds, pointwise)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
