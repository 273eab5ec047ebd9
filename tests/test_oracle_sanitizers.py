"""The float64 oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

tests/oracle_sanitizer_driver.c compiles oracle/hta_oracle.c into a stand-alone program with
-fsanitize=address,undefined; every array it hands to the oracle is a heap block of exactly the right size, so an
index that runs past a jagged edge (a user without history, without targets, without anything; the last user of a
batch; the row slice of a target layer; real-time tokens) ends the program with a report.  Its results must be those
of the ordinary oracle library, which the pins of test_oracle_pins.py / _rt_pins / _pointwise_pins hold in place."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import hta_oracle as O
from paper_2602_11235_amd import inputs

HERE = os.path.dirname(os.path.abspath(__file__))
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("asan") / "oracle_sanitizer_driver")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           # runtimes linked into the program: a dynamically linked one refuses to start behind a preloaded library
           "-static-libasan", "-static-libubsan", "-o", exe, os.path.join(HERE, "oracle_sanitizer_driver.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


def run_driver(exe, case, tmp_path, norm=0.01):
    cfg = case.cfg
    has_rt = case.rt_len is not None
    src, dst = str(tmp_path / "case.bin"), str(tmp_path / "results.bin")
    with open(src, "wb") as f:
        f.write(struct.pack("=6i2q2d", cfg.layer, case.batch, cfg.Hq, cfg.Hkv, cfg.head_dim, int(has_rt), case.total_q,
                            case.total_kv, case.scale, norm))
        for a in (case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets):
            f.write(np.ascontiguousarray(a, dtype=np.int32).tobytes())
        if has_rt:
            f.write(np.ascontiguousarray(case.rt_len, dtype=np.int32).tobytes())
            f.write(np.ascontiguousarray(case.timestamps, dtype=np.int32).tobytes())
        for a in (case.q, case.k, case.v, case.dout):
            f.write(np.ascontiguousarray(a, dtype=np.float64).tobytes())
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    proc = subprocess.run([exe, src, dst], capture_output=True, text=True, env=env, timeout=600)
    assert proc.returncode == 0 and "ERROR" not in proc.stderr and "runtime error" not in proc.stderr, (
        f"sanitizer run failed (exit {proc.returncode}):\n{proc.stderr[-4000:]}")
    flat = np.fromfile(dst, dtype=np.float64)
    nq, nkv, nl = case.q.size, case.k.size, case.total_q * cfg.Hq
    sizes = [nq, nl, nq, nkv, nkv, nq, nq, nkv, nkv]
    parts, at = [], 0
    for n in sizes:
        parts.append(flat[at:at + n])
        at += n
    return parts, flat[at:]


def reference(case, norm=0.01):
    rt = dict(rt_len=case.rt_len, timestamps=case.timestamps)
    args = (case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets, case.scale)
    out, lse = O.forward(case.q, case.k, case.v, *args, case.cfg.layer, **rt)
    dq, dk, dv = O.backward(case.dout, case.q, case.k, case.v, out, lse, *args, case.cfg.layer, **rt)
    p_out = O.forward_pointwise(case.q, case.k, case.v, *args, norm, case.cfg.layer, **rt)
    p_dq, p_dk, p_dv = O.backward_pointwise(case.dout, case.q, case.k, case.v, *args, norm, case.cfg.layer, **rt)
    R = 0 if case.rt_len is None else int(case.rt_len[0])
    probs = O.probs(case.q, case.k, int(case.q_offsets[0]), int(case.kv_offsets[0]), int(case.hist_len[0]),
                    int(case.n_targets[0]), case.cfg.Hq - 1, case.scale, case.cfg.layer, rt_len=R,
                    timestamps=case.timestamps)
    return [out, lse, dq, dk, dv, p_out, p_dq, p_dk, p_dv], probs


CASES = {
    "c1": lambda: inputs.make_case(inputs.CONFIGS["C1"]),
    # users without history, without targets, without anything; the last user is empty, the first is not
    "edges_full": lambda: inputs.make_case(inputs.custom_config("e", FULL, [3, 0, 5, 0, 17, 1, 0], [2, 3, 0, 0, 9, 1, 0],
                                                                6, 2, 8, dtype="fp32", seed=31)),
    "edges_target": lambda: inputs.make_case(inputs.custom_config("e", TARGET, [3, 0, 5, 0, 17, 1, 0],
                                                                  [2, 3, 0, 0, 9, 1, 0], 6, 2, 8, dtype="fp32", seed=32)),
    "realtime_full": lambda: inputs.make_case(inputs.custom_config("e", FULL, [4, 0, 5, 0, 9], [2, 3, 0, 0, 4], 4, 1, 8,
                                                                   dtype="fp32", seed=33, rt_len=[3, 2, 0, 0, 6])),
    "realtime_target": lambda: inputs.make_case(inputs.custom_config("e", TARGET, [4, 0, 5, 0, 9], [2, 3, 0, 0, 4], 4, 4,
                                                                     8, dtype="fp32", seed=34, rt_len=[3, 2, 0, 5, 6])),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_oracle_is_clean_under_asan_and_ubsan(driver, tmp_path, name):
    case = CASES[name]()
    got, got_probs = run_driver(driver, case, tmp_path)
    ref, ref_probs = reference(case)
    for g, r in zip(got, ref):
        assert g.shape[0] == r.size
        np.testing.assert_allclose(g, r.reshape(-1), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got_probs, ref_probs.reshape(-1), rtol=1e-12, atol=1e-13)


def test_the_sanitized_build_does_catch_an_overrun(tmp_path):
    """The tool itself: a program of the same build flags that reads one element past a heap block must fail."""
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint main(int argc, char** argv) { double* p = malloc(8 * sizeof(double)); "
                   "p[0] = argc; double x = p[argc + 7]; free(p); return x > 1e300; }\n")
    exe = str(tmp_path / "overrun")
    subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    "-static-libubsan", "-o", exe, str(src)],
                   check=True, capture_output=True)
    proc = subprocess.run([exe], capture_output=True, text=True)
    assert proc.returncode != 0 and ("heap-buffer-overflow" in proc.stderr or "runtime error" in proc.stderr)
