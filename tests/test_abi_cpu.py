"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad scalar arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2602_11235_amd import hta

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    # the attention interface and the optional timing instrumentation (a header of its own)
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("mtfm_hta.h", "mtfm_hta_timing.h"))
    return sorted(set(re.findall(r"MTFM_HTA_API[^;(]*?\b(mtfm_hta_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hta.load_library()
    names = _declared_symbols()
    assert set(names) == set(hta.EXPORTS) and len(names) == 13
    for n in names:
        assert getattr(lib, n) is not None
    assert re.fullmatch(r"\d+\.\d+\.\d+", hta.mtfm_hta_version())


def test_workspace_bytes_is_host_arithmetic():
    # forward of a batch that fills the chip (300 users x 2 kv heads x row tiles): the work counters (256 bytes) and
    # the user order (300 users -> 1280 bytes)
    assert hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.BF16, False, 300, 100000, 100000, 512, 64, 8, 2, 64) == 256 + 1280
    assert hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.FP32, False, 4, 1000, 1000, 512, 64, 8, 2, 64) == 0
    # forward of a few users: 4 users x 2 kv heads x 9 row tiles of 64 = 72 items for 256 compute units, so the keys
    # are split (8 tiles of history, at least 4 per split -> 2 splits) and the partial results live in the workspace
    few = hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.BF16, False, 4, 1000, 1000, 512, 64, 8, 2, 64)
    assert few == 512 + 2 * 1000 * 8 * 64 * 4 + 2 * 1000 * 8 * 4
    # a history of fewer than eight tiles is not split
    assert hta.mtfm_hta_workspace_bytes(hta.LAYER_TARGET, hta.BF16, False, 1, 16, 400, 384, 16, 8, 2, 64) == 512
    n = hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.BF16, True, 4, 1000, 1000, 512, 64, 8, 2, 64)
    # backward: two float rows per (head, query row) on top of that, one of them with a sentinel element
    assert n >= 512 + 2 * 1000 * 8 * 4 and n % 256 == 0
    assert hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.FP32, True, 4, 1000, 1000, 512, 64, 8, 2, 16) == 0
    with pytest.raises(hta.HtaError):
        hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.BF16, True, 4, 1000, 1000, 512, 64, 8, 3, 64)


def test_workspace_of_16_wide_bf16_heads_holds_the_padded_copies():
    # a 16-wide head runs on the 32-wide kernels over zero-padded copies: the workspace is that of head_dim 32 plus
    # q, out (and dout, dq) of [total_q][Hq][32] bf16 and k, v (and dk, dv) of [total_kv][Hkv][32] bf16
    align = lambda n: (n + 255) // 256 * 256
    tq, tkv, Hq, Hkv = 1000, 900, 8, 2
    for layer in (hta.LAYER_FULL, hta.LAYER_TARGET):
        for is_bwd, copies in ((False, 2), (True, 4)):
            at32 = hta.mtfm_hta_workspace_bytes(layer, hta.BF16, is_bwd, 4, tq, tkv, 512, 64, Hq, Hkv, 32)
            at16 = hta.mtfm_hta_workspace_bytes(layer, hta.BF16, is_bwd, 4, tq, tkv, 512, 64, Hq, Hkv, 16)
            assert at16 == at32 + copies * (align(tq * Hq * 64) + align(tkv * Hkv * 64))


@pytest.mark.parametrize("kwargs,status", [
    (dict(Hq=8, Hkv=3), hta.ERR_INVALID_ARG),
    (dict(head_dim=48), hta.ERR_UNSUPPORTED),
    (dict(head_dim=0), hta.ERR_INVALID_ARG),
    (dict(layer=7), hta.ERR_INVALID_ARG),
    (dict(dtype=9), hta.ERR_INVALID_ARG),
    (dict(batch=-1), hta.ERR_INVALID_ARG),
    (dict(scale=0.0), hta.ERR_INVALID_ARG),
    (dict(scale=float("nan")), hta.ERR_INVALID_ARG),
    (dict(q=0), hta.ERR_INVALID_ARG),
    (dict(q=4104), hta.ERR_INVALID_ARG),
    (dict(dtype=hta.FP32, head_dim=256), hta.ERR_UNSUPPORTED),
])
def test_forward_rejects_bad_scalars_without_launching(kwargs, status):
    a = dict(q=4096, k=4096, v=4096, out=4096, lse=4096, qo=4096, kvo=4096, hl=4096, nt=4096, batch=2, total_q=10,
             total_kv=10, max_hist=4, max_targets=1, Hq=8, Hkv=2, head_dim=64, scale=0.125, dtype=hta.BF16,
             layer=hta.LAYER_FULL)
    a.update(kwargs)
    lib = hta.load_library()
    rc = lib.mtfm_hta_fwd(a["q"], a["k"], a["v"], a["out"], a["lse"], a["qo"], a["kvo"], a["hl"], a["nt"], a["batch"],
                          a["total_q"], a["total_kv"], a["max_hist"], a["max_targets"], a["Hq"], a["Hkv"], a["head_dim"],
                          a["scale"], a["dtype"], a["layer"], None, 0, None)
    assert rc == status
    assert len(hta.mtfm_hta_last_error()) > 0


def test_backward_reports_missing_workspace():
    lib = hta.load_library()
    rc = lib.mtfm_hta_bwd(*([4096] * 13), 2, 10, 10, 4, 1, 8, 2, 64, 0.125, hta.BF16, hta.LAYER_FULL, None, 0, None)
    assert rc == hta.ERR_WORKSPACE and "workspace" in hta.mtfm_hta_last_error()


def test_backward_without_query_rows_takes_null_row_tensors():
    # a target layer whose users have no candidate: total_q = 0, the row-shaped tensors are empty.  The call gets past
    # its pointer checks (it stops at the missing workspace here); with a key/value tensor missing it does not.
    lib = hta.load_library()
    row, kv, idx = [None] * 2, [4096] * 2, [4096] * 4
    rc = lib.mtfm_hta_bwd(None, None, *kv, None, None, None, *kv, *idx, 2, 0, 10, 8, 0, 8, 2, 64, 0.125, hta.BF16,
                          hta.LAYER_TARGET, None, 0, None)
    assert rc == hta.ERR_WORKSPACE, hta.mtfm_hta_last_error()
    rc = lib.mtfm_hta_bwd(None, None, None, 4096, None, None, None, *kv, *idx, 2, 0, 10, 8, 0, 8, 2, 64, 0.125, hta.BF16,
                          hta.LAYER_TARGET, None, 0, None)
    assert rc == hta.ERR_INVALID_ARG and "null" in hta.mtfm_hta_last_error()
    rc = lib.mtfm_hta_bwd(None, None, *kv, None, None, None, *kv, *idx, 2, 5, 10, 8, 5, 8, 2, 64, 0.125, hta.BF16,
                          hta.LAYER_TARGET, None, 0, None)
    assert rc == hta.ERR_INVALID_ARG and "null" in hta.mtfm_hta_last_error()


def test_per_file_compiler_options_name_existing_sources():
    from paper_2602_11235_amd import build
    names = {os.path.basename(s) for s in build.sources()}
    assert set(build.FILE_FLAGS) <= names, set(build.FILE_FLAGS) - names


def test_empty_batch_is_ok_without_a_device():
    lib = hta.load_library()
    assert lib.mtfm_hta_fwd(None, None, None, None, None, None, None, None, None, 0, 0, 0, 0, 0, 8, 2, 64, 0.125,
                            hta.BF16, hta.LAYER_FULL, None, 0, None) == hta.OK


def test_validate_host():
    def call(qo, kvo, hl, nt, layer, max_hist=100, max_targets=100):
        arrs = [np.asarray(x, dtype=np.int32) for x in (qo, kvo, hl, nt)]
        lib = hta.load_library()
        return lib.mtfm_hta_validate_host(*[x.ctypes.data for x in arrs], len(hl), int(arrs[0][-1]), int(arrs[1][-1]),
                                          max_hist, max_targets, layer)
    assert call([0, 7, 10], [0, 7, 10], [5, 0], [2, 3], hta.LAYER_FULL) == hta.OK
    assert call([0, 2, 5], [0, 7, 10], [5, 0], [2, 3], hta.LAYER_TARGET) == hta.OK
    assert call([0, 7, 10], [0, 7, 10], [5, 0], [2, 3], hta.LAYER_TARGET) == hta.ERR_INVALID_ARG
    assert call([0, 7, 10], [0, 7, 10], [5, 1], [2, 3], hta.LAYER_FULL) == hta.ERR_INVALID_ARG
    assert call([0, 7, 10], [0, 7, 10], [5, 0], [2, 3], hta.LAYER_FULL, max_hist=4) == hta.ERR_INVALID_ARG
    assert "max_hist" in hta.mtfm_hta_last_error()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_11235_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f"{f} imports the oracle"
                assert "hta_oracle" not in text and "libhta_oracle" not in text, f"{f} refers to the oracle library"
