"""Host-side checks of the pointwise variant's C ABI that need no GPU."""
import os
import re

import pytest

from paper_2602_11235_amd import hta, hta_pw

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "mtfm_hta_pw.h")).read()
    names = sorted(set(re.findall(r"MTFM_HTA_API[^;(]*?\b(mtfm_hta_pw_\w+)\s*\(", text)))
    assert set(names) == set(hta_pw.EXPORTS) and len(names) == 6
    lib = hta_pw.load_library()
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_bytes_is_host_arithmetic():
    # a few users: the forward pass splits its keys exactly as the softmax variant does, same workspace
    assert (hta_pw.mtfm_hta_pw_workspace_bytes(hta.LAYER_FULL, hta.BF16, False, 4, 1000, 1000, 512, 64, 8, 2, 64) ==
            hta.mtfm_hta_workspace_bytes(hta.LAYER_FULL, hta.BF16, False, 4, 1000, 1000, 512, 64, 8, 2, 64))
    assert hta_pw.mtfm_hta_pw_workspace_bytes(hta.LAYER_FULL, hta.BF16, False, 300, 100000, 100000, 512, 64, 8, 2, 64) == 256 + 1280
    n = hta_pw.mtfm_hta_pw_workspace_bytes(hta.LAYER_FULL, hta.BF16, True, 4, 1000, 1000, 512, 64, 8, 2, 64)
    assert n >= 512 + 2 * 1000 * 8 * 4 and n % 256 == 0
    assert hta_pw.mtfm_hta_pw_workspace_bytes(hta.LAYER_FULL, hta.FP32, True, 4, 1000, 1000, 512, 64, 8, 2, 16) == 0
    with pytest.raises(hta.HtaError):
        hta_pw.mtfm_hta_pw_workspace_bytes(hta.LAYER_FULL, hta.BF16, True, 4, 1000, 1000, 512, 64, 8, 3, 64)


@pytest.mark.parametrize("kw, status", [
    (dict(scale=0.0), hta.ERR_INVALID_ARG), (dict(norm=0.0), hta.ERR_INVALID_ARG),
    (dict(norm=float("inf")), hta.ERR_INVALID_ARG), (dict(norm=float("nan")), hta.ERR_INVALID_ARG),
    (dict(d=48), hta.ERR_UNSUPPORTED), (dict(Hkv=3), hta.ERR_INVALID_ARG), (dict(q=None), hta.ERR_INVALID_ARG),
    (dict(ws_bytes=511), hta.ERR_WORKSPACE),
])
def test_forward_rejects_bad_arguments_without_launching(kw, status):
    lib = hta_pw.load_library()
    a = dict(q=FAKE, scale=0.125, norm=0.01, d=64, Hkv=2, ws_bytes=512)
    a.update(kw)
    rc = lib.mtfm_hta_pw_fwd(a["q"], FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 1000, 1000, 512, 64, 8, a["Hkv"],
                             a["d"], a["scale"], a["norm"], hta.BF16, hta.LAYER_FULL, FAKE * 16, a["ws_bytes"], None)
    assert rc == status and hta.mtfm_hta_last_error()


def test_backward_needs_neither_out_nor_lse_but_a_workspace():
    lib = hta_pw.load_library()
    rc = lib.mtfm_hta_pw_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 1000, 1000, 512, 64,
                             8, 2, 64, 0.125, 0.01, hta.BF16, hta.LAYER_FULL, None, 0, None)
    assert rc == hta.ERR_WORKSPACE
    assert lib.mtfm_hta_pw_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 0, 0, 0, 0, 8, 2, 64,
                               0.125, 0.01, hta.BF16, hta.LAYER_FULL, None, 0, None) == hta.OK
