"""Host-side checks of the group-layer-normalization C ABI that need no GPU: every declared symbol is exported and
bad scalar arguments are refused before anything touches a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2602_11235_amd import gln, hta

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a 16-byte aligned non-null address: refused calls never dereference it


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "mtfm_gln.h")).read()
    names = sorted(set(re.findall(r"MTFM_HTA_API[^;(]*?\b(mtfm_gln_\w+)\s*\(", text)))
    assert set(names) == set(gln.EXPORTS) and len(names) == 4
    lib = gln.load_library()
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_bytes_is_host_arithmetic():
    # one share of dgamma and dbeta for each of at most 512 workgroups
    assert gln.mtfm_gln_bwd_workspace_bytes(512, 8) == 512 * 2 * 8 * 512 * 4
    assert gln.mtfm_gln_bwd_workspace_bytes(64, 3) == 512 * 2 * 3 * 64 * 4
    assert gln.mtfm_gln_bwd_workspace_bytes(12, 3) == 0      # not a multiple of 8
    assert gln.mtfm_gln_bwd_workspace_bytes(4096, 1) == 0    # beyond 2048
    assert gln.mtfm_gln_bwd_workspace_bytes(512, 17) == 0    # 17 rows of 512 do not fit the LDS table
    assert gln.mtfm_gln_bwd_workspace_bytes(520, 8) == 512 * 2 * 8 * 520 * 4   # 8 rows padded to 1024: exactly the limit
    assert gln.mtfm_gln_bwd_workspace_bytes(520, 9) == 0


@pytest.mark.parametrize("kw, status", [
    (dict(d=12), hta.ERR_INVALID_ARG), (dict(d=0), hta.ERR_INVALID_ARG), (dict(groups=0), hta.ERR_INVALID_ARG),
    (dict(n=-1), hta.ERR_INVALID_ARG), (dict(dtype=7), hta.ERR_INVALID_ARG), (dict(eps=-1.0), hta.ERR_INVALID_ARG),
    (dict(eps=float("nan")), hta.ERR_INVALID_ARG), (dict(d=2056), hta.ERR_UNSUPPORTED),
    (dict(groups=17), hta.ERR_UNSUPPORTED), (dict(x=0), hta.ERR_INVALID_ARG), (dict(x=FAKE + 8), hta.ERR_INVALID_ARG),
])
def test_forward_rejects_bad_arguments_without_launching(kw, status):
    lib = gln.load_library()
    a = dict(x=FAKE, n=10, d=512, groups=8, eps=1e-5, dtype=hta.BF16)
    a.update(kw)
    rc = lib.mtfm_gln_fwd(a["x"], None, FAKE, FAKE, FAKE, FAKE, None, None, a["n"], a["d"], a["groups"], a["eps"],
                          a["dtype"], None)
    assert rc == status and hta.mtfm_hta_last_error()


def test_backward_rejects_bad_arguments_without_launching():
    lib = gln.load_library()
    need = gln.mtfm_gln_bwd_workspace_bytes(512, 8)

    def call(gate=None, dgate=None, beta=FAKE, ws=FAKE, ws_bytes=need, d=512):
        return lib.mtfm_gln_bwd(FAKE, FAKE, gate, FAKE, FAKE, beta, FAKE, FAKE, FAKE, dgate, FAKE, FAKE, 10, d, 8,
                                hta.BF16, ws, ws_bytes, None)

    assert call(ws=None) == hta.ERR_WORKSPACE and "workspace" in hta.mtfm_hta_last_error()
    assert call(ws_bytes=need - 1) == hta.ERR_WORKSPACE
    assert call(ws=FAKE + 16) == hta.ERR_WORKSPACE
    assert call(gate=FAKE) == hta.ERR_INVALID_ARG          # gate without dgate
    assert call(dgate=FAKE) == hta.ERR_INVALID_ARG
    assert call(gate=FAKE, dgate=FAKE, beta=None) == hta.ERR_INVALID_ARG
    assert call(d=12) == hta.ERR_INVALID_ARG


def test_empty_forward_is_ok_without_a_device():
    lib = gln.load_library()
    assert lib.mtfm_gln_fwd(FAKE, None, FAKE, FAKE, FAKE, FAKE, None, None, 0, 512, 8, 1e-5, hta.BF16, None) == hta.OK


def test_validate_host():
    lib = gln.load_library()
    ids = np.array([0, 2, 1, 2], dtype=np.int32)
    assert lib.mtfm_gln_validate_host(ids.ctypes.data, 4, 3) == hta.OK
    assert lib.mtfm_gln_validate_host(ids.ctypes.data, 4, 2) == hta.ERR_INVALID_ARG
    assert "token 1" in hta.mtfm_hta_last_error()
    ids[3] = -1
    assert lib.mtfm_gln_validate_host(ids.ctypes.data, 4, 3) == hta.ERR_INVALID_ARG
    assert lib.mtfm_gln_validate_host(None, 0, 3) == hta.OK
