"""Guard bands around every buffer the library writes.

Each result tensor (out, lse, dq, dk, dv; y, mean, rstd, dx, du, dgamma, dbeta) and each workspace is carved out of a
larger allocation whose surroundings hold a byte pattern, and is itself pre-filled with NaN bit patterns.  After a
forward + backward call on batches with ragged edges -- users without history, without targets, without anything,
lengths one off the 32 / 64 / 128-key tile sizes, the last user of the batch ending the buffers -- the test checks on
the host that no byte of a guard band changed (no store past the end or in front of a buffer) and that no NaN pattern
is left in a result (every element was written).  The values themselves are the business of the parity tests."""
import numpy as np
import pytest
import torch

from paper_2602_11235_amd import gln, hta, hta_pw, inputs
from tests.hta_testlib import device_batch, to_torch

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET
GUARD, PATTERN = 8192, 0xA5


class Guarded:
    """`nbytes` of payload (256-byte aligned, filled with 0xFF: NaN as bf16 and as float32) between two guard bands."""

    def __init__(self, nbytes: int):
        self.n = int(nbytes)
        self.raw = torch.full((GUARD + self.n + (-self.n) % 256 + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        self.payload = self.raw[GUARD:GUARD + self.n]
        self.payload.fill_(0xFF)

    @classmethod
    def like(cls, t: torch.Tensor):
        g = cls(t.numel() * t.element_size())
        g.view = g.payload.view(t.dtype).view(t.shape)
        return g

    def intact(self) -> bool:
        return bool((self.raw[:GUARD] == PATTERN).all().item() and (self.raw[GUARD + self.n:] == PATTERN).all().item())


def settle(guards: dict, results: dict):
    torch.cuda.synchronize()
    for name, g in guards.items():
        assert g.intact(), f"{name}: a guard band around the buffer was overwritten"
    for name, g in results.items():
        assert not torch.isnan(g.view.float()).any().item(), f"{name}: elements left unwritten"


def guarded_batch(b, case, pointwise=False):
    """Swap every buffer the call writes for a guarded one; returns ({all guards}, {result guards})."""
    guards, results = {}, {}

    def put(name, tensor, is_result=True):
        g = Guarded.like(tensor)
        guards[name] = g
        if is_result:
            results[name] = g
        return g.view

    b.out = put("out", b.out)
    if not pointwise:
        b.lse = put("lse", b.lse)
    b.prepare_backward()
    b.dq, b.dk, b.dv = put("dq", b.dq), put("dk", b.dk), put("dv", b.dv)
    if pointwise:
        if b.fwd_ws is not None:
            b.fwd_ws = put("fwd workspace", b.fwd_ws, False)
        if b.bwd_ws is not None:
            b.bwd_ws = put("bwd workspace", b.bwd_ws, False)
    else:
        if b.fwd_workspace is not None:
            b.fwd_workspace = put("fwd workspace", b.fwd_workspace, False)
        if b.workspace is not None:
            b.workspace = put("bwd workspace", b.workspace, False)
    return guards, results


def run_attention(case, pointwise=False):
    dt = case.cfg.dtype
    if pointwise:
        from tests.test_gpu_parity_pointwise import device_batch as pw_batch, norm_of
        b = pw_batch(case, norm_of(case))
    else:
        b = device_batch(case)
    guards, results = guarded_batch(b, case, pointwise)
    b.forward()
    b.backward(to_torch(case.dout, dt))
    settle(guards, results)


EDGE_HIST = [0, 1, 63, 64, 65, 130, 200, 0, 257, 31, 0]
EDGE_TGTS = [3, 0, 70, 1, 33, 2, 64, 0, 129, 0, 0]
EDGE_RT = [5, 0, 3, 70, 31, 2, 140, 0, 33, 32, 64]


def case_of(layer, Hq, Hkv, d, dtype, rt=False, seed=91, hist=EDGE_HIST, tgts=EDGE_TGTS):
    std = 0.5 if dtype == "fp32" else 0.3
    return inputs.make_case(inputs.custom_config(f"guard_{Hq}_{Hkv}_{d}", layer, hist, tgts, Hq, Hkv, d, dtype=dtype,
                                                 std=std, seed=seed, rt_len=EDGE_RT[:len(hist)] if rt else None))


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("rt", [False, True])
@pytest.mark.parametrize("Hq,Hkv,d,dtype", [(8, 2, 64, "bf16"), (16, 2, 128, "bf16"), (4, 2, 32, "bf16"),
                                            (3, 1, 64, "bf16"), (16, 1, 64, "bf16"), (6, 2, 24, "fp32"),
                                            (4, 1, 16, "bf16")])
def test_attention_edge_batches_stay_inside_their_buffers(layer, rt, Hq, Hkv, d, dtype):
    run_attention(case_of(layer, Hq, Hkv, d, dtype, rt))


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("rt", [False, True])
def test_pointwise_edge_batches_stay_inside_their_buffers(layer, rt):
    run_attention(case_of(layer, 8, 2, 64, "bf16", rt), pointwise=True)
    run_attention(case_of(layer, 6, 2, 24, "fp32", rt), pointwise=True)


@pytest.mark.parametrize("layer", [TARGET, FULL])
@pytest.mark.parametrize("rt", [False, True])
def test_split_forward_stays_inside_its_buffers(layer, rt):
    # a handful of users: the forward pass splits the keys and keeps partial results in the workspace
    hist, tg = ([2048, 0, 1, 63, 128, 65, 1000, 64], [16, 5, 1, 33, 64, 2, 70, 0]) if layer == TARGET else \
               ([600, 63, 0], [16, 33, 5])
    c = case_of(layer, 8, 2, 64, "bf16", rt, hist=hist, tgts=tg)
    b = device_batch(c)
    assert b.fwd_workspace_bytes > 65536, "expected the split-key forward"
    guards, results = guarded_batch(b, c)
    b.forward()
    for name in ("dq", "dk", "dv"):
        results.pop(name)
    settle(guards, results)


def test_few_rows_long_histories_stay_inside_their_buffers():
    # enough (user, kv head) items of a target-only layer for the dK/dV launch that keeps a user's query rows in LDS
    hist, tgts = [600, 0, 513, 1030, 64, 257, 255, 256, 0] * 15, [128, 5, 0, 33, 70, 1, 96, 2, 0] * 15
    run_attention(case_of(TARGET, 8, 2, 64, "bf16", hist=hist, tgts=tgts))
    run_attention(case_of(TARGET, 16, 4, 64, "bf16", hist=hist, tgts=tgts))


def test_the_last_user_ends_exactly_at_the_end_of_the_buffers():
    # one user whose rows end a row tile / key tile early by one, and one that fills them exactly
    for hist, tgts in (([127], [1]), ([128], [64]), ([129], [63]), ([255, 1], [1, 0])):
        for layer in (FULL, TARGET):
            run_attention(case_of(layer, 8, 2, 64, "bf16", hist=hist, tgts=tgts))


@pytest.mark.parametrize("n,d,groups,dtype,gated", [(301, 512, 4, "bf16", True), (1, 8, 1, "bf16", False),
                                                    (777, 520, 3, "bf16", True), (1025, 2048, 4, "bf16", True),
                                                    (130, 72, 5, "fp32", True), (64, 1024, 8, "fp32", False)])
def test_gln_stays_inside_its_buffers(n, d, groups, dtype, gated):
    c = inputs.make_gln_case("guard_gln", n, d, groups, dtype=dtype, gated=gated, seed=92)
    dev = lambda a, dt=None: (torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(torch.bfloat16) if dt == "bf16"
                              else torch.from_numpy(np.ascontiguousarray(a)).to("cuda"))
    x, dy = dev(c.x, dtype), dev(c.dy, dtype)
    u = dev(c.gate, dtype) if gated else None
    gid, gamma, beta = dev(c.group_id), dev(c.gamma), dev(c.beta)
    guards, results = {}, {}

    def put(name, like, is_result=True):
        g = Guarded.like(like)
        guards[name] = g
        if is_result:
            results[name] = g
        return g.view

    f32n = torch.empty(n, dtype=torch.float32, device="cuda")
    y, mean, rstd = put("y", x), put("mean", f32n), put("rstd", f32n)
    gln.mtfm_gln_fwd(x, gid, gamma, beta, c.eps, gate=u, y=y, stats=(mean, rstd))
    ws = put("workspace", torch.empty(max(gln.mtfm_gln_bwd_workspace_bytes(d, groups), 256), dtype=torch.uint8,
                                      device="cuda"), False)
    out = (put("dx", x), put("dgamma", gamma), put("dbeta", gamma), put("du", x) if gated else None)
    gln.mtfm_gln_bwd(dy, x, gid, gamma, beta, mean, rstd, gate=u, workspace=ws, out=out)
    settle(guards, results)
