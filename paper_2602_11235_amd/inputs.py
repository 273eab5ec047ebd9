"""Seeded synthetic inputs for Hybrid Target Attention (HTA).

This module only *draws* data: jagged lengths and q/k/v/dout values.  It holds none of the
attention arithmetic, so both the CPU oracle's tests and the HIP path's tests can consume the
very same bits from it.

Workload structure (Section 3.2.1, token order X = (H; R; T)): every aggregated user sample is
one history segment of ``L_b`` tokens followed by ``T_b`` target tokens; lengths vary per user,
so a batch is packed ("jagged") with prefix-sum offsets instead of padding.

Random numbers come from a counter-based generator (the splitmix64 sequence, one independent
stream per tensor) followed by a Box-Muller transform in float64, so the values depend only on
(seed, stream, index) and not on any library's generator.
"""
from __future__ import annotations

import dataclasses
import math
import os
from typing import Dict, Optional

import numpy as np

LAYER_FULL = 0     # queries = every token of the user (full attention layer, Eq. for A^(l,h))
LAYER_TARGET = 1   # queries = target tokens only (target attention layer, Eq. for A_T^(l,h))

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream_key(seed: int, stream: int) -> np.uint64:
    """Key of an independent stream: two rounds of the splitmix64 finaliser over (seed, stream)."""
    with np.errstate(over="ignore"):
        a = _mix(np.asarray([np.uint64(seed) * _GOLDEN + np.uint64(stream + 1)], dtype=np.uint64))
        a = _mix(a + _GOLDEN)
    return a[0]


def raw_bits(key: np.uint64, start: int, n: int) -> np.ndarray:
    """splitmix64 outputs number start .. start+n-1 of the sequence whose state begins at ``key``."""
    with np.errstate(over="ignore"):
        ctr = np.arange(start + 1, start + n + 1, dtype=np.uint64)
        return _mix(key + ctr * _GOLDEN)


def uniform01(key: np.uint64, start: int, n: int) -> np.ndarray:
    """float64 uniforms in (0, 1): the top 53 bits, shifted by half a unit so 0 never occurs."""
    return ((raw_bits(key, start, n) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(key: np.uint64, n: int, chunk: int = 1 << 21, dtype=np.float64, scale: float = 1.0) -> np.ndarray:
    """n standard normals by Box-Muller in float64 (element 2i and 2i+1 come from uniform pair i), times
    ``scale``, stored as ``dtype``.  The value of an element depends only on (key, index): chunks are
    independent and are drawn by a few threads."""
    out = np.empty(n, dtype=dtype)
    starts = list(range(0, n, chunk))

    def work(pos):
        m = min(chunk, n - pos)
        tmp = np.empty(m, dtype=np.float64)
        first_pair = pos // 2
        npairs = (pos + m + 1) // 2 - first_pair
        u = uniform01(key, 2 * first_pair, 2 * npairs)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        t = (2.0 * math.pi) * u[1::2]
        z = np.empty(2 * npairs, dtype=np.float64)
        z[0::2] = r * np.cos(t)
        z[1::2] = r * np.sin(t)
        off = pos - 2 * first_pair
        tmp[:] = z[off:off + m]
        if scale != 1.0:
            tmp *= scale
        out[pos:pos + m] = tmp

    if len(starts) <= 1:
        for pos in starts:
            work(pos)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(work, starts))
    return out


# ----------------------------------------------------------------------------- bf16 containers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- workload recipes
@dataclasses.dataclass(frozen=True)
class Config:
    """One synthetic workload.  hist/targets are ('fixed', n) | ('list', [...]) | ('uniform', lo, hi)
    | ('pareto', scale, cap) with L = min(cap, floor(scale / u)), u ~ U(0,1)."""
    name: str
    layer: int
    batch: int
    hist: tuple
    targets: tuple
    Hq: int
    Hkv: int
    head_dim: int
    dtype: str          # 'bf16' | 'fp32'
    std: float          # q, k, v ~ std * N(0, 1)
    seed: int
    dout_std: float = 1.0
    rt: Optional[tuple] = None   # length spec of the real-time segment between history and targets, or None


# Timestamp windows of the three token kinds when a workload has real-time tokens (integers, drawn uniformly; history
# and real-time tokens are then sorted by time inside their segment, as Section 3.2.1 prescribes).  The windows
# overlap and are narrow on purpose: real-time tokens before and after an exposure, ties, history tokens later than
# some real-time tokens all occur.
TS_WINDOW_HIST = (0, 1000)
TS_WINDOW_RT = (900, 1100)
TS_WINDOW_TGT = (880, 1120)


CONFIGS: Dict[str, Config] = {
    # The five benchmark/parity workloads.  C3 is the one the headline metric is quoted on.
    "C1": Config("C1", LAYER_FULL, 2, ("list", [40, 64]), ("fixed", 8), 4, 1, 16, "fp32", 0.5, 0),
    "C2": Config("C2", LAYER_FULL, 64, ("uniform", 128, 512), ("fixed", 32), 8, 2, 64, "bf16", 0.3, 1),
    "C3": Config("C3", LAYER_FULL, 256, ("uniform", 512, 1024), ("fixed", 64), 8, 2, 64, "bf16", 0.3, 2),
    "C3_1024": Config("C3_1024", LAYER_FULL, 256, ("fixed", 1024), ("fixed", 64), 8, 2, 64, "bf16", 0.3, 2),
    "C4": Config("C4", LAYER_TARGET, 512, ("fixed", 2048), ("fixed", 128), 16, 4, 64, "bf16", 0.3, 3),
    "C5": Config("C5", LAYER_FULL, 128, ("pareto", 750.0, 8192), ("uniform", 16, 256), 16, 2, 128, "bf16", 0.3, 4),
    # The same shapes with a real-time segment (mask rule 2): parity and a bench line of their own.
    "C2_RT": Config("C2_RT", LAYER_FULL, 64, ("uniform", 128, 512), ("fixed", 32), 8, 2, 64, "bf16", 0.3, 11,
                    rt=("uniform", 8, 96)),
    "C3_RT": Config("C3_RT", LAYER_FULL, 256, ("uniform", 512, 1024), ("fixed", 64), 8, 2, 64, "bf16", 0.3, 12,
                    rt=("uniform", 32, 128)),
    "C4_RT": Config("C4_RT", LAYER_TARGET, 128, ("fixed", 2048), ("fixed", 128), 16, 4, 64, "bf16", 0.3, 13,
                    rt=("uniform", 32, 128)),
    # Inference shapes (request-level aggregation, Section 3.1, and the serving set-up of Section 3.3.3: one request = one user's history and the candidates of a
    # scenario; forward only, target layer; the history K/V are shared by all candidates of the request).  A few
    # requests at a time: far fewer (user, kv head) groups than compute units.
    "I1": Config("I1", LAYER_TARGET, 1, ("fixed", 2048), ("fixed", 128), 8, 2, 64, "bf16", 0.3, 21),
    "I2": Config("I2", LAYER_TARGET, 8, ("uniform", 512, 4096), ("uniform", 16, 128), 8, 2, 64, "bf16", 0.3, 22),
    "I3": Config("I3", LAYER_TARGET, 4, ("fixed", 8192), ("fixed", 64), 16, 2, 128, "bf16", 0.3, 23),
    "I2_RT": Config("I2_RT", LAYER_TARGET, 8, ("uniform", 512, 4096), ("uniform", 16, 128), 8, 2, 64, "bf16", 0.3, 24,
                    rt=("uniform", 16, 96)),
}

# stream ids (fixed; part of the recipe)
_S_HIST, _S_TGT, _S_Q, _S_K, _S_V, _S_DO, _S_RT, _S_TS = 0, 1, 2, 3, 4, 5, 6, 7


def _draw_lengths(spec: tuple, key: np.uint64, batch: int) -> np.ndarray:
    kind = spec[0]
    if kind == "fixed":
        return np.full(batch, int(spec[1]), dtype=np.int32)
    if kind == "list":
        vals = np.asarray(spec[1], dtype=np.int32)
        assert vals.shape[0] == batch
        return vals.copy()
    u = uniform01(key, 0, batch)
    if kind == "uniform":
        lo, hi = int(spec[1]), int(spec[2])
        return (lo + np.floor(u * (hi - lo + 1)).astype(np.int64)).clip(lo, hi).astype(np.int32)
    if kind == "pareto":
        scale, cap = float(spec[1]), int(spec[2])
        return np.minimum(cap, np.floor(scale / u)).astype(np.int32)
    raise ValueError(f"unknown length spec {spec!r}")


@dataclasses.dataclass
class Case:
    """A packed jagged batch.  q/k/v/dout hold float32 values exactly representable in ``dtype``
    (for bf16 the *_bits arrays carry the uint16 patterns the device receives)."""
    cfg: Config
    hist_len: np.ndarray       # [B] int32
    n_targets: np.ndarray      # [B] int32
    kv_offsets: np.ndarray     # [B+1] int32, prefix sums of L_b + T_b
    q_offsets: np.ndarray      # [B+1] int32, == kv_offsets (FULL) or prefix sums of T_b (TARGET)
    q: np.ndarray              # [total_q, Hq, d]  float32
    k: np.ndarray              # [total_kv, Hkv, d] float32
    v: np.ndarray              # [total_kv, Hkv, d] float32
    dout: Optional[np.ndarray]  # [total_q, Hq, d] float32 or None
    scale: float
    rt_len: Optional[np.ndarray] = None      # [B] int32 real-time tokens per user, or None (no such segment)
    timestamps: Optional[np.ndarray] = None  # [total_kv] int32, one per K/V row, or None

    @property
    def total_q(self) -> int:
        return int(self.q_offsets[-1])

    @property
    def total_kv(self) -> int:
        return int(self.kv_offsets[-1])

    @property
    def batch(self) -> int:
        return int(self.hist_len.shape[0])


def _values(key: np.uint64, shape: tuple, std: float, dtype: str) -> np.ndarray:
    n = int(np.prod(shape)) if len(shape) else 1
    x = normal(key, n, dtype=np.float32, scale=std)  # scaled in float64, then rounded to float32
    if dtype == "bf16":
        x = bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x.reshape(shape)


def offsets_from_lengths(lengths: np.ndarray) -> np.ndarray:
    off = np.zeros(lengths.shape[0] + 1, dtype=np.int64)
    np.cumsum(lengths.astype(np.int64), out=off[1:])
    assert off[-1] < 2 ** 31
    return off.astype(np.int32)


def _draw_timestamps(key: np.uint64, kv_offsets: np.ndarray, hist_len: np.ndarray, rt_len: np.ndarray) -> np.ndarray:
    """One integer timestamp per K/V row: uniform in the window of the token's kind, history and real-time
    segments sorted ascending inside each user."""
    total = int(kv_offsets[-1])
    u = uniform01(key, 0, total)
    ts = np.zeros(total, dtype=np.int32)
    for b in range(hist_len.shape[0]):
        s0, L, R, e = int(kv_offsets[b]), int(hist_len[b]), int(rt_len[b]), int(kv_offsets[b + 1])
        for lo, hi, (w0, w1), sort in ((s0, s0 + L, TS_WINDOW_HIST, True), (s0 + L, s0 + L + R, TS_WINDOW_RT, True),
                                      (s0 + L + R, e, TS_WINDOW_TGT, False)):
            seg = (w0 + np.floor(u[lo:hi] * (w1 - w0))).astype(np.int32).clip(w0, w1 - 1)
            ts[lo:hi] = np.sort(seg) if sort else seg
    return ts


def make_case(cfg: Config, with_dout: bool = True, hist_len: Optional[np.ndarray] = None,
              n_targets: Optional[np.ndarray] = None, rt_len: Optional[np.ndarray] = None) -> Case:
    """Draw one batch for ``cfg``.  Order of draws: lengths (history, targets, real-time), then q, k, v, dout,
    timestamps, each from its own stream in memory order.  Explicit ``hist_len`` / ``n_targets`` / ``rt_len``
    override the drawn lengths (edge-case tests)."""
    if hist_len is None:
        hist_len = _draw_lengths(cfg.hist, stream_key(cfg.seed, _S_HIST), cfg.batch)
    if n_targets is None:
        n_targets = _draw_lengths(cfg.targets, stream_key(cfg.seed, _S_TGT), cfg.batch)
    hist_len = np.asarray(hist_len, dtype=np.int32)
    n_targets = np.asarray(n_targets, dtype=np.int32)
    has_rt = cfg.rt is not None or rt_len is not None
    if has_rt and rt_len is None:
        rt_len = _draw_lengths(cfg.rt, stream_key(cfg.seed, _S_RT), cfg.batch)
    rt = np.asarray(rt_len, dtype=np.int32) if has_rt else np.zeros_like(hist_len)
    kv_offsets = offsets_from_lengths(hist_len + rt + n_targets)
    q_offsets = kv_offsets.copy() if cfg.layer == LAYER_FULL else offsets_from_lengths(n_targets)
    tq, tkv = int(q_offsets[-1]), int(kv_offsets[-1])
    q = _values(stream_key(cfg.seed, _S_Q), (tq, cfg.Hq, cfg.head_dim), cfg.std, cfg.dtype)
    k = _values(stream_key(cfg.seed, _S_K), (tkv, cfg.Hkv, cfg.head_dim), cfg.std, cfg.dtype)
    v = _values(stream_key(cfg.seed, _S_V), (tkv, cfg.Hkv, cfg.head_dim), cfg.std, cfg.dtype)
    dout = None
    if with_dout:
        dout = _values(stream_key(cfg.seed, _S_DO), (tq, cfg.Hq, cfg.head_dim), cfg.dout_std, cfg.dtype)
    ts = _draw_timestamps(stream_key(cfg.seed, _S_TS), kv_offsets, hist_len, rt) if has_rt else None
    return Case(cfg, hist_len, n_targets, kv_offsets, q_offsets, q, k, v, dout,
                1.0 / math.sqrt(cfg.head_dim), rt if has_rt else None, ts)


def custom_config(name: str, layer: int, hist_len, n_targets, Hq: int, Hkv: int, head_dim: int,
                  dtype: str = "bf16", std: float = 0.3, seed: int = 1234, rt_len=None) -> Config:
    hist_len = list(int(x) for x in hist_len)
    n_targets = list(int(x) for x in n_targets)
    rt = None if rt_len is None else ("list", list(int(x) for x in rt_len))
    return Config(name, layer, len(hist_len), ("list", hist_len), ("list", n_targets), Hq, Hkv, head_dim,
                  dtype, std, seed, rt=rt)


def take_users(case: Case, users) -> Case:
    """The sub-batch made of the listed users (rows gathered, offsets rebuilt).  Users are
    independent samples, so a result on the sub-batch is the result for those users."""
    users = [int(u) for u in users]
    qrows = np.concatenate([np.arange(case.q_offsets[u], case.q_offsets[u + 1]) for u in users]) if users else np.zeros(0, np.int64)
    kvrows = np.concatenate([np.arange(case.kv_offsets[u], case.kv_offsets[u + 1]) for u in users]) if users else np.zeros(0, np.int64)
    hl, nt = case.hist_len[users], case.n_targets[users]
    rl = None if case.rt_len is None else case.rt_len[users]
    kvo = offsets_from_lengths(hl + nt + (0 if rl is None else rl))
    qo = kvo.copy() if case.cfg.layer == LAYER_FULL else offsets_from_lengths(nt)
    return Case(case.cfg, hl, nt, kvo, qo, case.q[qrows], case.k[kvrows], case.v[kvrows],
                None if case.dout is None else case.dout[qrows], case.scale, rl,
                None if case.timestamps is None else case.timestamps[kvrows])


def user_rows(offsets: np.ndarray, users) -> np.ndarray:
    """Row indices (into a packed tensor) of the listed users, in the listed order."""
    users = [int(u) for u in users]
    if not users:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(offsets[u], offsets[u + 1]) for u in users])


def take_kv_group(case: Case, g: int) -> Case:
    """The sub-problem of one key/value head and the r query heads that read it (heads of different kv
    groups never interact, so a result on the slice is the result for those heads)."""
    cfg = case.cfg
    r = cfg.Hq // cfg.Hkv
    sub = dataclasses.replace(cfg, name=f"{cfg.name}_g{g}", Hq=r, Hkv=1)
    hs = slice(g * r, (g + 1) * r)
    return Case(sub, case.hist_len, case.n_targets, case.kv_offsets, case.q_offsets,
                np.ascontiguousarray(case.q[:, hs]), np.ascontiguousarray(case.k[:, g:g + 1]),
                np.ascontiguousarray(case.v[:, g:g + 1]),
                None if case.dout is None else np.ascontiguousarray(case.dout[:, hs]), case.scale, case.rt_len,
                case.timestamps)


def repeat_kv_heads(case: Case) -> Case:
    """The same batch with one key/value head per query head: kv head g = h / r copied for each of its r query heads
    (consecutive query heads share a kv head).  A rearrangement of the data only."""
    cfg = case.cfg
    r = cfg.Hq // cfg.Hkv
    sub = dataclasses.replace(cfg, name=f"{cfg.name}_mha", Hkv=cfg.Hq)
    return Case(sub, case.hist_len, case.n_targets, case.kv_offsets, case.q_offsets, case.q,
                np.repeat(case.k, r, axis=1), np.repeat(case.v, r, axis=1), case.dout, case.scale, case.rt_len,
                case.timestamps)


# ----------------------------------------------------------------------------- group layer normalization
@dataclasses.dataclass
class GlnCase:
    """Inputs of one group-layer-normalization call: tokens of several groups (history / real-time sequences,
    scenarios) whose features follow different distributions, which is what the group-wise parameters are for."""
    name: str
    dtype: str                 # 'bf16' | 'fp32'
    x: np.ndarray              # [n_tokens, d_model] float32, exactly representable in dtype
    gate: Optional[np.ndarray]  # [n_tokens, d_model] or None
    dy: np.ndarray             # [n_tokens, d_model]
    group_id: np.ndarray       # [n_tokens] int32
    gamma: np.ndarray          # [n_groups, d_model] float32
    beta: np.ndarray           # [n_groups, d_model] float32
    eps: float


_S_GLN_X, _S_GLN_U, _S_GLN_DY, _S_GLN_G, _S_GLN_GAMMA, _S_GLN_BETA, _S_GLN_STATS = 20, 21, 22, 23, 24, 25, 26


def make_gln_case(name: str, n_tokens: int, d_model: int, n_groups: int, dtype: str = "bf16", gated: bool = True,
                  seed: int = 100, eps: float = 1e-5) -> GlnCase:
    """Group ids are uniform over the groups (tokens of all sequences are interleaved by time, Section 3.2.1); the
    features of group g are N(mu_g, sigma_g^2) with mu_g ~ U(-1, 1), sigma_g ~ U(0.5, 2); gamma ~ 1 + 0.2 N(0,1),
    beta ~ 0.2 N(0,1) in float32; gate and upstream gradient ~ N(0, 1)."""
    gid = np.minimum((uniform01(stream_key(seed, _S_GLN_G), 0, n_tokens) * n_groups).astype(np.int32), n_groups - 1)
    st = uniform01(stream_key(seed, _S_GLN_STATS), 0, 2 * n_groups)
    mu, sigma = 2.0 * st[:n_groups] - 1.0, 0.5 + 1.5 * st[n_groups:]
    z = normal(stream_key(seed, _S_GLN_X), n_tokens * d_model, dtype=np.float32, scale=1.0).reshape(n_tokens, d_model)
    x = (z.astype(np.float64) * sigma[gid][:, None] + mu[gid][:, None]).astype(np.float32)
    dy = normal(stream_key(seed, _S_GLN_DY), n_tokens * d_model, dtype=np.float32, scale=1.0).reshape(n_tokens, d_model)
    gate = None
    if gated:
        gate = normal(stream_key(seed, _S_GLN_U), n_tokens * d_model, dtype=np.float32, scale=1.0).reshape(n_tokens, d_model)
    if dtype == "bf16":
        x = bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(n_tokens, d_model)
        dy = bf16_bits_to_f32(f32_to_bf16_bits(dy)).reshape(n_tokens, d_model)
        if gate is not None:
            gate = bf16_bits_to_f32(f32_to_bf16_bits(gate)).reshape(n_tokens, d_model)
    gamma = (1.0 + normal(stream_key(seed, _S_GLN_GAMMA), n_groups * d_model, dtype=np.float32, scale=0.2)).astype(np.float32)
    beta = normal(stream_key(seed, _S_GLN_BETA), n_groups * d_model, dtype=np.float32, scale=0.2)
    return GlnCase(name, dtype, x, gate, dy, gid, gamma.reshape(n_groups, d_model), beta.reshape(n_groups, d_model), eps)
