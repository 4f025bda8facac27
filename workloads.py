"""Seeded synthetic inputs for the fused linear cross-entropy path.

This module only draws random numbers and rounds them to the storage type.
It holds none of the method's arithmetic (no projection, softmax, loss or
gradient), so the CPU oracle and the HIP path may both be fed from it
without sharing any code of the method itself.

The five named workloads are lm_head shapes: hidden states X[BT x H] ~ N(0,1),
head weight W[V x H] ~ N(0, 0.02^2), integer targets in [0, V) with a fraction
replaced by ignore_index = -100.  Everything is a pure function of
(workload, seed); the bit generator is numpy's counter-based Philox, keyed by
(seed, tensor id), so a tensor can be regenerated on any host.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

IGNORE_INDEX = -100
BASE_SEED = 241010989

# name, BT, H, V, dtype, target law, ignore law
CONFIGS = (
    dict(name="tiny_fp32", BT=256, H=512, V=4096, dtype="f32",
         targets="uniform", ignore=("none",)),
    dict(name="llama2_7b_lm_head", BT=4096, H=4096, V=32000, dtype="bf16",
         targets="uniform", ignore=("iid", 0.10)),
    dict(name="llama3_8b_lm_head", BT=8192, H=4096, V=128256, dtype="bf16",
         targets="zipf", ignore=("iid", 0.05)),
    dict(name="qwen2_7b_lm_head", BT=16384, H=3584, V=152064, dtype="bf16",
         targets="uniform", ignore=("pad", 2048, 819)),
    dict(name="gemma2_2b_lm_head", BT=8192, H=2304, V=256000, dtype="bf16",
         targets="uniform", ignore=("iid", 0.30)),
)

_TENSOR_X, _TENSOR_W, _TENSOR_T, _TENSOR_IGN = 1, 2, 3, 4


@dataclass
class Workload:
    name: str
    BT: int
    H: int
    V: int
    dtype: str                 # "f32" or "bf16": the storage type of X, W, dX, dW
    X: np.ndarray              # float32 [BT, H]; exactly representable in `dtype`
    W: np.ndarray              # float32 [V, H];  exactly representable in `dtype`
    targets: np.ndarray        # int64 [BT]; class id in [0, V) or ignore_index
    ignore_index: int
    seed: int

    @property
    def n_valid(self) -> int:
        return int((self.targets != self.ignore_index).sum())


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, tensor_id]))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), in place,
    returning the same float32 array (low 16 mantissa bits cleared)."""
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += np.uint32(0x7FFF)
    u += lsb
    u &= np.uint32(0xFFFF0000)
    return a


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of a float32 array whose values are already bf16."""
    u = np.ascontiguousarray(a).view(np.uint32)
    assert not (u & np.uint32(0xFFFF)).any(), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed, tid, shape, std, dtype):
    g = _rng(seed, tid)
    a = np.empty(shape, dtype=np.float32)
    flat = a.reshape(-1)
    step = 1 << 24
    for s in range(0, flat.size, step):          # bounded temporaries
        g.standard_normal(out=flat[s:s + step], dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if dtype == "bf16":
        round_to_bf16(a)
    elif dtype != "f32":
        raise ValueError(f"unknown dtype {dtype!r}")
    return a


def _targets(seed, BT, V, law):
    g = _rng(seed, _TENSOR_T)
    if law == "uniform":
        return g.integers(0, V, size=BT, dtype=np.int64)
    if law == "zipf":
        # Zipf(s = 1.1) over ranks 1..V, class id = rank - 1, by inverse CDF.
        p = np.arange(1, V + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(p)
        cdf /= cdf[-1]
        u = g.random(BT)
        return np.minimum(np.searchsorted(cdf, u, side="left"), V - 1).astype(np.int64)
    raise ValueError(f"unknown target law {law!r}")


def _apply_ignore(seed, t, law, ignore_index):
    g = _rng(seed, _TENSOR_IGN)
    kind = law[0]
    if kind == "none":
        return t
    if kind == "iid":
        t[g.random(t.size) < law[1]] = ignore_index
        return t
    if kind == "pad":
        # sequences of `seq` tokens; each ends in a run of ignored positions
        # whose length is uniform in [0, max_pad]
        seq, max_pad = law[1], law[2]
        for s in range(0, t.size, seq):
            e = min(s + seq, t.size)
            n = int(g.integers(0, max_pad + 1))
            n = min(n, e - s)
            if n:
                t[e - n:e] = ignore_index
        return t
    raise ValueError(f"unknown ignore law {law!r}")


def make(BT, H, V, dtype="bf16", targets="uniform", ignore=("none",), seed=BASE_SEED,
         name="custom", x_std=1.0, w_std=0.02, ignore_index=IGNORE_INDEX) -> Workload:
    X = _normal(seed, _TENSOR_X, (BT, H), x_std, dtype)
    W = _normal(seed, _TENSOR_W, (V, H), w_std, dtype)
    t = _targets(seed, BT, V, targets)
    t = _apply_ignore(seed, t, ignore, ignore_index)
    return Workload(name, BT, H, V, dtype, X, W, t, ignore_index, seed)


@dataclass
class MultiHeadWorkload:
    base: Workload                     # X, head 0's W and targets
    Ws: list                           # n_heads weights [V, H]
    targets: list                      # n_heads int64 [BT]
    weights: list                      # n_heads floats


def make_multihead(n_heads, BT, H, V, seq, dtype="bf16", targets="uniform", ignore=("none",),
                   seed=BASE_SEED, decay=0.8, **kw) -> MultiHeadWorkload:
    """Inputs for several decoding heads on shared hidden states.

    The rows are sequences of `seq` tokens.  Head 0 has the base workload's
    targets; head j looks j positions further on inside the same sequence (its
    target at position t is head 0's target at t + j) and ignores the last j
    positions of every sequence.  Each head has its own weight (tensor ids
    16 + j); head j's loss weight is decay**j.
    """
    base = make(BT, H, V, dtype, targets, ignore, seed, name=f"multihead{n_heads}", **kw)
    Ws, ts = [base.W], [base.targets]
    w_std = kw.get("w_std", 0.02)
    for j in range(1, n_heads):
        Ws.append(_normal(seed, 16 + j, (V, H), w_std, dtype))
        t = np.full(BT, base.ignore_index, dtype=np.int64)
        for s in range(0, BT, seq):
            e = min(s + seq, BT)
            if e - s > j:
                t[s:e - j] = base.targets[s + j:e]
        ts.append(t)
    return MultiHeadWorkload(base, Ws, ts, [float(decay) ** j for j in range(n_heads)])


def make_rmsnorm_inputs(w: Workload):
    """Raw hidden states and RMSNorm scale for workload w: h = w.X times a
    log-normal factor per row (tensor id 32), gamma = 1 + 0.1 N(0,1) (tensor id
    33), both rounded to w's storage type.  Returns (h, gamma) as float32."""
    g = _rng(w.seed, 32)
    scale = np.exp(0.5 * g.standard_normal(w.BT)).astype(np.float32)
    h = w.X * scale[:, None]
    gamma = (1.0 + 0.1 * _rng(w.seed, 33).standard_normal(w.H)).astype(np.float32)
    if w.dtype == "bf16":
        round_to_bf16(h)
        round_to_bf16(gamma)
    return h, gamma


def make_config(index: int, BT: int | None = None) -> Workload:
    """Workload `index` (1-based, the order of the benchmark's config list).
    `BT` overrides the row count (used for bounded samples and BT sweeps)."""
    c = CONFIGS[index - 1]
    return make(BT if BT is not None else c["BT"], c["H"], c["V"], c["dtype"],
                c["targets"], c["ignore"], seed=BASE_SEED + index, name=c["name"])


def checksum(w: Workload) -> str:
    """Short digest of the generated bits, to detect a generator that drifted."""
    import hashlib
    h = hashlib.sha256()
    h.update(np.ascontiguousarray(w.X[: min(w.BT, 64)]).tobytes())
    h.update(np.ascontiguousarray(w.W[:: max(1, w.V // 64)][:64]).tobytes())
    h.update(w.targets.tobytes())
    return h.hexdigest()[:16]
