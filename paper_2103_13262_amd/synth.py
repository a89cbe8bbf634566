"""Seeded synthetic inputs for the MoE layer (shared by tests and bench.py).

Holds none of the method's arithmetic: it only draws random tensors of the
shapes and distributions of the five workloads, shapes the expert load with a
gate bias, and rounds to the storage type.  numpy only (no torch, no GPU).

The paper's single-GPU experiment (Section 5.2) uses a randomly initialised gate
matrix and random inputs at n_b=4096, d_m=1024, d_h=4096, k=2; workload "C1" is
that shape.  No public dataset is involved anywhere on this path.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int          # n_b  tokens
    d: int          # d_m
    h: int          # d_h
    E: int          # n_e  experts (all local)
    k: int          # top-k
    dtype: str      # "f32" | "bf16"  storage of X, weights, outputs
    zipf_s: float = 0.0   # 0: gate bias zero (near-uniform load); >0: expected load ~ (e+1)^-s
    seed: int = 0
    bias_std: float = 0.0  # > 0: the experts have biases b1[E,h], b2[E,d] ~ N(0, bias_std) (the five workloads have none)
    score_all: bool = False  # scores = softmax over all experts instead of over the selected ones (ditto)

    @property
    def M(self):
        return self.N * self.k

    def expert_flops(self):
        """Multiply-add flops of the six expert GEMMs, forward + backward (12 M d h)."""
        return 12 * self.M * self.d * self.h


_BASE_SEED = 20210313 * 10

WORKLOADS = {
    "C0": Workload("C0", 256, 64, 128, 4, 2, "f32", 0.0, _BASE_SEED + 0),
    "C1": Workload("C1", 4096, 1024, 4096, 16, 2, "bf16", 0.0, _BASE_SEED + 1),
    "C2": Workload("C2", 8192, 1024, 4096, 64, 2, "bf16", 1.2, _BASE_SEED + 2),
    "C3": Workload("C3", 16384, 512, 1024, 256, 1, "bf16", 0.0, _BASE_SEED + 3),
    "C4": Workload("C4", 32768, 2048, 8192, 32, 2, "bf16", 0.8, _BASE_SEED + 4),
}


def f32_to_bf16_bits(a):
    """Round-to-nearest-even fp32 -> bfloat16 bit patterns (uint16). Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed, stream, shape, std):
    g = np.random.Generator(np.random.Philox(key=[seed, stream]))
    out = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def gate_bias(w: Workload):
    """b_g[e] = beta * ln p_e with p_e ~ (e+1)^-s: for Gumbel-like logit noise of std
    sigma_l = 0.02*sqrt(d) the arg-max then follows p approximately. float32 [E]."""
    if w.zipf_s <= 0.0:
        return np.zeros(w.E, np.float32)
    p = (np.arange(w.E, dtype=np.float64) + 1.0) ** (-w.zipf_s)
    p /= p.sum()
    beta = 0.02 * np.sqrt(w.d) / 1.2825
    return (beta * np.log(p)).astype(np.float32)


def make_inputs(w: Workload, with_dy=True):
    """Returns dict of numpy arrays: X[N,d], Wg[d,E], bg[E] f32, W1[E,d,h], W2[E,h,d], dY[N,d]
    (and b1[E,h], b2[E,d] when the workload has expert biases).

    For dtype "bf16" the tensors are uint16 bit patterns (exactly what both the
    oracle and the GPU receive); for "f32" they are float32.
    """
    t = {
        "X": _normal(w.seed, 0, (w.N, w.d), 1.0),
        "Wg": _normal(w.seed, 1, (w.d, w.E), 0.02),
        "W1": _normal(w.seed, 3, (w.E, w.d, w.h), 0.02),
        "W2": _normal(w.seed, 4, (w.E, w.h, w.d), 0.02),
    }
    if with_dy:
        t["dY"] = _normal(w.seed, 5, (w.N, w.d), 1.0)
    if w.bias_std > 0.0:
        t["b1"] = _normal(w.seed, 6, (w.E, w.h), w.bias_std)
        t["b2"] = _normal(w.seed, 7, (w.E, w.d), w.bias_std)
    if w.dtype == "bf16":
        t = {n: f32_to_bf16_bits(a) for n, a in t.items()}
    elif w.dtype != "f32":
        raise ValueError(w.dtype)
    t["bg"] = gate_bias(w)
    return t


def scaled(w: Workload, **kw):
    """A copy of a workload with some fields replaced (parity cases at other sizes)."""
    return replace(w, **kw)
