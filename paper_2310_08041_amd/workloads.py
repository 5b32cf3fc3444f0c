"""Seeded synthetic inputs for the reassembled low-bit linear layer.

This module only draws random numbers: activations with outlier channels, norm parameters and
full-precision weights, in the shapes and distributions of the five benchmark configurations.
It contains none of the method's arithmetic (no norm, no reassembly, no quantizer) and imports
neither the HIP binding nor the CPU oracle, so both can be fed from it.

The activations stand in for LLaMA hidden states on 2048-token calibration segments, which the
paper uses but which are not available here: a light- or heavy-tailed bulk plus a few channels
that are large for every token (the paper's Sec. 1 and Sec. 4.3 describe outliers as concentrated
in fixed channels and tens of times larger than the rest).
"""
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 23100804 * 10


@dataclass(frozen=True)
class Workload:
    name: str
    index: int               # 1..5, position in the benchmark's configuration list
    N: int                   # tokens
    C: int                   # input channels
    O: int                   # output features
    in_dtype: str            # "f32" | "bf16"
    bulk: str                # "normal" | "laplace" | "student_t3"
    n_outlier: int           # number of outlier channels
    factor: tuple            # outlier channel multiplier ~ U(lo, hi)
    norm: str                # "layer" | "rms" | "none"
    gamma: str               # "ones" | "uniform" (U(0.5, 1.5))
    a_bits: int
    w_bits: int
    theta_rule: tuple        # ("fixed", theta) | ("expand", ratio) | ("tmax", T_max)
    eps: float = 1e-5
    w_std: float = 0.02
    extra: dict = field(default_factory=dict)

    @property
    def seed(self):
        return SEED_BASE + self.index


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny", 1, 64, 512, 512, "f32", "normal", 8, (20.0, 80.0), "layer", "ones", 4, 4,
                 ("fixed", 4.0)),
        Workload("llama7b_qkv", 2, 2048, 4096, 3 * 4096, "bf16", "normal", 20, (30.0, 100.0), "rms",
                 "uniform", 4, 4, ("expand", 0.01)),
        Workload("llama13b_upgate", 3, 4096, 5120, 2 * 13824, "bf16", "laplace", 15, (50.0, 150.0), "rms",
                 "uniform", 4, 4, ("expand", 0.01)),
        Workload("llama70b_down", 4, 2048, 28672, 8192, "bf16", "student_t3", 57, (50.0, 200.0), "rms",
                 "uniform", 4, 4, ("tmax", 8)),
        Workload("llama70b_q_decode", 5, 16, 8192, 8192, "bf16", "normal", 41, (30.0, 100.0), "rms",
                 "uniform", 6, 6, ("expand", 0.01)),
    ]
}


def f32_to_bf16_bits(x):
    """Round-to-nearest-even conversion of finite float32 values to bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _streams(seed, n=5):
    """Independent sub-streams in a fixed order: bulk, outlier set, outlier factors, norm params, W."""
    return [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(n)]


def draw_activations(w: Workload, N=None, C=None, seed=None):
    """Returns (X, outlier_channels, outlier_factors).

    X is [N, C]: float32 for "f32" workloads, uint16 holding bfloat16 bits for "bf16" ones.
    Every token of outlier channel c is multiplied by the same factor f_c.
    """
    N = w.N if N is None else N
    C = w.C if C is None else C
    g_bulk, g_set, g_fac, _, _ = _streams(w.seed if seed is None else seed)
    if w.bulk == "normal":
        x = g_bulk.standard_normal((N, C), dtype=np.float32)
    elif w.bulk == "laplace":
        x = g_bulk.laplace(0.0, 1.0, (N, C)).astype(np.float32)
    elif w.bulk == "student_t3":
        x = g_bulk.standard_t(3.0, (N, C)).astype(np.float32)
    else:
        raise ValueError(w.bulk)
    n_out = min(w.n_outlier, C)
    chans = np.sort(g_set.choice(C, size=n_out, replace=False)).astype(np.int64)
    fac = g_fac.uniform(w.factor[0], w.factor[1], size=n_out).astype(np.float32)
    x[:, chans] *= fac[None, :]
    if w.in_dtype == "bf16":
        return f32_to_bf16_bits(x), chans, fac
    return x, chans, fac


def draw_norm_params(w: Workload, C=None, seed=None):
    """Returns (gamma, beta) float32 [C]; beta is None unless the workload uses LayerNorm."""
    C = w.C if C is None else C
    g = _streams(w.seed if seed is None else seed)[3]
    if w.gamma == "ones":
        gamma = np.ones(C, np.float32)
    else:
        gamma = g.uniform(0.5, 1.5, size=C).astype(np.float32)
    beta = np.zeros(C, np.float32) if w.norm == "layer" else None
    return gamma, beta


def draw_weight(w: Workload, C=None, O=None, seed=None):
    """Full-precision weight [C, O] (input channels x output features), N(0, w_std)."""
    C = w.C if C is None else C
    O = w.O if O is None else O
    g = _streams(w.seed if seed is None else seed)[4]
    W = g.standard_normal((C, O), dtype=np.float32)
    W *= np.float32(w.w_std)
    return W


def draw_weight_codes(w: Workload, K, O=None, seed=None):
    """Uniformly random weight codes [O, K] uint8 in [0, 2^w_bits) with plausible per-channel
    scale / zero-point vectors, for throughput runs that need no particular weight values."""
    O = w.O if O is None else O
    g = _streams(w.seed if seed is None else seed)[4]
    codes = g.integers(0, 1 << w.w_bits, size=(O, K), dtype=np.uint8)
    scale = g.uniform(0.005, 0.02, size=O).astype(np.float32)
    zero = g.integers(0, 1 << w.w_bits, size=O).astype(np.int32)
    return codes, scale, zero
