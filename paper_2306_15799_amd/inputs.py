"""Seeded synthetic inputs for FLuRKA attention workloads.

This module only draws random numbers, scales them and rounds them to the
storage type.  It contains none of the method's arithmetic, so the CPU oracle
and the HIP path can both be fed from it without sharing any computation.

Distributions follow the paper's set-up: the sequence projections E, F are
(k x n) with iid N(0, 1/k) entries (Sec. 2, "Low-rank Methods"; written there
with d_k for k and N for n), the random-feature directions omega are iid
N(0, 1) (Sec. 2, "Kernel Methods": iid random variables psi_1..psi_m), and
Q, K, V are iid N(0, 1) scaled by d^(-1/4) so that q.k has the variance the
usual 1/sqrt(d) temperature would give (the library itself applies no
temperature).  The upstream gradient dOut is iid N(0, 1).

Draw order is fixed (Q, K, V, E, F, omega, dOut) so that a seed names one
input set for good.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np

PHI_PERFORMER = "performer"
PHI_ELU1 = "elu1"


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    n: int
    d: int
    k: int
    m: int
    dtype: str          # "f32" or "bf16": storage type of every tensor argument
    phi: str            # PHI_PERFORMER or PHI_ELU1
    backward: bool      # whether the workload includes the backward pass
    omega_per_head: bool = True

    @property
    def tokens_heads(self) -> int:
        return self.B * self.H * self.n

    def as_dict(self) -> dict:
        return asdict(self)


# The five benchmark / parity workloads.  C1 is the small fp32 case, C5 the
# forward+backward (training step) case, C4 the long-sequence case.
WORKLOADS = {
    "C1": Workload("C1", 1, 1, 512, 64, 64, 64, "f32", PHI_PERFORMER, False),
    "C2": Workload("C2", 8, 8, 4096, 64, 256, 256, "bf16", PHI_PERFORMER, False),
    "C3": Workload("C3", 4, 16, 16384, 64, 256, 64, "bf16", PHI_ELU1, False),
    "C4": Workload("C4", 1, 16, 65536, 128, 512, 256, "bf16", PHI_PERFORMER, False),
    "C5": Workload("C5", 4, 12, 8192, 64, 256, 256, "bf16", PHI_PERFORMER, True),
}

# Not benchmark configurations: shapes derived from them for timing code paths the five do not reach.
# C4T is the long-sequence shape as a training step (head size 128 through the backward kernels; with
# 256 features the dQ kernel streams one operand term through an LDS ring), D128T the same with 192
# features, the most for which that kernel holds all its operand images in LDS; C3T is the elu1
# workload as a training step.
DERIVED_WORKLOADS = {
    "C4T": Workload("C4T", 1, 16, 65536, 128, 512, 256, "bf16", PHI_PERFORMER, True),
    "D128T": Workload("D128T", 1, 16, 65536, 128, 512, 192, "bf16", PHI_PERFORMER, True),
    "C3T": Workload("C3T", 4, 16, 16384, 64, 256, 64, "bf16", PHI_ELU1, True),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even).

    Returns float32 values that are exactly representable in bfloat16.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng: np.random.Generator, shape, scale: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        out *= np.float32(scale)
    return out


def make_inputs(w: Workload, seed: int = 0) -> dict:
    """Draw one input set for workload `w`.

    Every array is float32; for a "bf16" workload each value has already been
    rounded to bfloat16, so the oracle (which widens to float64) and the GPU
    (which stores the 16-bit patterns) see identical numbers.
    Keys: Q, K, V (B,H,n,d); E, F (k,n); omega (H,m,d) or (1,m,d), None for
    the elu1 map; dOut (B,H,n,d) only when the workload has a backward pass.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    qkv_scale = float(w.d) ** -0.25
    ef_scale = float(w.k) ** -0.5
    shape = (w.B, w.H, w.n, w.d)
    t = {}
    t["Q"] = _normal(rng, shape, qkv_scale)
    t["K"] = _normal(rng, shape, qkv_scale)
    t["V"] = _normal(rng, shape, qkv_scale)
    t["E"] = _normal(rng, (w.k, w.n), ef_scale)
    t["F"] = _normal(rng, (w.k, w.n), ef_scale)
    if w.phi == PHI_PERFORMER:
        t["omega"] = _normal(rng, (w.H if w.omega_per_head else 1, w.m, w.d), 1.0)
    else:
        t["omega"] = None
    if w.backward:
        t["dOut"] = _normal(rng, shape, 1.0)
    if w.dtype == "bf16":
        for key, val in t.items():
            if val is not None:
                t[key] = round_to_bf16(val)
    elif w.dtype != "f32":
        raise ValueError(f"unknown dtype {w.dtype!r}")
    return t


def make_paper_order_inputs(w: Workload, dm: int, seed: int = 0) -> dict:
    """Inputs of the forward in the paper's order (projection before the per-head transform).

    As `make_inputs`, with K, V replaced by the model-wide layer inputs XK, XV (B, n, dm) ~ N(0, 1) and
    the per-head transforms WK, WV (H, d, dm) ~ N(0, 1 / dm) * d^(-1/4), stored transposed, so that
    X W has the scale K and V have in the other workloads.  Draw order: Q, XK, XV, E, F, omega, WK, WV.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    qkv_scale = float(w.d) ** -0.25
    t = {}
    t["Q"] = _normal(rng, (w.B, w.H, w.n, w.d), qkv_scale)
    t["XK"] = _normal(rng, (w.B, w.n, dm), 1.0)
    t["XV"] = _normal(rng, (w.B, w.n, dm), 1.0)
    t["E"] = _normal(rng, (w.k, w.n), float(w.k) ** -0.5)
    t["F"] = _normal(rng, (w.k, w.n), float(w.k) ** -0.5)
    t["omega"] = _normal(rng, (w.H if w.omega_per_head else 1, w.m, w.d), 1.0) if w.phi == PHI_PERFORMER else None
    t["WK"] = _normal(rng, (w.H, w.d, dm), qkv_scale * float(dm) ** -0.5)
    t["WV"] = _normal(rng, (w.H, w.d, dm), qkv_scale * float(dm) ** -0.5)
    if w.dtype == "bf16":
        for key, val in t.items():
            if val is not None:
                t[key] = round_to_bf16(val)
    elif w.dtype != "f32":
        raise ValueError(f"unknown dtype {w.dtype!r}")
    return t


def shrink(w: Workload, **over) -> Workload:
    """A copy of `w` with some fields replaced (used for small parity cases)."""
    d = w.as_dict()
    d.update(over)
    return Workload(**d)
