"""Seeded synthetic inputs shaped like the paper's LLM-layer workloads.

This module only draws random arrays (numpy); it holds none of the method's arithmetic and is
the one piece of code that the GPU path's tests and the CPU oracle's tests both use.  The arrays
are the contract: the same arrays are uploaded to the GPU and upcast to float64 for the oracle.

Recipe (all workloads): q, k rows i.i.d. N(0, I) then L2-normalised along the head dimension
(the paper normalises q and k this way in its synthetic solver study, Appendix D); v ~ N(0, 1);
decay gate gamma = sigmoid(N(gate_mean, 1)) per head and token; ridge lambda =
lambda_mult * softplus(N(0, 1)) + lambda_add.  The "lowrank" workload draws keys from a rank-16
Gaussian subspace plus 1e-3 isotropic noise before normalising.  Draw order for a workload:
q, k (or basis, coefficients, noise), v, gate logits, lambda logits, all float32 draws from
numpy.random.default_rng(seed).  bf16 workloads round q, k, v to bfloat16 (round to nearest
even); gate and lambda stay float32.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    T: int
    d: int
    chunk: int
    n_iter: int
    dtype: str            # "f32" or "bf16": dtype of q, k, v, o
    gate_mean: float
    lambda_mult: float
    lambda_add: float
    seed: int
    lowrank: int = 0      # > 0: keys from a rank-`lowrank` subspace + 1e-3 noise

    def scaled(self, **kw):
        """Same distributions at another size (parity cases that the oracle finishes quickly)."""
        return replace(self, **kw)


# The five benchmark configurations.
CFG1 = Workload("cfg1_tiny_f32", B=1, H=1, T=256, d=64, chunk=64, n_iter=8, dtype="f32",
                gate_mean=2.0, lambda_mult=1.0, lambda_add=1e-2, seed=0)
CFG2 = Workload("cfg2_layer_bf16", B=4, H=16, T=4096, d=128, chunk=64, n_iter=10, dtype="bf16",
                gate_mean=3.0, lambda_mult=1.0, lambda_add=1e-2, seed=1)
CFG3 = Workload("cfg3_long_bf16", B=1, H=32, T=32768, d=128, chunk=64, n_iter=10, dtype="bf16",
                gate_mean=4.0, lambda_mult=1.0, lambda_add=1e-2, seed=2)
CFG4 = Workload("cfg4_illcond_bf16", B=2, H=8, T=8192, d=128, chunk=64, n_iter=16, dtype="bf16",
                gate_mean=3.0, lambda_mult=1e-3, lambda_add=0.0, seed=3, lowrank=16)
# Decode: 256 sequences x 32 heads, prefilled from 2048 tokens, then 1024 single-token steps.
CFG5 = Workload("cfg5_decode_bf16", B=256, H=32, T=2048, d=128, chunk=64, n_iter=10, dtype="bf16",
                gate_mean=3.0, lambda_mult=1.0, lambda_add=1e-2, seed=4)
CFG5_DECODE_STEPS = 1024

CONFIGS = {w.name: w for w in (CFG1, CFG2, CFG3, CFG4, CFG5)}


def round_to_bf16(x):
    """float32 array -> float32 array holding the nearest bfloat16 values (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + rounding) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def bf16_bits(x):
    """float32 array of bf16-representable values -> uint16 bit patterns (for upload)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def bf16_from_bits(bits):
    """uint16 bfloat16 bit patterns -> float32 values."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _normalise_rows(x):
    n = np.sqrt(np.sum(x.astype(np.float64) ** 2, axis=-1, keepdims=True))
    return (x / n).astype(np.float32)


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x.astype(np.float64)))


def _softplus(x):
    x = x.astype(np.float64)
    return np.log1p(np.exp(-np.abs(x))) + np.maximum(x, 0.0)


def draw_tokens(rng, w, B, T):
    """Draw B x T tokens of workload w's distribution from rng. Returns dict of float32 arrays
    q, k, v [B,T,H,d]; gate, lam [B,T,H]."""
    shape = (B, T, w.H, w.d)
    q = _normalise_rows(rng.standard_normal(shape, dtype=np.float32))
    if w.lowrank > 0:
        basis = rng.standard_normal((B, w.H, w.lowrank, w.d), dtype=np.float32)
        coeff = rng.standard_normal((B, T, w.H, w.lowrank), dtype=np.float32)
        noise = rng.standard_normal(shape, dtype=np.float32)
        k = np.einsum("bthr,bhrd->bthd", coeff, basis) + np.float32(1e-3) * noise
        k = _normalise_rows(k)
    else:
        k = _normalise_rows(rng.standard_normal(shape, dtype=np.float32))
    v = rng.standard_normal(shape, dtype=np.float32)
    gate_logits = rng.standard_normal((B, T, w.H), dtype=np.float32) + np.float32(w.gate_mean)
    lam_logits = rng.standard_normal((B, T, w.H), dtype=np.float32)
    gate = _sigmoid(gate_logits).astype(np.float32)
    lam = (w.lambda_mult * _softplus(lam_logits) + w.lambda_add).astype(np.float32)
    if w.dtype == "bf16":
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return {"q": q, "k": k, "v": v, "gate": gate, "lam": lam}


def make_inputs(w):
    """All tokens of workload w (forward / prefill part)."""
    rng = np.random.default_rng(w.seed)
    return draw_tokens(rng, w, w.B, w.T)


def make_gates(w, T=None, seed_offset=5000):
    """Optional per-token gates of the layer's variants, [B,T,H] float32 each, both in (0, 1) as sigmoid
    outputs: beta (write gate of the beta-augmented recurrence) and alpha (alpha-connection)."""
    rng = np.random.default_rng(w.seed + seed_offset)
    T = w.T if T is None else T
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    beta = sig(rng.normal(1.0, 1.0, (w.B, T, w.H))).astype(np.float32)
    alpha = sig(rng.normal(1.0, 1.0, (w.B, T, w.H))).astype(np.float32)
    return {"beta": beta, "alpha": alpha}


def make_decode_tokens(w, n_steps, seed_offset=1000):
    """Single-token inputs for n_steps decode steps: arrays [n_steps, B, H, d] / [n_steps, B, H]."""
    rng = np.random.default_rng(w.seed + seed_offset)
    x = draw_tokens(rng, w, w.B, n_steps)          # [B, n_steps, H, ...]
    return {name: np.ascontiguousarray(np.moveaxis(a, 1, 0)) for name, a in x.items()}
