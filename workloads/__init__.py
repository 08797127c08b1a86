"""Seeded synthetic inputs for the batched token-sampling stage.

This module only *draws inputs* (logits, per-row sampling parameters, token
histories).  It contains none of the sampler's arithmetic, so that the CPU
oracle and the HIP library can both be fed from it without sharing any of the
method's code.

The five workloads stand in for the evaluation workload of the paper (prompts
from a public chat dataset decoded by large models with every sampling
strategy switched on, Sec. 7.1 "Workload"): they take the paper's shapes
(batch 256..1024, vocabulary up to ~2.5e5, Sec. 5.1) and fixed, seeded value
distributions instead of model outputs.

All draws of workload ``i`` (0-based) come from one
``numpy.random.Generator(PCG64(i))`` in the fixed order
logits -> spikes -> per-row parameters -> histories.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

__all__ = ["Workload", "make", "NAMES", "f32_to_bf16_bits", "bf16_bits_to_f32"]

NAMES = ("C1", "C2", "C3", "C4", "C5")


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    B: int
    V: int
    dtype: str                      # "f32" or "bf16"
    logits: np.ndarray              # [B, V] float32, or uint16 bf16 bit patterns
    params: Dict[str, Optional[np.ndarray]]   # per-row arrays of length B, or None = feature off
    hist_indptr: Optional[np.ndarray]         # int64 [B+1] or None
    hist_tokens: Optional[np.ndarray]         # int32 [nnz] or None
    k_logprobs: int
    seed: int = 0
    recipe: str = ""
    extra: dict = field(default_factory=dict)

    def logits_f32(self) -> np.ndarray:
        return self.logits if self.dtype == "f32" else bf16_bits_to_f32(self.logits)

    def history(self, b: int) -> np.ndarray:
        if self.hist_indptr is None:
            return np.zeros(0, dtype=np.int32)
        return self.hist_tokens[self.hist_indptr[b]:self.hist_indptr[b + 1]]

    def row_params(self, b: int) -> dict:
        out = {}
        for k, v in self.params.items():
            out[k] = None if v is None else v[b]
        return out


_PARAM_KEYS = ("temperature", "top_k", "top_p", "min_p",
               "repetition_penalty", "frequency_penalty", "presence_penalty")


def _empty_params() -> Dict[str, Optional[np.ndarray]]:
    return {k: None for k in _PARAM_KEYS}


def _zipf_ranks(rng: np.random.Generator, a: float, V: int, size) -> np.ndarray:
    """Ranks r in [1, V] with P(r) proportional to r**-a (truncated Zipf), by inverse CDF."""
    pmf = np.arange(1, V + 1, dtype=np.float64) ** (-a)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    u = rng.random(size)
    r = np.searchsorted(cdf, u, side="right")
    return np.minimum(r, V - 1) + 1


def _uniform_hist(rng, B, V, H):
    tok = rng.integers(0, V, size=(B, H), dtype=np.int64).astype(np.int32)
    indptr = np.arange(B + 1, dtype=np.int64) * H
    return indptr, tok.reshape(-1)


def _zipf_hist(rng, B, V, H, a):
    perm = rng.permutation(V).astype(np.int32)     # one vocabulary permutation shared by all rows
    ranks = _zipf_ranks(rng, a, V, (B, H))
    tok = perm[ranks - 1]
    indptr = np.arange(B + 1, dtype=np.int64) * H
    return indptr, tok.reshape(-1).astype(np.int32)


def make(index: int, B: Optional[int] = None, V: Optional[int] = None,
         H: Optional[int] = None) -> Workload:
    """Build workload ``index`` (0..4 = C1..C5).  ``B``, ``V``, ``H`` shrink the shape
    (same recipe, same seed) for tests that need a case a slow checker finishes quickly."""
    if not 0 <= index < 5:
        raise ValueError("workload index must be 0..4")
    rng = np.random.Generator(np.random.PCG64(index))
    P = _empty_params()
    f32 = np.float32

    if index == 0:
        B = 4 if B is None else B
        V = 32000 if V is None else V
        z = (rng.standard_normal((B, V), dtype=np.float32) * f32(2.0)).astype(np.float32)
        # four row kinds, repeated if B > 4
        kinds = np.arange(B) % 4
        P["temperature"] = np.select([kinds == 0, kinds == 1, kinds == 2, kinds == 3],
                                     [0.0, 0.8, 1.0, 0.7]).astype(np.float32)
        P["top_k"] = np.where(kinds == 1, 50, 0).astype(np.int32)
        P["top_p"] = np.where(kinds == 2, 0.9, 1.0).astype(np.float32)
        P["min_p"] = np.where(kinds == 3, 0.05, 0.0).astype(np.float32)
        return Workload("C1", B, V, "f32", z, P, None, None, 5, 0,
                        "fp32 N(0,2^2); rows greedy | T0.8+k50 | T1.0+p0.9 | T0.7+minp0.05; no history; top-5")

    if index == 1:
        B = 64 if B is None else B
        V = 128256 if V is None else V
        H = 512 if H is None else H
        z = (rng.standard_normal((B, V), dtype=np.float32) * f32(3.0)).astype(np.float32)
        for b in range(B):
            sp = rng.choice(V, size=min(8, V), replace=False)
            z[b, sp] += f32(8.0)
        bits = f32_to_bf16_bits(z)
        P["temperature"] = np.full(B, 0.7, dtype=np.float32)
        P["top_p"] = np.full(B, 0.95, dtype=np.float32)
        P["repetition_penalty"] = np.full(B, 1.1, dtype=np.float32)
        indptr, tok = _uniform_hist(rng, B, V, H)
        return Workload("C2", B, V, "bf16", bits, P, indptr, tok, 0, 0,
                        "bf16 N(0,3^2)+8 spikes(+8)/row; T0.7 p0.95; rep 1.1; 512 uniform history; sampled logprob only")

    if index == 2:
        B = 256 if B is None else B
        V = 152064 if V is None else V
        H = 1024 if H is None else H
        z = (rng.standard_normal((B, V), dtype=np.float32) * f32(2.5)).astype(np.float32)
        P["temperature"] = rng.uniform(0.3, 1.5, B).astype(np.float32)
        P["top_k"] = rng.choice(np.array([0, 20, 50, 1000]), size=B).astype(np.int32)
        P["top_p"] = rng.uniform(0.8, 1.0, B).astype(np.float32)
        P["min_p"] = np.full(B, 0.05, dtype=np.float32)
        P["frequency_penalty"] = np.full(B, 0.5, dtype=np.float32)
        P["presence_penalty"] = np.full(B, 0.3, dtype=np.float32)
        indptr, tok = _zipf_hist(rng, B, V, H, 1.1)
        return Workload("C3", B, V, "f32", z, P, indptr, tok, 20, 0,
                        "fp32 N(0,2.5^2); T~U[.3,1.5], k in {0,20,50,1000}, p~U[.8,1], minp .05; "
                        "freq .5 pres .3; 1024 Zipf(1.1) history; top-20")

    if index == 3:
        B = 1024 if B is None else B
        V = 129280 if V is None else V
        H = 2048 if H is None else H
        z = (rng.standard_t(3.0, size=(B, V)).astype(np.float32) * f32(2.0)).astype(np.float32)
        sp = rng.integers(0, V, size=B)
        z[np.arange(B), sp] += f32(12.0)
        bits = f32_to_bf16_bits(z)
        P["temperature"] = np.full(B, 1.0, dtype=np.float32)
        P["top_p"] = np.full(B, 0.9, dtype=np.float32)
        P["repetition_penalty"] = np.full(B, 1.05, dtype=np.float32)
        indptr, tok = _uniform_hist(rng, B, V, H)
        return Workload("C4", B, V, "bf16", bits, P, indptr, tok, 20, 0,
                        "bf16 2*t(3)+one spike(+12)/row; T1 p0.9; rep 1.05; 2048 uniform history; top-20")

    # index == 4
    B = 2048 if B is None else B
    V = 256000 if V is None else V
    H = 4096 if H is None else H
    z = (rng.standard_normal((B, V), dtype=np.float32) * f32(2.0)).astype(np.float32)
    greedy = (np.arange(B) % 2) == 0
    tau = rng.uniform(0.5, 1.2, B).astype(np.float32)
    tau[greedy] = 0.0
    kmax = min(4096, V)
    k = rng.integers(0, kmax + 1, size=B).astype(np.int32)
    k[greedy] = 0
    p = rng.uniform(0.85, 1.0, B).astype(np.float32)
    p[greedy] = 1.0
    P["temperature"] = tau
    P["top_k"] = k
    P["top_p"] = p
    P["repetition_penalty"] = np.full(B, 1.1, dtype=np.float32)
    P["frequency_penalty"] = np.full(B, 0.5, dtype=np.float32)
    P["presence_penalty"] = np.full(B, 0.3, dtype=np.float32)
    indptr, tok = _zipf_hist(rng, B, V, H, 1.2)
    return Workload("C5", B, V, "f32", z, P, indptr, tok, 20, 0,
                    "fp32 N(0,2^2); even rows greedy, odd rows T~U[.5,1.2], k~U{0..4096}, p~U[.85,1]; "
                    "rep 1.1 freq .5 pres .3; 4096 Zipf(1.2) history; top-20")
