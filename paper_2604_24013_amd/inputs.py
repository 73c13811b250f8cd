"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds shapes and random-number recipes only -- none of the
method's arithmetic.  Both the GPU path and the CPU oracle are fed the arrays
produced here (bf16 tensors as raw ``uint16`` bit patterns, so both sides
read exactly the same values).

The paper (Sec. 5, experiments) measures on random activations of stated
shapes, not on a dataset; the workloads below take Llama-7B / Llama-70B layer
shapes.  Every tensor gets its own spawned ``numpy`` bit stream:
``SeedSequence(24013000 + config_number).spawn(...)[tensor_index]``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 24013000


@dataclass(frozen=True)
class Workload:
    """One emulated rank step.  ``kind``: 'rs' (GEMM + reduce-scatter, Alg. 2/3),
    'ag' (all-gather + GEMM, Alg. 1), 'dp' (gradient reduce-scatter step)."""
    name: str
    number: int          # position in the benchmark's list of configurations
    kind: str
    p: int               # ring size T = N
    m_chunk: int         # rows per sequence slice (B*S/p); for 'dp': elements per slice
    n: int               # output features of this rank's shard (0 for 'dp')
    k: int               # contraction length of this rank's shard (0 for 'dp')
    dtype: str           # 'bf16' or 'f32' operands (accumulation is always fp32)
    out_dtype: str       # 'f32' or 'bf16' (AG output only)
    sigma_a: float       # std of activations / gradient values
    sigma_w: float       # std of weights
    recv_rule: str       # 'unit' -> N(0, sigma_a); 'partial' -> N(0, sigma_a*sigma_w*sqrt(k*i))

    @property
    def flops(self) -> float:
        return 2.0 * self.p * self.m_chunk * self.n * self.k


CONFIGS: Dict[str, Workload] = {
    # GEMM + reduce-scatter, simulated TP p=2, fp32, all values N(0,1)
    "c1_rs_f32": Workload("c1_rs_f32", 0, "rs", 2, 128, 256, 512, "f32", "f32", 1.0, 1.0, "unit"),
    # Llama-7B MLP down-projection, p=8: K-shard 11008/8
    "c2_rs_7b": Workload("c2_rs_7b", 1, "rs", 8, 512, 4096, 1376, "bf16", "f32", 0.02, 0.02, "partial"),
    # Llama-7B QKV projection, p=8: N-shard 3*4096/8
    "c3_ag_7b": Workload("c3_ag_7b", 2, "ag", 8, 512, 1536, 4096, "bf16", "f32", 0.02, 0.02, "partial"),
    # Llama-70B MLP pair, p=8, seq 8192, hidden 8192, ffn 28672/8 = 3584
    "c4_ag_70b_up": Workload("c4_ag_70b_up", 3, "ag", 8, 1024, 3584, 8192, "bf16", "bf16", 0.01, 0.01, "partial"),
    "c4_rs_70b_down": Workload("c4_rs_70b_down", 3, "rs", 8, 1024, 8192, 3584, "bf16", "f32", 0.01, 0.01, "partial"),
    # data-parallel gradient bucket of 1e9 fp32 values in 8 slices
    "c5_dp": Workload("c5_dp", 4, "dp", 8, 125_000_000, 0, 0, "f32", "f32", 1e-3, 0.0, "unit"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller parity cases)."""
    return replace(w, **kw)


def _rng(w: Workload, tensor_index: int, salt: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence(BASE_SEED + w.number + 1000 * salt)
    return np.random.default_rng(ss.spawn(tensor_index + 1)[tensor_index])


def normal_f32(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 bit patterns (round to nearest, ties to even)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _as_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    if dtype == "f32":
        return a
    raise ValueError(dtype)


def as_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 image of a generated tensor (what the oracle consumes)."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def _recv_sigma(w: Workload, i: int) -> float:
    if w.recv_rule == "unit":
        return w.sigma_a
    return w.sigma_a * w.sigma_w * float(np.sqrt(w.k * max(i, 1)))


def make_rs(w: Workload, salt: int = 0) -> dict:
    """Inputs of one GEMM + reduce-scatter rank step: ``A[p*m_chunk x k]``, ``W[k x n]``
    in ``w.dtype``; ``R[i]`` (i = 1..p-1) fp32 partial sums as rank r-1 would deliver."""
    assert w.kind == "rs"
    A = _as_dtype(normal_f32(_rng(w, 0, salt), (w.p * w.m_chunk, w.k), w.sigma_a), w.dtype)
    W = _as_dtype(normal_f32(_rng(w, 1, salt), (w.k, w.n), w.sigma_w), w.dtype)
    R: List[Optional[np.ndarray]] = [None]
    for i in range(1, w.p):
        R.append(normal_f32(_rng(w, 1 + i, salt), (w.m_chunk, w.n), _recv_sigma(w, i)))
    return {"A": A, "W": W, "R": R}


def make_ag(w: Workload, salt: int = 0) -> dict:
    """Inputs of one all-gather + GEMM rank step: own slice ``X[m_chunk x k]``, ``W[k x n]``,
    ``S[i]`` (i = 1..p-1) the slices that arrive in ring order."""
    assert w.kind == "ag"
    X = _as_dtype(normal_f32(_rng(w, 0, salt), (w.m_chunk, w.k), w.sigma_a), w.dtype)
    W = _as_dtype(normal_f32(_rng(w, 1, salt), (w.k, w.n), w.sigma_w), w.dtype)
    S: List[Optional[np.ndarray]] = [None]
    for i in range(1, w.p):
        S.append(_as_dtype(normal_f32(_rng(w, 1 + i, salt), (w.m_chunk, w.k), w.sigma_a), w.dtype))
    return {"X": X, "W": W, "S": S}


def make_dp(w: Workload, salt: int = 0) -> dict:
    """Inputs of the gradient path: local bucket of ``p*m_chunk`` fp32 values and
    ``R[i]`` (i = 1..p-1), each ``m_chunk`` values."""
    assert w.kind == "dp"
    g = normal_f32(_rng(w, 0, salt), (w.p * w.m_chunk,), w.sigma_a)
    R: List[Optional[np.ndarray]] = [None]
    for i in range(1, w.p):
        R.append(normal_f32(_rng(w, i, salt), (w.m_chunk,), w.sigma_a))
    return {"bucket": g, "R": R}


def small_int_like(a_shape, rng: np.random.Generator, lo: int = -3, hi: int = 3) -> np.ndarray:
    """Small-integer-valued float32 data: every product and partial sum is exact in
    bf16 x bf16 -> fp32, so results can be compared bit for bit."""
    return rng.integers(lo, hi + 1, size=a_shape).astype(np.float32)
