"""Seeded synthetic inputs for the codebook-quantized linear layer y = x W^T.

This module only draws random tensors and names workloads.  It contains none
of the method's arithmetic, so both the CPU oracle's tests and the HIP path's
tests may import it without sharing any computation.

Canonical layouts (all row-major, contiguous):
    x          [B][K]        float16   activations, N(0, 1)
    codes      [m][N][K/v]   uint8     centroid indices, uniform on 0..255
    codebooks  [m][256][v]   float16   centroids, N(0, 0.02^2)
    scales     [N]           float16   per-output-channel scale, U[0.5, 1.5]   (g = -1)
               [N][K/g]      float16   one scale per run of g weights of a row   (g > 0)

Draw order is fixed: codes, codebooks, scales, x.  Values are drawn in float64,
rounded once to float16, and those float16 values are what every consumer sees.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np

SEED_BASE = 251217000
NUM_CENTROIDS = 256


@dataclass(frozen=True)
class Case:
    """One workload: a linear layer shape, a quantization format and a batch."""
    name: str
    cfg: int          # index of the workload family (1..5)
    K: int            # in_features
    N: int            # out_features
    v: int            # vector length
    m: int            # additive codebooks
    B: int            # batch
    seed: int
    g: int = -1       # normalisation group size along K; -1 = one scale per output row

    @property
    def J(self) -> int:
        return self.K // self.v


@dataclass
class Inputs:
    case: Case
    x: np.ndarray
    codes: np.ndarray
    codebooks: np.ndarray
    scales: np.ndarray


def _case(cfg: int, idx: int, K: int, N: int, v: int, m: int, B: int, g: int = -1) -> Case:
    tag = "" if g == -1 else f"g{g}"
    return Case(name=f"c{cfg}_{K}x{N}_v{v}m{m}{tag}_b{B}", cfg=cfg, K=K, N=N, v=v, m=m, B=B,
                seed=SEED_BASE + 100 * cfg + idx, g=g)


def workloads() -> Dict[int, List[Case]]:
    """Workload families: 1 a tiny layer, 2 Llama-3-8B shapes (v4 m1), 3 Llama-3-70B
    shapes (v8 m2), 4 a batch sweep, 5 a bit-width sweep (all with one scale per row),
    6 a sweep of the normalisation group size g at 8192->28672, 7 and 8 the 8B and 70B
    shapes in the formats the paper's latency table uses (m1v4g128, m2v8g128), 9 and 10 the
    same two decoder blocks with fused projections (QKV as one matrix, gate and up as one),
    11 the five formats of the paper's average-bits table (all close to 2 bits) at 8192->28672,
    12 and 13 the (batch, N, K) grid of the paper's appendix table of kernel latencies across
    problem sizes (batch 1, 4, 8 at nine shapes from 2048^2 to 8192->28672) for m2v8g128 and m1v4g128."""
    out: Dict[int, List[Case]] = {}
    out[1] = [_case(1, 0, 512, 512, 8, 1, 1)]
    out[2] = [_case(2, i, K, N, 4, 1, 1) for i, (K, N) in
              enumerate([(4096, 4096), (4096, 1024), (4096, 14336), (14336, 4096)])]
    out[3] = [_case(3, i, K, N, 8, 2, 1) for i, (K, N) in
              enumerate([(8192, 8192), (8192, 1024), (8192, 28672), (28672, 8192)])]
    c4 = []
    for si, (K, N) in enumerate([(4096, 14336), (14336, 4096)]):
        for bi, B in enumerate([1, 4, 8, 16, 32]):
            c4.append(_case(4, 10 * si + bi, K, N, 8, 2, B))
    out[4] = c4
    out[5] = [_case(5, i, 8192, 28672, v, m, 1) for i, (v, m) in
              enumerate([(8, 1), (8, 2), (8, 3), (4, 1)])]
    out[6] = [_case(6, i, 8192, 28672, v, m, 1, g) for i, (v, m, g) in
              enumerate([(8, 2, 128), (8, 2, 64), (8, 2, 32), (8, 2, 16), (8, 2, 8),
                         (4, 1, 128), (4, 1, 32), (4, 1, 4), (8, 1, 128), (8, 1, 16)])]
    out[7] = [_case(7, i, K, N, 4, 1, 1, 128) for i, (K, N) in
              enumerate([(4096, 4096), (4096, 1024), (4096, 14336), (14336, 4096)])]
    out[8] = [_case(8, i, K, N, 8, 2, 1, 128) for i, (K, N) in
              enumerate([(8192, 8192), (8192, 1024), (8192, 28672), (28672, 8192)])]
    out[9] = [_case(9, i, K, N, 4, 1, 1, 128) for i, (K, N) in
              enumerate([(4096, 6144), (4096, 4096), (4096, 28672), (14336, 4096)])]
    out[10] = [_case(10, i, K, N, 8, 2, 1, 128) for i, (K, N) in
               enumerate([(8192, 10240), (8192, 8192), (8192, 57344), (28672, 8192)])]
    out[11] = [_case(11, i, 8192, 28672, v, m, 1, g) for i, (v, m, g) in
               enumerate([(4, 1, -1), (8, 2, -1), (16, 4, -1), (8, 1, 16), (16, 3, 32)])]
    grid = [(2048, 2048), (2048, 8192), (8192, 2048), (4096, 4096), (4096, 14336), (14336, 4096),
            (8192, 8192), (8192, 28672), (28672, 8192)]                     # (K, N)
    for cfg, (v, m) in ((12, (8, 2)), (13, (4, 1))):
        out[cfg] = [_case(cfg, 3 * si + bi, K, N, v, m, B, 128)
                    for si, (K, N) in enumerate(grid) for bi, B in enumerate([1, 4, 8])]
    return out


def find_case(name: str) -> Case:
    for cases in workloads().values():
        for c in cases:
            if c.name == name:
                return c
    raise KeyError(name)


def custom_case(K: int, N: int, v: int, m: int, B: int, seed: int, name: str = "", g: int = -1) -> Case:
    tag = "" if g == -1 else f"g{g}"
    return Case(name=name or f"custom_{K}x{N}_v{v}m{m}{tag}_b{B}_s{seed}", cfg=0, K=K, N=N, v=v, m=m, B=B, seed=seed, g=g)


def generate(case: Case) -> Inputs:
    """Draw the tensors of one workload from its seed."""
    if case.K % case.v:
        raise ValueError("K must be a multiple of v")
    rng = np.random.default_rng(case.seed)
    codes = rng.integers(0, NUM_CENTROIDS, size=(case.m, case.N, case.J), dtype=np.uint8)
    codebooks = (rng.standard_normal((case.m, NUM_CENTROIDS, case.v)) * 0.02).astype(np.float16)
    if case.g == -1:
        scales = rng.uniform(0.5, 1.5, size=(case.N,)).astype(np.float16)
    else:
        if case.g < case.v or case.g % case.v or case.K % case.g:
            raise ValueError("g must be a multiple of v that divides K")
        scales = rng.uniform(0.5, 1.5, size=(case.N, case.K // case.g)).astype(np.float16)
    x = rng.standard_normal((case.B, case.K)).astype(np.float16)
    return Inputs(case, x, codes, codebooks, scales)


def skewed_codes(case: Case, alpha: float = 1.2) -> np.ndarray:
    """Codes with a Zipf-like usage histogram (a few centroids dominate), the
    shape trained codebooks tend to have.  Uniform codes are the adversarial
    case for data-dependent LDS gathers; this one is used to show the other end."""
    rng = np.random.default_rng(case.seed + 7)
    w = 1.0 / np.arange(1, NUM_CENTROIDS + 1) ** alpha
    w /= w.sum()
    perm = rng.permutation(NUM_CENTROIDS)
    draws = rng.choice(NUM_CENTROIDS, size=(case.m, case.N, case.J), p=w)
    return perm[draws].astype(np.uint8)
