"""Seeded synthetic inputs for the SALR linear layer: shapes, seeds and random tensors only.

This module serves both the CPU oracle (tests) and the HIP path (tests, bench).  It holds none of
the method's arithmetic: no masking, no bitmap work, no matmul.  It draws Gaussian tensors in fp32
with numpy's PCG64 generator, rounds them to bf16 (round-to-nearest-even) and hands back the raw
16-bit patterns as ``numpy.uint16`` arrays, which is the element type of every pointer at the
C boundary.

The shapes are Llama-shaped projection layers (weight ``W`` is ``[N=out, K=in]``), stand-ins for the
pretrained layers the paper evaluates on; weights ~ N(0, std_w), activations ~ N(0, 1), adapters
~ N(0, 0.01), several rank-r adapters concatenated along the rank dimension (paper Sec. 3.2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED_BASE = 16991_000


@dataclass(frozen=True)
class LayerConfig:
    """One synthetic layer: W [N, K], adapters of ranks ``ranks`` (R = sum), activations [M, K]."""

    name: str
    index: int                 # position in the workload list; enters the seed
    N: int                     # out features (rows of W)
    K: int                     # in features (contraction dim)
    ranks: Tuple[int, ...]     # ranks of the concatenated adapters
    Ms: Tuple[int, ...]        # batch sizes of interest
    sparsity_permille: Tuple[int, ...] = (500,)
    std_w: float = 0.02
    std_x: float = 1.0
    std_ab: float = 0.01

    @property
    def R(self) -> int:
        return int(sum(self.ranks))

    def keep(self, permille: int) -> int:
        """Entries kept per row at a sparsity given in 1/1000: K - floor(p*K), integer arithmetic."""
        return self.K - (self.K * permille) // 1000


CONFIGS: Dict[str, LayerConfig] = {
    c.name: c
    for c in [
        LayerConfig("tiny", 0, 512, 512, (8, 8), (16,)),
        LayerConfig("llama3_8b_q_proj", 1, 4096, 4096, (16, 16), (1, 4, 16)),
        LayerConfig("llama3_8b_gate_up_proj", 2, 14336, 4096, (16, 16), (2048,)),
        LayerConfig("llama3_8b_down_proj", 3, 4096, 14336, (32, 32), (1, 8, 64, 512, 4096),
                    sparsity_permille=(500, 700)),
        LayerConfig("llama3_70b_attn", 4, 8192, 8192, (32, 32), (1, 16, 4096), std_w=0.015),
        LayerConfig("llama3_70b_gate_up_proj", 5, 28672, 8192, (32, 32), (1, 16, 4096), std_w=0.015),
        LayerConfig("llama3_70b_down_proj", 6, 8192, 28672, (32, 32), (1, 16, 4096), std_w=0.015),
    ]
}

# tensor indices that enter the seed
T_W, T_X, T_A, T_B = 0, 1, 2, 3


def seed_for(config_index: int, tensor_index: int, extra: int = 0) -> int:
    return SEED_BASE + 10 * config_index + tensor_index + 1000 * extra


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the 16-bit patterns.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gaussian_bf16(shape: Sequence[int], std: float, seed: int) -> np.ndarray:
    """bf16 bit patterns of N(0, std) samples: fp32 draw, scale, round to bf16."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(size=tuple(shape), dtype=np.float32) * np.float32(std)
    return f32_to_bf16_bits(x)


def dense_weight(cfg: LayerConfig, rows: int | None = None) -> np.ndarray:
    """Unpruned W [N, K] (or its first ``rows`` rows) as bf16 bits.  Row r depends on r only through
    the stream position, so a row prefix of the full matrix is what ``rows`` returns."""
    n = cfg.N if rows is None else int(rows)
    rng = np.random.default_rng(seed_for(cfg.index, T_W))
    out = np.empty((n, cfg.K), dtype=np.uint16)
    step = max(1, (1 << 24) // cfg.K)
    for r0 in range(0, n, step):
        r1 = min(n, r0 + step)
        blk = rng.standard_normal(size=(r1 - r0, cfg.K), dtype=np.float32) * np.float32(cfg.std_w)
        out[r0:r1] = f32_to_bf16_bits(blk)
    return out


def activations(cfg: LayerConfig, M: int, extra: int = 0) -> np.ndarray:
    return gaussian_bf16((M, cfg.K), cfg.std_x, seed_for(cfg.index, T_X, extra))


def adapters(cfg: LayerConfig, std: float | None = None) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """The separate adapters (A_i [K, r_i], B_i [r_i, N]) as bf16 bits, one pair per rank entry."""
    s = cfg.std_ab if std is None else std
    As, Bs = [], []
    for i, r in enumerate(cfg.ranks):
        As.append(gaussian_bf16((cfg.K, r), s, seed_for(cfg.index, T_A, extra=i)))
        Bs.append(gaussian_bf16((r, cfg.N), s, seed_for(cfg.index, T_B, extra=i)))
    return As, Bs


def concat_adapters(As: Sequence[np.ndarray], Bs: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Stack along the rank dimension: A_cat [K, R] = [A_1 ... A_n], B_cat [R, N] = [B_1; ...; B_n].
    Pure data movement (paper Sec. 3.2 defines the stacking)."""
    return (np.ascontiguousarray(np.concatenate(list(As), axis=1)),
            np.ascontiguousarray(np.concatenate(list(Bs), axis=0)))


def algorithmic_bytes(M: int, K: int, N: int, R: int, nnz: int) -> int:
    """Bytes one call of the linear must move: bitmap + packed values + row offsets + X + A_cat +
    B_cat + Y (bf16 tensors, 1 bit per weight element, 4 B per row offset)."""
    return (N * K) // 8 + 2 * nnz + 4 * (N + 1) + 2 * M * K + 2 * K * R + 2 * R * N + 2 * M * N


def algorithmic_flops(M: int, K: int, N: int, R: int) -> int:
    """Flops the method executes: the decoded weight is multiplied densely (zeros included)."""
    return 2 * M * N * K + 2 * M * R * (K + N)
