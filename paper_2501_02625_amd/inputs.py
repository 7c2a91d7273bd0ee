"""Seeded synthetic inputs for the HALO linear layer.

This module only *draws data*.  It holds none of the method's arithmetic (no
Hadamard transform, no quantizer, no GEMM) and is the one piece of code that
both the CPU oracle's tests and the HIP path's tests/bench may import.

The tensors stand in for the paper's Llama-3-8B fine-tuning tensors (Section 4,
"Speedup Analysis": linear layers of size 4096 x 4096, sequence length 512,
tokens = batch x 512).  Their value structure follows what the paper says about
the real ones:

* activations X: a few channels (columns) are far larger than the rest
  (Section 3.2, Step 1) -> N(0,1) with a small fraction of columns scaled x50;
* weights W: small, well behaved -> N(0, 0.02^2);
* output gradients E: heavy tailed, with outliers running along rows/tokens
  (Section 3.2, Step 3) -> Student-t with 3 degrees of freedom, scaled by 1e-3.

All tensors are returned as bf16 *bit patterns* (numpy uint16, row-major),
because bf16 is the storage type of the layer's inputs (Section 4: the model
outside the linear layers stays in BF16).  Rounding to bf16 is round-to-nearest
-even, done here with integer arithmetic on the fp32 bit pattern.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

__all__ = [
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "outlier_columns",
    "make_activations",
    "make_weights",
    "make_errors",
    "make_adapters",
    "LinearShape",
    "LayerConfig",
    "CONFIGS",
    "make_linear_inputs",
]

OUTLIER_GAIN = 50.0
WEIGHT_STD = 0.02
ERROR_SCALE = 1e-3
ERROR_DOF = 3


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (ties to even); return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    # One counter-based generator per (seed, tensor-kind) pair.
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def outlier_columns(cols: int, frac: float, seed: int) -> np.ndarray:
    """Indices of the outlier channels: max(1, round(frac*cols)) distinct columns."""
    if frac <= 0.0:
        return np.zeros((0,), dtype=np.int64)
    count = max(1, int(round(frac * cols)))
    perm = _rng(seed, 100).permutation(cols)
    return np.sort(perm[:count]).astype(np.int64)


def make_activations(rows: int, cols: int, outlier_frac: float, seed: int) -> np.ndarray:
    """X ~ N(0,1) with outlier columns x50, as bf16 bits [rows, cols]."""
    x = _rng(seed, 0).standard_normal((rows, cols), dtype=np.float32)
    idx = outlier_columns(cols, outlier_frac, seed)
    if idx.size:
        x[:, idx] *= np.float32(OUTLIER_GAIN)
    return f32_to_bf16_bits(x)


def make_weights(rows: int, cols: int, seed: int) -> np.ndarray:
    """W ~ N(0, 0.02^2) as bf16 bits [rows, cols] (rows = out-features n, cols = in-features m)."""
    w = _rng(seed, 1).standard_normal((rows, cols), dtype=np.float32)
    w *= np.float32(WEIGHT_STD)
    return f32_to_bf16_bits(w)


def make_errors(rows: int, cols: int, seed: int) -> np.ndarray:
    """E ~ 1e-3 * Student-t(3) as bf16 bits [rows, cols] (rows = tokens b, cols = out-features n)."""
    # t_3 = Z / sqrt(chi2_3 / 3), drawn in fp32 blocks to bound memory.
    g = _rng(seed, 2)
    out = np.empty((rows, cols), dtype=np.uint16)
    step = max(1, (1 << 22) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        z = g.standard_normal((r1 - r0, cols), dtype=np.float32)
        c = g.standard_normal((ERROR_DOF, r1 - r0, cols), dtype=np.float32)
        denom = np.sqrt((c * c).sum(axis=0) / np.float32(ERROR_DOF))
        out[r0:r1] = f32_to_bf16_bits(z / denom * np.float32(ERROR_SCALE))
    return out


ADAPTER_V_STD = 0.01


def make_adapters(rank: int, n: int, m: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """LoRA adapters of a linear with W [n, m], as bf16 bits: U [rank, m] and V [n, rank]  (Y = X W^T + (X U^T) V^T).

    U is drawn as LoRA initialises its down-projection, uniform in +-1/sqrt(m).  V starts at zero in LoRA; a few
    steps into fine-tuning it is small and dense, which is what is drawn here: N(0, 0.01^2).
    """
    g = _rng(seed, 3)
    bound = np.float32(1.0 / np.sqrt(float(m)))
    u = (g.random((rank, m), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)) * bound
    v = g.standard_normal((n, rank), dtype=np.float32) * np.float32(ADAPTER_V_STD)
    return f32_to_bf16_bits(u), f32_to_bf16_bits(v)


@dataclass(frozen=True)
class LinearShape:
    """One linear layer: W is [n, m]; it maps b x m inputs to b x n outputs."""
    name: str
    n: int
    m: int
    shares_input_with: str = ""   # name of an earlier linear whose X it reuses


@dataclass(frozen=True)
class LayerConfig:
    key: str
    tokens: int                   # b
    linears: Tuple[LinearShape, ...]
    level: int                    # HALO level 0/1/2
    outlier_frac: float
    backward: bool
    seed: int = 0
    kronecker: bool = False       # in-feature widths of the form 2^n * 28 get one block of the whole width
    per_tensor: bool = False      # one scale per tensor (the paper's own quantiser) instead of one per row
    peft_rank: int = 0            # > 0: HALO-PEFT, frozen quantised weight + LoRA adapters of this rank

    def had_block_m(self, m: int) -> int:
        """Right-hand Hadamard block: the largest power of two dividing m, at most 4096 (block-diagonal when that is
        not m itself); with `kronecker`, the whole of m when m = 2^n * 28 with 64 <= 2^n <= 512."""
        if self.kronecker and m % 28 == 0:
            p = m // 28
            if p & (p - 1) == 0 and 64 <= p <= 512:
                return m
        return min(m & -m, 4096)

    def had_block_b(self) -> int:
        """Left-hand Hadamard block over tokens: largest power of two dividing b."""
        return self.tokens & -self.tokens

    def gemm_ops(self) -> int:
        per = 2 * self.tokens * sum(l.n * l.m for l in self.linears)
        if self.peft_rank:
            # F and E on the frozen weight (no G), plus the six low-rank products of the adapters
            return per * 2 + 6 * self.tokens * self.peft_rank * sum(l.n + l.m for l in self.linears)
        return per * (3 if self.backward else 1)


CONFIGS: Dict[str, LayerConfig] = {
    # Small forward-only case (shape of the paper's outlier figure: 128 tokens x 512 channels).
    "c1": LayerConfig("c1", 128, (LinearShape("proj", 512, 512),), level=1,
                      outlier_frac=0.005, backward=False),
    # Llama-3-8B attention projection, batch 4 x seq 512, HALO-1.
    "c2": LayerConfig("c2", 2048, (LinearShape("proj", 4096, 4096),), level=1,
                      outlier_frac=0.001, backward=True),
    # Llama-3-8B MLP down projection, K = 14336 = 7 x 2048, HALO-2.
    "c3": LayerConfig("c3", 4096, (LinearShape("down", 4096, 14336),), level=2,
                      outlier_frac=0.001, backward=True),
    # All seven linears of one Llama-3-8B decoder layer, HALO-2.
    "c4": LayerConfig("c4", 8192, (
        LinearShape("q", 4096, 4096),
        LinearShape("k", 1024, 4096, shares_input_with="q"),
        LinearShape("v", 1024, 4096, shares_input_with="q"),
        LinearShape("o", 4096, 4096),
        LinearShape("gate", 14336, 4096),
        LinearShape("up", 14336, 4096, shares_input_with="gate"),
        LinearShape("down", 4096, 14336),
    ), level=2, outlier_frac=0.001, backward=True),
    # MXFP6 variant: 8192 x 4096 . 4096 x 4096, FP6 E3M2 with an E8M0 scale per 32 along K after the rotation, forward product.
    "c5": LayerConfig("c5", 8192, (LinearShape("proj", 4096, 4096),), level=1,
                      outlier_frac=0.001, backward=False, seed=5),
    # The shape of c3 with the paper's Kronecker rotation H_512 (x) H_28 over K = 14336 in place of the block-diagonal one.
    "c6": LayerConfig("c6", 4096, (LinearShape("down", 4096, 14336),), level=2,
                      outlier_frac=0.001, backward=True, seed=6, kronecker=True),
    # The shape of c2 with the paper's own quantiser: one scale per tensor.
    "c7": LayerConfig("c7", 2048, (LinearShape("proj", 4096, 4096),), level=1,
                      outlier_frac=0.001, backward=True, seed=7, per_tensor=True),
    # HALO-PEFT (Appendix "LoRA-style Linear Module and HALO for PEFT"): frozen quantised 4096 x 4096 weight, rank-16
    # adapters (the rank of the paper's PEFT table), level-2 forms of F and E, 4096 tokens.
    "c8": LayerConfig("c8", 4096, (LinearShape("proj", 4096, 4096),), level=2,
                      outlier_frac=0.001, backward=True, seed=8, peft_rank=16),
}


def make_linear_inputs(cfg: LayerConfig, which: int = 0, *, tokens: int | None = None,
                       need_error: bool | None = None) -> Dict[str, np.ndarray]:
    """bf16-bit tensors X [b,m], W [n,m] and (if the config has a backward pass) E [b,n].

    Different linears of one config use different sub-seeds so no two tensors coincide.
    """
    lin = cfg.linears[which]
    b = cfg.tokens if tokens is None else tokens
    sub = cfg.seed * 1000 + which
    out = {
        "X": make_activations(b, lin.m, cfg.outlier_frac, sub),
        "W": make_weights(lin.n, lin.m, sub),
    }
    if cfg.backward if need_error is None else need_error:
        out["E"] = make_errors(b, lin.n, sub)
    if cfg.peft_rank:
        out["U"], out["V"] = make_adapters(cfg.peft_rank, lin.n, lin.m, sub)
    return out
