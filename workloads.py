"""Seeded synthetic inputs for the dynamic-M dense / batch_matmul / LSTM workloads.

This module is the one piece shared by the CPU oracle's tests and the HIP
path's tests and benchmark.  It holds no arithmetic of the method itself:
it only draws random numbers, rounds them once to bfloat16 (round to nearest,
ties to even) and hands back both the 16-bit patterns (what the GPU reads) and
the exactly equal float32 values (what the oracle reads).

The paper evaluates on sentences of varying length (Section 5.1); those
corpora are not available here, so uniform length draws stand in for them and
N(0, 0.02) weights stand in for trained weights.

Seeds: ``SEED_BASE + config_index`` with config_index 1..5.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Tuple

import numpy as np

SEED_BASE = 20060303100


# --------------------------------------------------------------------------
# bfloat16 <-> float32 bit handling (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    # NaN stays NaN (not produced by the generators, kept for completeness)
    nan = np.isnan(a)
    out = r.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


@dataclass
class BF16Array:
    """A tensor stored as bfloat16: ``bits`` (uint16) and the equal ``f32``."""

    bits: np.ndarray
    f32: np.ndarray

    @property
    def shape(self) -> Tuple[int, ...]:
        return self.bits.shape

    def rows(self, m: int) -> "BF16Array":
        return BF16Array(self.bits[:m], self.f32[:m])


def _as_bf16(a: np.ndarray) -> BF16Array:
    bits = f32_to_bf16_bits(a)
    return BF16Array(bits, bf16_bits_to_f32(bits))


def uniform_bf16(rng: np.random.Generator, shape) -> BF16Array:
    """uniform[-1, 1) as 2*random()-1, then rounded to bf16."""
    return _as_bf16((2.0 * rng.random(shape) - 1.0).astype(np.float32))


def normal_bf16(rng: np.random.Generator, shape, std: float = 0.02) -> BF16Array:
    """N(0, std) (std is the standard deviation), then rounded to bf16."""
    return _as_bf16(rng.normal(0.0, std, shape).astype(np.float32))


def rng_for(config_index: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([SEED_BASE + config_index, stream])


# --------------------------------------------------------------------------
# Config 1: one dynamic dense 128 -> 128, 64 calls, M ~ U{1..64}
# --------------------------------------------------------------------------
@dataclass
class DenseProblem:
    x: BF16Array  # [M, K]
    w: BF16Array  # [N, K]
    b: BF16Array  # [N]
    epilogue: str  # "bias" | "bias_gelu" | "none"

    @property
    def M(self) -> int:
        return self.x.shape[0]

    @property
    def N(self) -> int:
        return self.w.shape[0]

    @property
    def K(self) -> int:
        return self.w.shape[1]


def config1_calls(n_calls: int = 64) -> List[DenseProblem]:
    rng = rng_for(1)
    w = uniform_bf16(rng, (128, 128))
    b = uniform_bf16(rng, (128,))
    ms = rng.integers(1, 65, size=n_calls)
    return [DenseProblem(uniform_bf16(rng, (int(m), 128)), w, b, "bias") for m in ms]


# --------------------------------------------------------------------------
# Config 2: LSTM cell, dynamic batch B ~ U{1..64} per sequence, 128 steps
# --------------------------------------------------------------------------
LSTM_IX = 512
LSTM_H = 512
LSTM_STEPS = 128


@dataclass
class LSTMWeights:
    w: BF16Array  # [4H, Ix+H], gate blocks i, f, g, o
    b: BF16Array  # [4H]


def config2_weights(H: int = LSTM_H, Ix: int = LSTM_IX) -> LSTMWeights:
    rng = rng_for(2)
    return LSTMWeights(normal_bf16(rng, (4 * H, Ix + H)), normal_bf16(rng, (4 * H,)))


def config2_batches(n_seq: int = 64) -> np.ndarray:
    return rng_for(2, 1).integers(1, 65, size=n_seq)


def config2_inputs(seq: int, B: int, steps: int = LSTM_STEPS, Ix: int = LSTM_IX) -> BF16Array:
    """x_t for all steps of one sequence: [steps, B, Ix] uniform[-1,1)."""
    return uniform_bf16(rng_for(2, 100 + seq), (steps, B, Ix))


# --------------------------------------------------------------------------
# Config 3: BERT-base shaped encoder GEMMs, L ~ U{1..512}, batch 1
# --------------------------------------------------------------------------
BERT_BASE_GEMMS = (
    # name, K (in), N (out), epilogue
    ("qkv", 768, 2304, "bias"),
    ("proj", 768, 768, "bias"),
    ("ffn1", 768, 3072, "bias_gelu"),
    ("ffn2", 3072, 768, "bias"),
)


def dense_weights(config_index: int, gemm_index: int, N: int, K: int) -> Tuple[BF16Array, BF16Array]:
    rng = rng_for(config_index, 10 + gemm_index)
    return normal_bf16(rng, (N, K)), normal_bf16(rng, (N,))


def config3_lengths(n_draws: int = 100) -> np.ndarray:
    return rng_for(3, 1).integers(1, 513, size=n_draws)


def activations(config_index: int, draw: int, M: int, K: int) -> BF16Array:
    return uniform_bf16(rng_for(config_index, 1000 + draw), (M, K))


# --------------------------------------------------------------------------
# Config 4: attention batch_matmul, 12 heads x head_dim 64, L ~ U{1..512}
# --------------------------------------------------------------------------
ATT_HEADS = 12
ATT_D = 64


def config4_lengths(n_draws: int = 100) -> np.ndarray:
    return rng_for(4, 1).integers(1, 513, size=n_draws)


def config4_qkv(draw: int, L: int) -> Tuple[BF16Array, BF16Array, BF16Array]:
    rng = rng_for(4, 1000 + draw)
    shape = (ATT_HEADS, L, ATT_D)
    return uniform_bf16(rng, shape), uniform_bf16(rng, shape), uniform_bf16(rng, shape)


# --------------------------------------------------------------------------
# Config 5: BERT-large FFN at ragged token count M = sum of 32 lengths
# --------------------------------------------------------------------------
BERT_LARGE_FFN = (
    ("ffn1", 1024, 4096, "bias_gelu"),
    ("ffn2", 4096, 1024, "bias"),
)


def config5_token_counts(n_draws: int = 64) -> np.ndarray:
    lens = rng_for(5, 1).integers(1, 513, size=(n_draws, 32))
    return lens.sum(axis=1)


def residue_sweep(base: int = 2048, span: int = 256) -> Iterator[int]:
    """Deterministic M = base + r for r in 0..span-1 (every residue of every tile)."""
    return iter(range(base, base + span))
