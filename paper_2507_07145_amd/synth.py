"""Seeded synthetic inputs shared by the tests, the smoke check and bench.py.

This module holds none of the method's arithmetic: it only draws random
numbers (numpy PCG64) and formats them (fp32 -> bf16 / fp16 bit patterns).
Both the CPU oracle and the GPU library are handed the arrays made here.

The recipes mirror the operator benchmarks of the paper's "Inference
Performance" section (no dataset is involved there): Gaussian weights and
activations, random code bitstreams (every bit pattern is decodable because the
decode is a lookup-free linear map), fp16 group scales, per-channel code-cluster
parameters and a uniform top-k routing table for the grouped GEMM.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 250707145


def rng(config: int, stream: int = 0) -> np.random.Generator:
    """One independent generator per (config index, tensor stream)."""
    return np.random.Generator(np.random.PCG64([BASE_SEED + config, stream]))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def weights_normal(N: int, K: int, g: np.random.Generator, std: float = 0.02) -> np.ndarray:
    return (g.standard_normal((N, K), dtype=np.float32) * np.float32(std)).astype(np.float32)


def activations_bf16(M: int, K: int, g: np.random.Generator) -> np.ndarray:
    """N(0,1) activations as bf16 bit patterns [M][K]."""
    return f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))


def one_hot_bf16(ks, K: int) -> np.ndarray:
    """Row i is the unit vector e_{ks[i]} in bf16 (1.0 = 0x3F80)."""
    x = np.zeros((len(ks), K), dtype=np.uint16)
    for i, k in enumerate(ks):
        x[i, int(k)] = 0x3F80
    return x


def random_codes(N: int, row_bytes: int, g: np.random.Generator) -> np.ndarray:
    return g.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)


def scales_log_uniform_fp16(N: int, G: int, g: np.random.Generator, lo: float = 1e-3, hi: float = 1e-1) -> np.ndarray:
    """fp16 bit patterns, log-uniform in [lo, hi]."""
    s = np.exp(g.uniform(np.log(lo), np.log(hi), size=(N, G))).astype(np.float16)
    return s.view(np.uint16)


def cluster_params(N: int, g: np.random.Generator, code_bits: int = 15):
    """Per-output-channel code scale alpha ~ U(64,128) and integer code
    zero-point beta with 255*alpha + beta < 2^code_bits."""
    alpha = g.uniform(64.0, 128.0, size=N).astype(np.float32)
    top = float(2 ** code_bits - 1)
    room = top - 255.0 * alpha.astype(np.float64) - 1.0
    beta = np.floor(g.uniform(0.0, 1.0, size=N) * np.maximum(room, 0.0)).astype(np.float32)
    return alpha, beta


def group_format_map(G: int, n_wide: int, g: np.random.Generator) -> np.ndarray:
    """uint8[G] with exactly n_wide entries equal to 1 (wide format)."""
    m = np.zeros(G, dtype=np.uint8)
    m[g.choice(G, size=n_wide, replace=False)] = 1
    return m


def routing_topk(tokens: int, experts: int, topk: int, g: np.random.Generator):
    """Per token `topk` distinct experts, uniformly without replacement.
    Returns (sorted_rows int32 [tokens*topk], expert_offsets int32 [experts+1]):
    rows grouped by expert, token order kept inside an expert."""
    choice = np.stack([g.choice(experts, size=topk, replace=False) for _ in range(tokens)])
    tok = np.repeat(np.arange(tokens, dtype=np.int32), topk)
    exp = choice.reshape(-1)
    order = np.argsort(exp, kind="stable")
    sorted_rows = tok[order].astype(np.int32)
    counts = np.bincount(exp, minlength=experts)
    offsets = np.zeros(experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return sorted_rows, offsets
