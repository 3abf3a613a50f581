"""Shared builders for the GPU parity tests: seeded inputs (synth), the oracle's
decoded weights, and the tolerance check.  Imported by tests only."""
from __future__ import annotations

import numpy as np

from oracle import ccq_oracle as o
from paper_2507_07145_amd import synth

# GEMM tolerance (bf16 output, fp32 accumulation, against the fp64 oracle):
#   per element |y - ref| <= 1e-2 * max(|ref|, rms(ref))   and   ||y - ref|| / ||ref|| <= 1e-2.
# The error budget is the bf16 output rounding (2^-9 relative) plus fp32 accumulation noise;
# the skinny path decodes weights exactly, the prefill path also rounds them to bf16.
REL_TOL = 1e-2
# The LDS-tiled kernels (more than 16 rows) multiply bf16-rounded weights (relative error <= 2^-9 each), so an element can be off by
# 2^-9 * sum_k |x_k W_nk| whatever the size of the sum itself; with heavy-tailed group scales and a short K a
# single large term can make that exceed 1e-2 * rms.  Tests of that kernel pass the absolute sum and allow
# 2^-8 of it on top (weight rounding plus fp32 accumulation), a bound that follows from the arithmetic.
ABS_SUM_TOL = 2.0 ** -8


def canon_zero(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns with -0 mapped to +0 (the sign of an exact zero is not part of parity)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return np.where((bits & 0x7FFF) == 0, np.uint16(0), bits)


def assert_gemm_close(y_bits: np.ndarray, ref: np.ndarray, what: str = "", abs_sum: np.ndarray | None = None) -> dict:
    y = o.bf16_bits_to_f64(y_bits)
    assert y.shape == ref.shape, (what, y.shape, ref.shape)
    assert np.all(np.isfinite(y)), what
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    err = np.abs(y - ref)
    tol = REL_TOL * np.maximum(np.abs(ref), rms)
    if abs_sum is not None:
        tol = tol + ABS_SUM_TOL * abs_sum
    bad = np.argwhere(err > tol)
    assert bad.size == 0, f"{what}: {len(bad)} elements out of tolerance, first {bad[:5].tolist()}, max err {err.max():.4g}, rms {rms:.4g}"
    rel = float(np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-300))
    assert rel <= REL_TOL, f"{what}: relative L2 error {rel}"
    return {"max_abs_err": float(err.max()) if err.size else 0.0, "rel_l2": rel}


class Case:
    """Canonical arrays of one quantized matrix plus lazily decoded oracle weights."""

    def __init__(self, K, N, kinds, codes, scales, alpha=None, beta=None, group_fmt=None):
        self.K, self.N, self.kinds = K, N, kinds
        self.codes, self.scales, self.alpha, self.beta, self.group_fmt = codes, scales, alpha, beta, group_fmt
        self._W = None

    @property
    def oracle_fmt(self):
        m = {"narrow": o.F2, "wide": o.F275}
        return m[self.kinds[0]] if len(self.kinds) == 1 else (m[self.kinds[0]], m[self.kinds[1]])

    def W(self, rows=None) -> np.ndarray:
        """Oracle-decoded weights fp64 [N][K] (or the given rows only)."""
        if rows is None:
            if self._W is None:
                self._W = o.decode(self.K, self.N, self.oracle_fmt, self.codes, self.scales, self.alpha, self.beta, self.group_fmt)
            return self._W
        rows = np.asarray(rows)
        a = None if self.alpha is None else self.alpha[rows]
        b = None if self.beta is None else self.beta[rows]
        return o.decode(self.K, len(rows), self.oracle_fmt, self.codes[rows], self.scales[rows], a, b, self.group_fmt)

    def device_weight(self, device="cuda:0"):
        from paper_2507_07145_amd import binding
        m = {"narrow": binding.NARROW, "wide": binding.WIDE}
        return binding.Weight.from_canonical(self.K, self.N, [m[k] for k in self.kinds], self.codes, self.scales, self.alpha, self.beta,
                                             self.group_fmt, device=device)


def random_case(K, N, kinds, seed_cfg, stream0=0, n_wide=None) -> Case:
    """Random code bitstream (every pattern is decodable), log-uniform fp16 scales, random cluster parameters."""
    G = K // 64
    group_fmt = None
    if len(kinds) == 2:
        group_fmt = synth.group_format_map(G, n_wide, synth.rng(seed_cfg, stream0 + 4))
        fm = (o.F2, o.F275) if kinds[0] == "narrow" else (o.F275, o.F2)
        rb = o.row_bytes(K, fm, group_fmt)
    else:
        rb = o.row_bytes(K, o.F2 if kinds[0] == "narrow" else o.F275)
    codes = synth.random_codes(N, rb, synth.rng(seed_cfg, stream0))
    scales = synth.scales_log_uniform_fp16(N, G, synth.rng(seed_cfg, stream0 + 1))
    alpha = beta = None
    if "narrow" in kinds:
        alpha, beta = synth.cluster_params(N, synth.rng(seed_cfg, stream0 + 2))
    return Case(K, N, kinds, codes, scales, alpha, beta, group_fmt)


def encoded_case(K, N, seed_cfg, kind="narrow") -> Case:
    """N(0, 0.02) weights quantized by the oracle's encoder (Alg. 1 + Code Cluster + Eq. 4)."""
    W = synth.weights_normal(N, K, synth.rng(seed_cfg, 0))
    fmt = o.F2 if kind == "narrow" else o.F275
    codes, scales, alpha, beta = o.quantize(W, fmt)
    if kind != "narrow":
        alpha = beta = None
    return Case(K, N, [kind], codes, scales, alpha, beta)
