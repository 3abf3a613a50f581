"""GPU parity on the method's edge cases, through every kernel the row count selects:

* weight zero-points at the ends of and off the integer grid of what the ABI accepts (Alg. 2 / Alg. 3, `zp`);
* Code Cluster parameters that put q * alpha + beta on .5 ties, at 0 and at 2^15 - 1 (Alg. 3's round, Eq. 1);
* group scales 0, fp16 subnormal and 65504, super scales and fields at their ends (Sec. 3.4);
* activations with -0, subnormal and large magnitudes.

Decoded weights are compared bit for bit through one-hot activations, products within the plain tolerance."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close, canon_zero
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# row counts that reach, on narrow-format weights: the one-row kernel, the 2-4-row kernel, the per-row-tile kernel,
# the per-group-tile kernel, the 64-row kernel (register decode) -- and on the wide format the corresponding ones
ROWS = (1, 3, 16, 24, 64, 130)


def _bits(w, x_bits):
    y = b.gemm(w, b.bf16_tensor(x_bits, DEV))
    torch.cuda.synchronize()
    return b.bf16_bits(y)


def _decode_through_every_kernel(w, W, K, rows=ROWS, seed=0):
    """One-hot rows: y[m] must be bf16(W[:, k_m]) exactly, whatever kernel M rows select."""
    for M in rows:
        ks = synth.rng(77, 1000 * seed + M).integers(0, K, M)
        ks[:min(M, 4)] = [0, K - 1, 63, 64][:min(M, 4)]
        got = _bits(w, synth.one_hot_bf16(ks, K))
        want = o.to_bf16_bits(W[:, ks].T)
        assert np.array_equal(canon_zero(got), canon_zero(want)), f"decoded weights differ, M={M}"


def _products_through_every_kernel(w, W, K, what, rows=ROWS, seed=0):
    for M in rows:
        x = synth.activations_bf16(M, K, synth.rng(78, 1000 * seed + M))
        assert_gemm_close(_bits(w, x), o.matmul(x, W), f"{what} M={M}", rounded=(x, W) if M > 32 else None)


@pytest.mark.parametrize("kind,zp", [("narrow", 0.0), ("narrow", 7.5), ("narrow", 31.5), ("narrow", 64.0),
                                     ("wide", 0.0), ("wide", 7.5), ("wide", 31.5), ("wide", 64.0),
                                     ("h16", 0.0), ("h16", 3.5), ("h16", 64.0)])
def test_zero_points(kind, zp):
    """`zp` is an input of Alg. 2 / Alg. 3 with no value fixed: every multiple of 0.5 in [0, 64] the ABI accepts."""
    K, N = 1024, 96
    G = K // 64
    scales = synth.scales_log_uniform_fp16(N, G, synth.rng(70, 1))
    if kind == "narrow":
        codes = synth.random_codes(N, K // 4, synth.rng(70, 0))
        alpha, beta = synth.cluster_params(N, synth.rng(70, 2))
        W = o.decode(K, N, o.Code(6, 4, 3, True, zp=zp), codes, scales, alpha, beta)
        w = b.Weight.from_canonical(K, N, [b.ccq_code(6, 4, 3, 1, zp)], codes, scales, alpha, beta, device=DEV)
    elif kind == "wide":
        codes = synth.random_codes(N, G * 22, synth.rng(70, 3))
        W = o.decode(K, N, o.Code(4, 3, 2, False, zp=zp), codes, scales)
        w = b.Weight.from_canonical(K, N, [b.ccq_code(4, 3, 2, 0, zp)], codes, scales, device=DEV)
    else:
        codes = synth.random_codes(N, o.h16_row_bytes(K), synth.rng(70, 4))
        W = o.h16_decode(K, N, codes, scales, zp=zp)
        w = b.Weight.from_canonical(K, N, [b.ccq_code(3, 3, 2, 0, zp), b.ccq_code(3, 4, 2, 0, zp)], codes, scales, device=DEV)
    _decode_through_every_kernel(w, W, K, seed=int(2 * zp))
    _products_through_every_kernel(w, W, K, f"{kind} zp={zp}", seed=int(2 * zp))


def _tie_cluster_params(N):
    """(alpha, beta) pairs on the edges of Alg. 3's round: alpha = 0 (every byte decodes to beta, at both ends of the
    code range), alpha = 0.5, 1.5, 2.5 (q alpha + beta lands on .5 for every odd q: ties to even), alpha = 128, 1.5 and
    128 - 2^-9 with round(255 alpha + beta) = 2^15 - 1 or just below, and ordinary values in between."""
    edge = [(0.0, 0.0), (0.0, 32767.0), (0.5, 0.0), (0.5, 7.0), (1.5, 0.0), (1.5, 32384.0), (2.5, 1.0), (128.0, 127.0),
            (128.0, 0.0), (0.25, 3.0), (1.0, 0.0), (1.0, 32512.0), (127.998046875, 127.0), (100.37000274658203, 5.0)]
    rng = synth.rng(71, 9)
    alpha = np.empty(N, np.float32)
    beta = np.empty(N, np.float32)
    for n in range(N):
        if n % 2 == 0:
            alpha[n], beta[n] = edge[(n // 2) % len(edge)]
        else:
            a = np.float32(rng.uniform(0.0, 128.0))
            alpha[n] = a
            beta[n] = np.floor(rng.uniform(0.0, 1.0) * max(32767.0 - 255.0 * float(a) - 1.0, 0.0))
    assert np.all(np.rint(255.0 * alpha.astype(np.float64) + beta) <= 32767.0)   # the largest code stays below 2^15
    return alpha, beta


@pytest.mark.parametrize("K,N,rows", [(1024, 96, ROWS), (256, 1536, (2900,))])
def test_code_cluster_ties_and_range_ends(K, N, rows):
    """Alg. 3: w = round(q * s_code + zp_code), read as round-half-to-even of the exact value.  Every byte value occurs in
    every row; the rows' parameters sit on ties and on both ends of the 15-bit range.  The second shape runs the
    256-row kernel."""
    G = K // 64
    nb = K // 4
    if nb >= 256:     # every byte value in every row, the order shifted from row to row
        codes = synth.random_codes(N, nb, synth.rng(71, 0))
        codes[:, :256] = ((np.arange(256)[None, :] + 37 * np.arange(N)[:, None]) % 256).astype(np.uint8)
    else:             # odd and even bytes in every row
        codes = ((7 * np.arange(N)[:, None] + 5 * np.arange(nb)[None, :] + 1) % 256).astype(np.uint8)
    scales = synth.scales_log_uniform_fp16(N, G, synth.rng(71, 1))
    alpha, beta = _tie_cluster_params(N)
    W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
    w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    # all columns of the first groups (they hold every byte value when K allows) plus random ones, through every kernel
    for M in rows:
        ks = np.concatenate([np.arange(min(K, 1024)), synth.rng(71, M).integers(0, K, 64)])
        for n_chunk, i in enumerate(range(0, len(ks), M)):
            chunk = np.resize(ks[i:], M)          # a short last chunk wraps around
            got = _bits(w, synth.one_hot_bf16(chunk, K))
            want = o.to_bf16_bits(W[:, chunk].T)
            assert np.array_equal(canon_zero(got), canon_zero(want)), f"decoded weights differ, M={M}, columns {chunk[:4]}..."
            if M == 1 and n_chunk >= 300:
                break
    _products_through_every_kernel(w, W, K, "cluster ties", rows=rows, seed=5)


@pytest.mark.parametrize("kind", ["narrow", "wide"])
def test_scale_extremes(kind):
    """fp16 group scales 0, the smallest subnormal, the largest subnormal, the smallest normal and 65504, next to ordinary ones."""
    K, N = 1024, 64
    G = K // 64
    scales = synth.scales_log_uniform_fp16(N, G, synth.rng(72, 1))
    special = np.array([0x0000, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0x8000 | 0x3C00], dtype=np.uint16)   # the last: a negative scale (-1.0)
    for n in range(N):
        for j, g in enumerate(synth.rng(72, 100 + n).choice(G, size=len(special), replace=False)):
            scales[n, g] = special[(j + n) % len(special)]
    if kind == "narrow":
        codes = synth.random_codes(N, K // 4, synth.rng(72, 0))
        alpha, beta = synth.cluster_params(N, synth.rng(72, 2))
        W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
        w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    else:
        codes = synth.random_codes(N, G * 22, synth.rng(72, 3))
        W = o.decode(K, N, o.F275, codes, scales)
        w = b.Weight.from_canonical(K, N, [b.WIDE], codes, scales, device=DEV)
    # every column of the groups of row 0 that carry a special scale, then random columns
    for M in ROWS:
        ks = synth.rng(72, 200 + M).integers(0, K, M)
        got = _bits(w, synth.one_hot_bf16(ks, K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"decoded weights differ, M={M}"
    for i in range(0, K, 16):
        ks = np.arange(i, i + 16)
        got = _bits(w, synth.one_hot_bf16(ks, K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"decoded weights differ at columns {i}.."
    # products: the 65504-scale groups dominate the sums; the bound is relative to them
    _products_through_every_kernel(w, W, K, f"scale extremes {kind}", seed=9)


@pytest.mark.parametrize("kind", ["narrow", "wide", "h16"])
def test_compressed_scale_extremes(kind):
    """scale_mode 1 (Sec. 3.4): fields 0 and the largest one, super scales 0, subnormal and 65504 / field."""
    K, N = 1024, 64
    G = K // 64
    rng = synth.rng(73, 0)
    ssup = synth.scales_log_uniform_fp16(N, 1, synth.rng(73, 1), 1e-4, 1e-2).reshape(N)
    ssup[0], ssup[1], ssup[2], ssup[3] = 0x0000, 0x0001, 0x03FF, 0x5000 if kind != "h16" else 0x2000   # 0, subnormals, 32 (h16: 2^-7)
    if kind == "narrow":
        codes = synth.random_codes(N, K // 4, rng)
        sq = rng.integers(0, 256, size=(N, G // 2), dtype=np.uint8)
        sq[:, 0] = 0x0F            # group 0: field 15, group 1: field 0
        alpha, beta = synth.cluster_params(N, synth.rng(73, 2))
        W = o.decode_cs(K, N, o.F2, codes, sq, ssup, alpha, beta)
        w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=DEV)
    elif kind == "wide":
        codes = synth.random_codes(N, G * 22, rng)
        codes[:, 21] = (codes[:, 21] & 0xF0) | 0x0F      # group 0: field 15
        codes[:, 43] = codes[:, 43] & 0xF0               # group 1: field 0
        W = o.decode_cs(K, N, o.F275, codes, None, ssup)
        w = b.Weight.from_canonical_compressed(K, N, [b.WIDE], codes, None, ssup, device=DEV)
    else:
        codes = synth.random_codes(N, o.h16_row_bytes(K), rng)
        codes[:, 18] = 0xFF
        codes[:, 19] = codes[:, 19] | 0x1F               # group 0: field 8191
        codes[:, 38] = 0x00
        codes[:, 39] = codes[:, 39] & 0xE0               # group 1: field 0
        W = o.h16_decode_cs(K, N, codes, ssup)
        w = b.Weight.from_canonical_compressed(K, N, b.H16, codes, None, ssup, device=DEV)
    assert np.all(W[:, 64:128] == 0.0) and np.all(W[0] == 0.0)
    for M in ROWS:
        ks = synth.rng(73, 200 + M).integers(0, K, M)
        ks[:min(M, 3)] = [0, 63, 64][:min(M, 3)]
        got = _bits(w, synth.one_hot_bf16(ks, K))
        want = W[:, ks].T
        if kind == "h16":
            want = want.astype(np.float32).astype(np.float64)   # the kernel's precision for the 27-bit product (fp32), then bf16
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(want))), f"decoded weights differ, M={M}"
    _products_through_every_kernel(w, W, K, f"compressed scale extremes {kind}", seed=11)


def test_activation_extremes():
    """-0, bf16 subnormals and magnitudes near both ends of the fp32 range in the activations: decoded weights stay exact
    on a background of -0, products stay finite and within tolerance (the exact sums are far from overflow)."""
    K, N = 1024, 64
    codes = synth.random_codes(N, K // 4, synth.rng(74, 0))
    scales = synth.scales_log_uniform_fp16(N, K // 64, synth.rng(74, 1))
    alpha, beta = synth.cluster_params(N, synth.rng(74, 2))
    W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
    w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    for M in ROWS:
        ks = synth.rng(74, 10 + M).integers(0, K, M)
        xe = synth.one_hot_bf16(ks, K)
        xe[xe == 0] = 0x8000                                     # -0 everywhere else
        got = _bits(w, xe)
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"decode on a -0 background, M={M}"
        x = synth.activations_bf16(M, K, synth.rng(74, 50 + M))
        f = synth.bf16_bits_to_f32(x)
        for m in range(M):
            scale = [np.float32(2.0 ** 100), np.float32(2.0 ** -100), np.float32(1.0)][m % 3]
            f[m] *= scale
        xs = synth.f32_to_bf16_bits(f)
        xs[:, 5] = 0x0001                                        # smallest bf16 subnormal
        xs[:, 70] = 0x807F                                       # largest negative subnormal
        xs[:, 200] = 0x8000
        ref = o.matmul(xs, W)
        y = o.bf16_bits_to_f64(_bits(w, xs))
        assert np.all(np.isfinite(y))
        # rows differ by 2^200 in magnitude: compare row by row
        for m in range(M):
            assert_gemm_close(o.to_bf16_bits(y[m:m + 1]), ref[m:m + 1], f"activation extremes M={M} row {m}",
                              rounded=(xs[m:m + 1], W) if M > 32 else None)
