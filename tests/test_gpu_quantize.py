"""GPU parity of the quantizer (Alg. 1 search, Eq. 4 scale refit, Code Cluster map of Sec. 3.3 / Eq. 1) through the C ABI:
codes, fp16 scales and the per-channel alpha / beta must equal the oracle's bit for bit (the oracle's canonical arrays
are put into device order by the library's own pack routines), on Gaussian weights, heavy-tailed weights, all-zero rows
and groups, and values that produce exact ties."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FMT = {"narrow": (b.NARROW, o.F2), "wide": (b.WIDE, o.F275)}


def _weights(kind: str, N: int, K: int, seed: int) -> np.ndarray:
    rng = synth.rng(30, seed)
    if kind == "normal":
        return synth.weights_normal(N, K, rng)
    if kind == "heavy":                                   # outliers decide the group scale
        W = synth.weights_normal(N, K, rng)
        W[rng.random((N, K)) < 0.01] *= 12.0
        return W.astype(np.float32)
    if kind == "zeros":                                   # all-zero rows and groups among ordinary ones
        W = synth.weights_normal(N, K, rng)
        W[1] = 0.0
        W[3, 64:192] = 0.0
        W[N - 1, K - 64:] = 0.0
        return W
    if kind == "ties":                                    # few distinct values on a dyadic grid: many exact ties
        return (rng.integers(-8, 9, size=(N, K)) / 64.0).astype(np.float32)
    raise ValueError(kind)


def _compare(fmt_name, W):
    bfmt, ofmt = FMT[fmt_name]
    N, K = W.shape
    codes, scales, alpha, beta = o.quantize(W, ofmt)
    d = b.descriptor(K, N, [bfmt])
    want_codes = b.pack_codes(d, codes)
    want_scales = b.pack_scales(d, scales)
    got = b.quantize(torch.from_numpy(W).to(DEV), bfmt)
    torch.cuda.synchronize()
    g_codes = got.codes.cpu().numpy().reshape(-1)
    g_scales = got.scales.cpu().numpy().view(np.uint16).reshape(-1)
    if fmt_name == "narrow":
        assert np.array_equal(got.alpha.cpu().numpy().reshape(-1), alpha), "alpha differs"
        assert np.array_equal(got.beta.cpu().numpy().reshape(-1), beta), "beta differs"
    bad = np.flatnonzero(g_codes != want_codes)
    assert bad.size == 0, f"{bad.size} code bytes differ, first at {bad[:5]}"
    assert np.array_equal(g_scales, want_scales), "scales differ"
    return got, (codes, scales, alpha, beta)


@pytest.mark.parametrize("fmt_name", ["narrow", "wide"])
@pytest.mark.parametrize("kind", ["normal", "heavy", "zeros", "ties"])
def test_quantizer_matches_the_oracle(fmt_name, kind):
    K = 512 if fmt_name == "wide" else 256
    _compare(fmt_name, _weights(kind, 48, K, 1))


@pytest.mark.parametrize("fmt_name,N,K", [("narrow", 16, 1024), ("narrow", 208, 768), ("wide", 16, 1024), ("wide", 80, 1536)])
def test_shapes_and_row_stride(fmt_name, N, K):
    W = _weights("normal", N, K, 2)
    got, _ = _compare(fmt_name, W)
    # a strided source (ldw > K) gives the same result
    bfmt = FMT[fmt_name][0]
    big = torch.zeros((N, K + 64), dtype=torch.float32, device=DEV)
    big[:, :K] = torch.from_numpy(W).to(DEV)
    again = b.quantize(big[:, :K], bfmt)
    torch.cuda.synchronize()
    assert torch.equal(again.codes, got.codes) and torch.equal(again.scales, got.scales)


def test_quantize_then_multiply():
    """The quantizer's output is what ccq_gemm reads: quantize on the GPU, multiply on the GPU, compare with the oracle's
    product over the oracle's own encoding of the same matrix."""
    N, K, M = 256, 1024, 5
    W = _weights("normal", N, K, 3)
    got, (codes, scales, alpha, beta) = _compare("narrow", W)
    x = synth.activations_bf16(M, K, synth.rng(30, 9))
    y = b.gemm(got, b.bf16_tensor(x, DEV))
    torch.cuda.synchronize()
    Wd = o.decode(K, N, o.F2, codes, scales, alpha, beta)
    assert_gemm_close(b.bf16_bits(y), o.matmul(x, Wd), "quantize -> gemm")
    assert np.linalg.norm(Wd - W) / np.linalg.norm(W) < 0.45         # 2 bits per weight on Gaussian weights


@pytest.mark.parametrize("fmt_name", ["narrow", "wide"])
@pytest.mark.parametrize("kind", ["normal", "heavy", "zeros", "ties"])
def test_compressed_scales_match_the_oracle(fmt_name, kind):
    """scale_mode 1 (Sec. 3.4): quantize, then channel-wise super scale, 4-bit fields and one more search with the scale
    that is stored; codes (with the wide format's fields inside), packed narrow fields, super scales, alpha and beta."""
    bfmt, ofmt = FMT[fmt_name]
    N, K = 48, (512 if fmt_name == "wide" else 256)
    W = _weights(kind, N, K, 5)
    codes, scales, alpha, beta = o.quantize(W, ofmt)
    c2, sq, ssup = o.compress_scales(W, ofmt, codes, scales, alpha, beta)
    d = b.descriptor(K, N, [bfmt], scale_mode=1)
    got = b.quantize(torch.from_numpy(W).to(DEV), bfmt, scale_mode=1)
    torch.cuda.synchronize()
    assert np.array_equal(got.ssup.cpu().numpy().view(np.uint16).reshape(-1), ssup), "super scales differ"
    bad = np.flatnonzero(got.codes.cpu().numpy().reshape(-1) != b.pack_codes(d, c2))
    assert bad.size == 0, f"{bad.size} code bytes differ, first at {bad[:5]}"
    if fmt_name == "narrow":
        assert np.array_equal(got.scales.cpu().numpy().view(np.uint16).reshape(-1), b.pack_scales4(d, sq)), "scale fields differ"
        assert np.array_equal(got.alpha.cpu().numpy().reshape(-1), alpha) and np.array_equal(got.beta.cpu().numpy().reshape(-1), beta)
    else:
        assert got.scales is None
    # and the result multiplies: against the oracle's decode of its own compressed encoding
    x = synth.activations_bf16(3, K, synth.rng(30, 77))
    y = b.gemm(got, b.bf16_tensor(x, DEV))
    torch.cuda.synchronize()
    Wd = o.decode_cs(K, N, ofmt, c2, sq, ssup, alpha, beta)
    assert_gemm_close(b.bf16_bits(y), o.matmul(x, Wd), "quantize (compressed scales) -> gemm")


@pytest.mark.parametrize("kind", ["normal", "heavy", "zeros", "ties"])
@pytest.mark.parametrize("mode", [0, 1])
def test_hybrid_word_matches_the_oracle(kind, mode):
    """The hybrid 16-bit word (Sec. 3.2): two independent searches per word, fp16 scales or the 13-bit field of Sec. 3.4."""
    N, K = 32, 512
    W = _weights(kind, N, K, 6)
    codes, scales = o.h16_quantize(W)
    ssup = None
    if mode == 1:
        codes, ssup = o.h16_compress_scales(W, codes, scales)
    d = b.descriptor(K, N, b.H16, scale_mode=mode)
    got = b.quantize(torch.from_numpy(W).to(DEV), b.H16, scale_mode=mode)
    torch.cuda.synchronize()
    bad = np.flatnonzero(got.codes.cpu().numpy().reshape(-1) != b.pack_codes(d, codes))
    assert bad.size == 0, f"{bad.size} code bytes differ, first at {bad[:5]}"
    if mode == 0:
        assert np.array_equal(got.scales.cpu().numpy().view(np.uint16).reshape(-1), b.pack_scales(d, scales)), "scales differ"
        Wd = o.h16_decode(K, N, codes, scales)
    else:
        assert np.array_equal(got.ssup.cpu().numpy().view(np.uint16).reshape(-1), ssup), "super scales differ"
        Wd = o.h16_decode_cs(K, N, codes, ssup)
    x = synth.activations_bf16(2, K, synth.rng(30, 78))
    y = b.gemm(got, b.bf16_tensor(x, DEV))
    torch.cuda.synchronize()
    assert_gemm_close(b.bf16_bits(y), o.matmul(x, Wd), "quantize (hybrid word) -> gemm")


@pytest.mark.parametrize("mode", [0, 1])
def test_mixed_formats_match_the_oracle(mode):
    """A per-group mix of the narrow and wide formats (group_fmt shared by all rows): the Code Cluster map is fitted to the
    narrow groups' codes only, the super scale to all groups of the row."""
    N, K = 32, 2048
    G = K // 64
    gf = synth.group_format_map(G, 8, synth.rng(30, 50))
    W = _weights("heavy", N, K, 7)
    W[2, 64 * int(np.flatnonzero(gf == 1)[0]):][:64] = 0.0          # an all-zero wide group
    fmt = (o.F2, o.F275)
    codes, scales, alpha, beta = o.quantize(W, fmt, gf)
    d = b.descriptor(K, N, [b.NARROW, b.WIDE], gf, scale_mode=mode)
    got = b.quantize(torch.from_numpy(W).to(DEV), [b.NARROW, b.WIDE], scale_mode=mode, group_fmt=gf)
    torch.cuda.synchronize()
    if mode == 0:
        want_codes, want_scales = b.pack_codes(d, codes), b.pack_scales(d, scales)
        Wd = o.decode(K, N, fmt, codes, scales, alpha, beta, gf)
    else:
        c2, sq, ssup = o.compress_scales(W, fmt, codes, scales, alpha, beta, gf)
        want_codes, want_scales = b.pack_codes(d, c2), b.pack_scales4(d, sq)
        assert np.array_equal(got.ssup.cpu().numpy().view(np.uint16).reshape(-1), ssup), "super scales differ"
        Wd = o.decode_cs(K, N, fmt, c2, sq, ssup, alpha, beta, gf)
    bad = np.flatnonzero(got.codes.cpu().numpy().reshape(-1) != want_codes)
    assert bad.size == 0, f"{bad.size} code bytes differ, first at {bad[:5]}"
    assert np.array_equal(got.scales.cpu().numpy().view(np.uint16).reshape(-1), want_scales), "scales differ"
    assert np.array_equal(got.alpha.cpu().numpy().reshape(-1), alpha) and np.array_equal(got.beta.cpu().numpy().reshape(-1), beta)
    x = synth.activations_bf16(2, K, synth.rng(30, 79))
    y = b.gemm(got, b.bf16_tensor(x, DEV))
    torch.cuda.synchronize()
    assert_gemm_close(b.bf16_bits(y), o.matmul(x, Wd), "quantize (mixed formats) -> gemm")


def test_full_size_sampled_rows():
    """The 8192 x 8192 matrix of the benchmark: every row is independent of the others (scales per group, alpha / beta per
    row), so the oracle encodes a sample of rows and those are compared bit for bit, read out of the device layout
    (narrow k-tile: byte 4 kq + b of group j of the tile at (kq * 16 + row) * 16 + 4 j + b)."""
    K = N = 8192
    W = synth.weights_normal(N, K, synth.rng(30, 40))
    got = b.quantize(torch.from_numpy(W).to(DEV), b.NARROW)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 15, 16, 17, 4095, 4096, 8176, 8191] + synth.rng(30, 41).integers(0, N, 7).tolist())
    codes, scales, alpha, beta = o.quantize(W[rows], o.F2)
    dev_codes = got.codes.cpu().numpy().reshape(-1)
    dev_scales = got.scales.cpu().numpy().view(np.uint16).reshape(-1)
    G = K // 64
    g, j = np.meshgrid(np.arange(G), np.arange(16), indexing="ij")
    for i, n in enumerate(rows):
        off = (n // 16) * got.info.row_tile_bytes + (g // 4) * 1024 + ((j // 4) * 16 + n % 16) * 16 + (g % 4) * 4 + j % 4
        assert np.array_equal(dev_codes[off].reshape(-1), codes[i]), f"row {n}: codes differ"
        soff = (n // 16) * (G // 4) * 64 + (np.arange(G) // 4) * 64 + (n % 16) * 4 + np.arange(G) % 4
        assert np.array_equal(dev_scales[soff], scales[i]), f"row {n}: scales differ"
    assert np.array_equal(got.alpha.cpu().numpy().reshape(-1)[rows], alpha) and np.array_equal(got.beta.cpu().numpy().reshape(-1)[rows], beta)


def test_rejections_need_no_kernel():
    lib = b.load()
    assert lib.ccq_quantize_workspace_bytes(b.ctypes.byref(b.descriptor(512 + 32, 16, [b.NARROW]))) == -1            # K not a whole number of groups
    assert lib.ccq_quantize_workspace_bytes(b.ctypes.byref(b.descriptor(512 + 64, 16, [b.NARROW]))) == (16 * 9 * 16 + 16 * 9) * 2   # a ragged k-tile: real groups only
    assert lib.ccq_quantize_workspace_bytes(b.ctypes.byref(b.descriptor(512, 16, b.H16))) == 0                       # hybrid word: no workspace
    d = b.descriptor(512, 16, [b.NARROW])
    assert lib.ccq_quantize_workspace_bytes(b.ctypes.byref(d)) == (16 * 8 * 16 + 16 * 8) * 2
    d1 = b.descriptor(512, 16, [b.NARROW], scale_mode=1)
    assert lib.ccq_quantize_workspace_bytes(b.ctypes.byref(d1)) == (16 * 8 * 16 + 16 * 8) * 2 + 16 * 8 * 2 + 16 * 8
    assert lib.ccq_quantize(b.ctypes.byref(d), None, 512, None, None, None, None, None, None, 0, None) == -1
