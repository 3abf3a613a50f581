"""GPU parity for the compressed scales of Sec. 3.4 (scale_mode 1): group scale = 4-bit field * per-row fp16 super
scale (first line of Alg. 2 / Alg. 3), through every kernel the dense entry point uses.  Decoded weights bit-exact
through one-hot rows, products within the tolerance of tests/cases.py."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close, canon_zero
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FM = {"narrow": (o.F2, b.NARROW), "wide": (o.F275, b.WIDE)}


def _case(kinds, K, N, stream0, n_wide=None):
    """Random code bytes (for the wide format the spare nibbles are random scale fields), random 4-bit fields for the
    narrow groups, fp16 super scales log-uniform in [1e-4, 1e-2], random Code Cluster parameters."""
    rng = synth.rng(6, stream0)
    G = K // 64
    ofmt = FM[kinds[0]][0] if len(kinds) == 1 else (o.F2, o.F275)
    gfmts = [FM[k][1] for k in kinds]
    gf = synth.group_format_map(G, n_wide, rng) if len(kinds) == 2 else None
    codes = synth.random_codes(N, o.row_bytes(K, ofmt, gf), rng)
    nb = o.sq_row_bytes(K, ofmt, gf)
    sq = rng.integers(0, 256, size=(N, max(nb, 1)), dtype=np.uint8)[:, :nb]
    ssup = synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)
    ssup = (o.fp16_bits_to_f64(ssup) * 0.1).astype(np.float16).view(np.uint16)
    alpha, beta = synth.cluster_params(N, rng)
    W = o.decode_cs(K, N, ofmt, codes, sq, ssup, alpha, beta, gf)
    w = b.Weight.from_canonical_compressed(K, N, gfmts, codes, sq, ssup, alpha, beta, gf, device=DEV)
    return W, w


def _gemm_bits(w, x_bits, **kw):
    y = b.gemm(w, b.bf16_tensor(x_bits, DEV), **kw)
    torch.cuda.synchronize()
    return b.bf16_bits(y)


@pytest.mark.parametrize("kinds,K,N,n_wide", [(["narrow"], 2048, 272, None), (["wide"], 2048, 144, None), (["narrow", "wide"], 4096, 208, 32),
                                              (["narrow"], 1024, 576, None)])
@pytest.mark.parametrize("M", [1, 2, 8, 16, 17, 40, 70, 130, 300])
def test_compressed_scales_every_kernel(kinds, K, N, n_wide, M):
    """M = 1: GEMV kernel (narrow) or one-row skinny path; 2..16: skinny kernel; 17..: 64-row kernel, and the 256-row
    kernel for narrow-only weights beyond 128 rows."""
    W, w = _case(kinds, K, N, 10 * len(kinds) + N % 13, n_wide)
    x = synth.activations_bf16(M, K, synth.rng(6, 400 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, W), f"compressed scales {kinds} M={M}", rounded=(x, W) if M > 16 else None)
    ks = synth.rng(6, 410 + M).integers(0, K, M)
    ks[:min(M, 4)] = [0, 63, K - 64, K - 1][:min(M, 4)]
    got = _gemm_bits(w, synth.one_hot_bf16(ks, K))
    assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"{kinds} M={M}: decoded weights differ"


@pytest.mark.parametrize("K,N,M", [(256, 1536, 2900), (256, 1024, 3400), (256, 2064, 4000)])
def test_compressed_scales_256_row_kernel(K, N, M):
    """Shapes the library sends to the 256-row kernel (column blocks of 192, 128 and 256)."""
    W, w = _case(["narrow"], K, N, 31 + N % 7, None)
    x = synth.activations_bf16(M, K, synth.rng(6, 600 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, W), f"compressed scales, 256-row kernel N={N} M={M}", rounded=(x, W))
    ks = synth.rng(6, 610 + M).integers(0, K, M)
    got = _gemm_bits(w, synth.one_hot_bf16(ks, K))
    assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"N={N} M={M}: decoded weights differ"


def test_compressed_scales_explicit_shapes_and_errors():
    W, w = _case(["narrow", "wide"], 2048, 64, 77, 8)
    x = synth.activations_bf16(8, 2048, synth.rng(6, 500))
    ref = o.matmul(x, W)
    for launch in ((1, 1, 1, 1), (1, 2, 2, 1), (1, 1, 2, 2), (1, 4, 1, 1)):
        assert_gemm_close(_gemm_bits(w, x, launch=b.ccq_launch(*launch)), ref, f"launch={launch}")
    # more rows than the kernel holds at a time with compressed scales (16): walked 16 at a time
    x40 = synth.activations_bf16(40, 2048, synth.rng(6, 501))
    assert_gemm_close(_gemm_bits(w, x40, launch=b.ccq_launch(1, 2, 1, 2)), o.matmul(x40, W), "40 rows, explicit launch")


def test_compressed_scales_grouped_many_rows_per_expert():
    """Experts with more than 16 rows (a prefill-sized routing) through the grouped entry point."""
    E, K, N, T = 3, 512, 48, 50
    rng = synth.rng(6, 600)
    cases = []
    for e in range(E):
        codes = synth.random_codes(N, K // 4, rng)
        sq = rng.integers(0, 256, size=(N, K // 128), dtype=np.uint8)
        ssup = synth.scales_log_uniform_fp16(N, 1, rng, 1e-4, 1e-2).reshape(N)
        alpha, beta = synth.cluster_params(N, rng)
        cases.append((codes, sq, ssup, alpha, beta))
    w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], np.stack([c[0] for c in cases]), np.stack([c[1] for c in cases]),
                                           np.stack([c[2] for c in cases]), np.stack([c[3] for c in cases]), np.stack([c[4] for c in cases]),
                                           device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(6, 601))
    offs = np.array([0, 40, 43, 100], dtype=np.int32)          # 40, 3 and 57 rows
    rows = synth.rng(6, 602).integers(0, T, 100).astype(np.int32)
    y = b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), offs)
    torch.cuda.synchronize()
    got = b.bf16_bits(y)
    for e in range(E):
        lo, hi = offs[e], offs[e + 1]
        Wd = o.decode_cs(K, N, o.F2, *cases[e][:3], cases[e][3], cases[e][4])
        assert_gemm_close(got[lo:hi], o.matmul(x[rows[lo:hi]], Wd), f"expert {e}")


def test_config2_shape_compressed_scales():
    """K = N = 8192 at 2.0625 bits per weight all told: sampled output channels, M = 1 and 16."""
    K = N = 8192
    W_rows = np.concatenate([np.arange(16), np.arange(4096, 4112), np.arange(N - 16, N)])
    rng = synth.rng(6, 900)
    codes = synth.random_codes(N, K // 4, rng)
    sq = rng.integers(0, 256, size=(N, K // 128), dtype=np.uint8)
    ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
    alpha, beta = synth.cluster_params(N, rng)
    w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=DEV)
    Wr = o.decode_cs(K, len(W_rows), o.F2, codes[W_rows], sq[W_rows], ssup[W_rows], alpha[W_rows], beta[W_rows])
    for M in (1, 16):
        x = synth.activations_bf16(M, K, synth.rng(6, 910 + M))
        got = _gemm_bits(w, x)
        assert_gemm_close(got[:, W_rows], o.matmul(x, Wr), f"config-2 shape, compressed scales, M={M}")
