"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Decoded weights are compared bit for bit (one-hot activations make ccq_gemm
return bf16(W_dq[:, k])); GEMM outputs are compared element by element within
the tolerance of tests/cases.py.  Sizes here finish in seconds on the oracle and
still span several tiles, ragged splits and every launch decomposition; the
full benchmark configurations are in test_gpu_configs.py."""
import numpy as np
import pytest
import torch

from cases import Case, assert_gemm_close, canon_zero, encoded_case, random_case, grouped_rounded_weight_sigma
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _gemm_bits(w, x_bits, **kw):
    y = b.gemm(w, b.bf16_tensor(x_bits, DEV), **kw)
    torch.cuda.synchronize()
    return b.bf16_bits(y)


def _built(kinds, M, launch) -> bool:
    """Launch shapes the kernels are built for: two row tiles per wavefront only for the narrow format
    with at most 32 held rows; at most 8 wavefronts per workgroup for M = 1 and beyond 16 held rows, 4 beyond 32."""
    rt, wr, wk, _ = launch
    held = min(M, 64)
    if rt == 2 and (held > 32 or "wide" in kinds):
        return False
    if held > 32 and wr * wk > 4:
        return False
    if (held > 16 or held == 1) and wr * wk > 8:
        return False
    return True


def _check_decode(case: Case, w, ks, **kw):
    """One-hot rows e_k through the GEMM return column k of the decoded matrix, exactly."""
    ks = list(ks)
    got = _gemm_bits(w, synth.one_hot_bf16(ks, case.K), **kw)
    want = o.to_bf16_bits(case.W()[:, ks].T)
    assert np.array_equal(canon_zero(got), canon_zero(want)), f"decoded weights differ at columns {ks[:8]}..."


@pytest.fixture(scope="module")
def cfg1():
    """Config 1: W 1024x1024 ~ N(0, 0.02), encoded by the oracle at 2.0 bits/weight."""
    c = encoded_case(1024, 1024, 1)
    return c, c.device_weight(DEV)


def test_cfg1_decode_bit_exact(cfg1):
    c, w = cfg1
    rng = np.random.default_rng(0)
    cols = np.concatenate([np.arange(0, 64), [255, 256, 511, 960, 1023], rng.integers(0, 1024, 59)])
    for i in range(0, len(cols), 16):
        _check_decode(c, w, cols[i:i + 16])
    _check_decode(c, w, [7])                                     # M = 1 path
    _check_decode(c, w, [1, 2, 1022])                            # M = 3 path (4 held rows)


def test_cfg1_gemv_and_skinny(cfg1):
    c, w = cfg1
    for M in (1, 2, 3, 4, 5, 8, 15, 16, 17, 32, 33, 48, 64):
        x = synth.activations_bf16(M, c.K, synth.rng(1, 100 + M))
        assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"cfg1 M={M}")


def test_more_rows_than_one_pass(cfg1):
    c, w = cfg1
    for M in (65, 100, 130):
        x = synth.activations_bf16(M, c.K, synth.rng(1, 200 + M))
        assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"cfg1 M={M}")


@pytest.mark.parametrize("K,N,M", [(768, 384, 300), (512, 208, 70), (256, 16, 65), (1024, 576, 257), (2048, 192, 512),
                                   (256, 1536, 2900), (256, 1024, 3400), (256, 2064, 4000)])
def test_large_m_kernel_small_shapes(K, N, M):
    """More than 64 rows on narrow-format weights go through the LDS-tiled MFMA kernels: the 64-row one, and (the
    three shapes with thousands of rows, where the library expects it to be faster) the 256-row one with column
    blocks of 192, 128 and 256; ragged last blocks in M and N, decoded weights exact and products within tolerance."""
    c = random_case(K, N, ["narrow"], 1, stream0=900 + N)
    w = c.device_weight(DEV)
    x = synth.activations_bf16(M, K, synth.rng(1, 950 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"large-M K={K} N={N} M={M}", rounded=(x, c.W()))
    ks = synth.rng(1, 960 + M).integers(0, K, M)
    got = _gemm_bits(w, synth.one_hot_bf16(ks, K))
    want = o.to_bf16_bits(c.W()[:, ks].T)
    assert np.array_equal(canon_zero(got), canon_zero(want)), "large-M kernel: decoded weights differ"


@pytest.mark.parametrize("launch", [(1, 1, 1, 1), (2, 1, 1, 1), (1, 4, 1, 1), (1, 1, 4, 1), (2, 2, 2, 1), (1, 2, 1, 2), (2, 1, 2, 4),
                                    (1, 4, 4, 1), (1, 1, 16, 1), (2, 3, 3, 3), (1, 2, 8, 1), (1, 1, 1, 5)])
@pytest.mark.parametrize("M", [1, 4, 16, 40])
def test_every_decomposition_gives_the_same_answer(cfg1, launch, M):
    c, w = cfg1
    if not _built(c.kinds, M, launch):
        pytest.skip("launch shape not built for this many held rows")
    x = synth.activations_bf16(M, c.K, synth.rng(1, 300 + M))
    ref = o.matmul(x, c.W())
    assert_gemm_close(_gemm_bits(w, x, launch=b.ccq_launch(*launch)), ref, f"M={M} launch={launch}")
    _check_decode(c, w, [3, 64 + 17, 1023, 500][:min(M, 4)], launch=b.ccq_launch(*launch))


@pytest.mark.parametrize("kinds,K,N,n_wide", [(["wide"], 1024, 256, None), (["wide"], 512, 48, None), (["narrow"], 1280, 80, None),
                                              (["narrow", "wide"], 2048, 128, 8), (["narrow", "wide"], 4096, 64, 24)])
def test_formats_decode_and_gemm(kinds, K, N, n_wide):
    c = random_case(K, N, kinds, 7, stream0=10 * len(kinds) + K % 7, n_wide=n_wide)
    w = c.device_weight(DEV)
    ks = [0, 1, 2, 3, 17, 18, 19, 53, 54, 59, 60, 61, 62, 63, 64, K - 1]
    _check_decode(c, w, ks)
    if c.group_fmt is not None:                                  # every column of one wide and one narrow group
        gw, gn = int(np.flatnonzero(c.group_fmt == 1)[0]), int(np.flatnonzero(c.group_fmt == 0)[-1])
        for g in (gw, gn):
            for i in range(0, 64, 16):
                _check_decode(c, w, range(64 * g + i, 64 * g + i + 16))
    else:
        for i in range(0, 64, 16):
            _check_decode(c, w, range(64 + i, 64 + i + 16))
    for M in (1, 3, 8, 16, 33, 64):
        x = synth.activations_bf16(M, K, synth.rng(7, 50 + M))
        ref = o.matmul(x, c.W())
        assert_gemm_close(_gemm_bits(w, x), ref, f"{kinds} K={K} N={N} M={M}")
        for launch in ((2, 2, 1, 1), (1, 1, 3, 2), (1, 2, 2, 1), (1, 2, 1, 4), (2, 2, 1, 4), (1, 1, 1, 8)):
            if not _built(kinds, M, launch):
                continue
            assert_gemm_close(_gemm_bits(w, x, launch=b.ccq_launch(*launch)), ref, f"{kinds} M={M} launch={launch}")


@pytest.mark.parametrize("kinds,K,N,M,n_wide", [(["wide"], 2048, 144, 70, None), (["narrow", "wide"], 4096, 272, 40, 32),
                                                (["narrow"], 2048, 128, 100, None), (["narrow", "wide"], 2048, 64, 17, 8),
                                                (["wide"], 1024, 400, 130, None)])
def test_mid_kernel_formats(kinds, K, N, M, n_wide):
    """17 and more rows (any format mix; beyond 128 rows unless narrow only) run the 64-row LDS-tiled kernel: K cut into
    one or several shares, ragged row and column blocks, the group map of mixed formats.  Decoded weights exact through
    one-hot rows, products within tolerance."""
    c = random_case(K, N, kinds, 9, stream0=20 * len(kinds) + N % 11, n_wide=n_wide)
    w = c.device_weight(DEV)
    x = synth.activations_bf16(M, K, synth.rng(9, 300 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"mid {kinds} K={K} N={N} M={M}", rounded=(x, c.W()))
    ks = synth.rng(9, 310 + M).integers(0, K, M)
    ks[:4] = [0, 63, K - 64, K - 1]
    got = _gemm_bits(w, synth.one_hot_bf16(ks, K))
    want = o.to_bf16_bits(c.W()[:, ks].T)
    assert np.array_equal(canon_zero(got), canon_zero(want)), f"mid kernel {kinds}: decoded weights differ"


@pytest.mark.parametrize("kinds,K,N,M", [(["wide"], 1024, 48, 7), (["wide"], 4096, 64, 9), (["wide"], 512, 208, 16), (["wide"], 2048, 16, 5),
                                         (["narrow"], 1280, 80, 20), (["narrow"], 4096, 48, 32), (["narrow"], 256, 144, 17)])
def test_per_group_tile_kernel(kinds, K, N, M):
    """5-16 rows on the wide format and 17-32 rows on the narrow one go through the kernel that stages one activation
    tile per 64-weight group: ragged last row block (fewer than four row tiles), K cut into shares, rows past M in the
    last activation tile; decoded weights exact, products within the tolerance of the exact-weight kernels."""
    c = random_case(K, N, kinds, 9, stream0=N + M)
    w = c.device_weight(DEV)
    x = synth.activations_bf16(M, K, synth.rng(9, 500 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"{kinds} K={K} N={N} M={M}")
    ks = synth.rng(9, 600 + M).integers(0, K, M)
    ks[:5] = [0, 63, 64, K - 1, K - 64]
    _check_decode(c, w, ks)


@pytest.mark.parametrize("K,N", [(2048, 96), (8192, 64), (1280, 48)])
def test_two_to_four_rows(K, N):
    """2..4 rows on narrow-format weights: the GEMV kernel with MFMA 4x4x4 fed four different rows (K = 1280 does not
    split into shares of at most 4 k-tiles and takes the general kernel instead).  Decoded weights exact, products close, and a row's
    result independent of the rows that ride along."""
    c = random_case(K, N, ["narrow"], 12, stream0=K % 97)
    w = c.device_weight(DEV)
    for M in (2, 3, 4):
        x = synth.activations_bf16(M, K, synth.rng(12, 40 + M))
        got = _gemm_bits(w, x)
        assert_gemm_close(got, o.matmul(x, c.W()), f"K={K} M={M}")
        for m in range(M):    # a row's result does not depend on which other rows ride along
            alone = np.concatenate([x[m:m + 1], x[(m + 1) % M:(m + 1) % M + 1]]) if M > 2 else None
            if alone is not None:
                assert np.array_equal(got[m], _gemm_bits(w, alone)[0]), f"row {m} depends on its neighbours"
        ks = [0, K - 1, 63, 64][:M]
        _check_decode(c, w, ks)


def test_strided_activations_and_guard_bands():
    """ldx > K, ldy > N: nothing outside y[:M, :N] is written."""
    c = random_case(1024, 96, ["narrow"], 8)
    w = c.device_weight(DEV)
    for M in (1, 2, 3, 4, 7, 17, 64, 70, 200):
        xb = synth.activations_bf16(M, c.K, synth.rng(8, M))
        xt = torch.zeros((M, c.K + 64), dtype=torch.bfloat16, device=DEV)
        xt[:, :c.K] = b.bf16_tensor(xb, DEV)
        big = torch.full((M + 2, c.N + 40), -7.0, dtype=torch.bfloat16, device=DEV)
        b.gemm(w, xt[:, :c.K], out=big[1:M + 1, 8:8 + c.N])
        torch.cuda.synchronize()
        assert_gemm_close(b.bf16_bits(big[1:M + 1, 8:8 + c.N]), o.matmul(xb, c.W()), f"strided M={M}")
        guard = big.clone()
        guard[1:M + 1, 8:8 + c.N] = -7.0
        assert bool((guard == -7.0).all()), "wrote outside the output block"


def test_deterministic(cfg1):
    c, w = cfg1
    for M, launch in ((1, None), (16, None), (16, (1, 2, 2, 4)), (64, None)):
        x = synth.activations_bf16(M, c.K, synth.rng(1, 400 + M))
        kw = {} if launch is None else {"launch": b.ccq_launch(*launch)}
        first = _gemm_bits(w, x, **kw)
        for _ in range(3):
            assert np.array_equal(_gemm_bits(w, x, **kw), first)


def test_linearity_in_activations(cfg1):
    """The path is linear in x: exact powers of two scale the output exactly."""
    c, w = cfg1
    x = synth.activations_bf16(4, c.K, synth.rng(1, 500))
    y1 = o.bf16_bits_to_f64(_gemm_bits(w, x))
    x4 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(x) * np.float32(4.0))
    y4 = o.bf16_bits_to_f64(_gemm_bits(w, x4))
    assert np.array_equal(y4, 4.0 * y1)


def _grouped_reference(cases, x, rows, offs):
    return o.grouped_matmul(x, rows, offs, lambda e: cases[e].W())


@pytest.mark.parametrize("kinds,K,N", [(["narrow"], 512, 64), (["wide"], 512, 32), (["narrow"], 1024, 160)])
def test_grouped_small(kinds, K, N):
    E, T = 6, 40
    cases = [random_case(K, N, kinds, 9, stream0=10 * e) for e in range(E)]
    w = b.Weight.from_canonical(K, N, [b.NARROW if kinds[0] == "narrow" else b.WIDE],
                                np.stack([c.codes for c in cases]), np.stack([c.scales for c in cases]),
                                None if kinds[0] != "narrow" else np.stack([c.alpha for c in cases]),
                                None if kinds[0] != "narrow" else np.stack([c.beta for c in cases]), device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(9, 99))
    # expert 2 is empty, expert 4 has more rows than one pass holds at the chosen tile height
    counts = [5, 1, 0, 17, 38, 16]
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    rows = synth.rng(9, 98).integers(0, T, size=int(offs[-1])).astype(np.int32)
    P = int(offs[-1])
    y = torch.full((P + 1, N), 3.0, dtype=torch.bfloat16, device=DEV)
    b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), offs, out=y[:P])
    torch.cuda.synchronize()
    assert_gemm_close(b.bf16_bits(y[:P]), _grouped_reference(cases, x, rows, offs), f"grouped {kinds}")
    assert bool((y[P] == 3.0).all())
    # decoded weights of every expert, bit exact: one-hot tokens routed to each expert
    ks = [0, 63, 64, K - 1]
    xe = synth.one_hot_bf16(ks, K)
    counts2 = [len(ks)] * E
    offs2 = np.concatenate([[0], np.cumsum(counts2)]).astype(np.int32)
    rows2 = np.tile(np.arange(len(ks), dtype=np.int32), E)
    y2 = b.grouped_gemm(w, b.bf16_tensor(xe, DEV), torch.from_numpy(rows2).to(DEV), torch.from_numpy(offs2).to(DEV), offs2)
    torch.cuda.synchronize()
    got = b.bf16_bits(y2).reshape(E, len(ks), N)
    for e in range(E):
        assert np.array_equal(canon_zero(got[e]), canon_zero(o.to_bf16_bits(cases[e].W()[:, ks].T))), f"expert {e}"


@pytest.mark.parametrize("kinds,K,N,n_wide", [(["narrow"], 512, 160, None), (["narrow"], 1024, 64, None), (["wide"], 512, 160, None),
                                              (["narrow", "wide"], 2048, 144, 8)])
def test_grouped_many_rows_per_expert(kinds, K, N, n_wide):
    """A prefill-sized routing: experts with several 64-row blocks, one with none, one with a single row; with the
    host copy of the offsets the 64-row kernel runs, without it the per-row-tile kernel does."""
    E, T = 5, 90
    cases = [random_case(K, N, kinds, 13, stream0=10 * e, n_wide=n_wide) for e in range(E)]
    for c in cases:
        c.group_fmt = cases[0].group_fmt  # one format map for all experts
    fmts = [b.NARROW if k == "narrow" else b.WIDE for k in kinds]
    has_n = "narrow" in kinds
    w = b.Weight.from_canonical(K, N, fmts, np.stack([c.codes for c in cases]), np.stack([c.scales for c in cases]),
                                np.stack([c.alpha for c in cases]) if has_n else None, np.stack([c.beta for c in cases]) if has_n else None,
                                cases[0].group_fmt, device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(13, 99))
    counts = [130, 0, 70, 1, 33]
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    P = int(offs[-1])
    rows = synth.rng(13, 98).integers(0, T, size=P).astype(np.int32)
    ref = _grouped_reference(cases, x, rows, offs)
    sigma = grouped_rounded_weight_sigma(x, rows, offs, lambda e: cases[e].W())
    for host_offsets in (offs, None):
        y = torch.full((P + 1, N), 3.0, dtype=torch.bfloat16, device=DEV)
        b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), host_offsets, out=y[:P])
        torch.cuda.synchronize()
        assert_gemm_close(b.bf16_bits(y[:P]), ref, f"grouped, many rows, host offsets {'given' if host_offsets is not None else 'absent'}", rounded=sigma)
        assert bool((y[P] == 3.0).all())
    # decoded weights, bit exact, through the 64-row kernel: 40 one-hot tokens per expert
    ks = synth.rng(13, 97).integers(0, K, 40)
    ks[:4] = [0, 63, K - 64, K - 1]
    xe = synth.one_hot_bf16(ks, K)
    offs2 = (np.arange(E + 1) * len(ks)).astype(np.int32)
    rows2 = np.tile(np.arange(len(ks), dtype=np.int32), E)
    y2 = b.grouped_gemm(w, b.bf16_tensor(xe, DEV), torch.from_numpy(rows2).to(DEV), torch.from_numpy(offs2).to(DEV), offs2)
    torch.cuda.synchronize()
    got = b.bf16_bits(y2).reshape(E, len(ks), N)
    for e in range(E):
        assert np.array_equal(canon_zero(got[e]), canon_zero(o.to_bf16_bits(cases[e].W()[:, ks].T))), f"expert {e}"


@pytest.mark.parametrize("kinds,K,N", [(["narrow"], 512, 64), (["wide"], 512, 32), (["narrow"], 2048, 160)])
def test_grouped_one_token(kinds, K, N):
    """One token's decode step: no expert has more than one row (some have none); with the host copy of the
    offsets the library treats every expert as a GEMV, without it the 16-row path runs; both must agree with the oracle."""
    E = 6
    cases = [random_case(K, N, kinds, 12, stream0=10 * e) for e in range(E)]
    w = b.Weight.from_canonical(K, N, [b.NARROW if kinds[0] == "narrow" else b.WIDE],
                                np.stack([c.codes for c in cases]), np.stack([c.scales for c in cases]),
                                None if kinds[0] != "narrow" else np.stack([c.alpha for c in cases]),
                                None if kinds[0] != "narrow" else np.stack([c.beta for c in cases]), device=DEV, experts=E)
    x = synth.activations_bf16(3, K, synth.rng(12, 99))
    counts = [1, 0, 1, 1, 0, 1]
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    rows = np.array([2, 0, 2, 1], dtype=np.int32)
    ref = _grouped_reference(cases, x, rows, offs)
    for host_offsets in (offs, None):
        y = b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), host_offsets)
        torch.cuda.synchronize()
        assert_gemm_close(b.bf16_bits(y), ref, f"grouped, one token, {kinds}, host offsets {'given' if host_offsets is not None else 'absent'}")
    # decoded weights, bit exact: a one-hot token per expert
    ks = [0, 63, K - 64, K - 1, 17, 64]
    xe = synth.one_hot_bf16(ks, K)
    offs2 = np.arange(E + 1, dtype=np.int32)
    rows2 = np.arange(E, dtype=np.int32)
    y2 = b.grouped_gemm(w, b.bf16_tensor(xe, DEV), torch.from_numpy(rows2).to(DEV), torch.from_numpy(offs2).to(DEV), offs2)
    torch.cuda.synchronize()
    got = b.bf16_bits(y2)
    for e in range(E):
        assert np.array_equal(canon_zero(got[e]), canon_zero(o.to_bf16_bits(cases[e].W()[:, ks[e]]))), f"expert {e}"


def test_grouped_all_experts_empty_and_errors():
    c = random_case(512, 32, ["narrow"], 10)
    w = c.device_weight(DEV)
    x = b.bf16_tensor(synth.activations_bf16(4, 512, synth.rng(10, 1)), DEV)
    rows = torch.zeros(0, dtype=torch.int32, device=DEV)
    offs = torch.zeros(2, dtype=torch.int32, device=DEV)
    y = b.grouped_gemm(w, x, rows, offs, np.zeros(2, np.int32))
    assert y.shape == (0, 32)
    rows = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(b.CcqError) as ei:
        b.grouped_gemm(w, x, rows, offs, np.array([0, 3], np.int32))      # offsets[E] != P
    assert ei.value.status == -6


@pytest.mark.parametrize("kinds,K,N,M", [(["narrow"], 2048, 1024, 16), (["narrow"], 2048, 1024, 8), (["narrow"], 2048, 1024, 64),
                                         (["narrow"], 4096, 256, 24), (["wide"], 4096, 256, 12), (["wide"], 2048, 272, 70),
                                         (["narrow", "wide"], 4096, 128, 40), (["narrow", "wide"], 4096, 128, 9), (["wide"], 8192, 64, 16)])
def test_workspace_guard_bands(kinds, K, N, M):
    """The K shares' fp32 partial tiles stay inside the workspace the library asked for: canaries on both sides of a
    workspace of exactly ccq_gemm_workspace_bytes are untouched, and the result does not depend on what the workspace held."""
    c = random_case(K, N, kinds, 14, stream0=M, n_wide=32 if len(kinds) == 2 else None)
    w = c.device_weight(DEV)
    need = b.gemm_workspace_bytes(w.desc, M)
    assert need > 0, "the case must cut K"
    band = 4096
    buf = torch.full((need + 2 * band,), 0x5A, dtype=torch.uint8, device=DEV)
    ws = buf[band:band + need]
    x = synth.activations_bf16(M, K, synth.rng(14, 70 + M))
    xt = b.bf16_tensor(x, DEV)
    y1 = b.bf16_bits(b.gemm(w, xt, workspace=ws))
    torch.cuda.synchronize()
    assert bool((buf[:band] == 0x5A).all()) and bool((buf[band + need:] == 0x5A).all()), "wrote outside the workspace"
    assert_gemm_close(y1, o.matmul(x, c.W()), f"guarded workspace {kinds} M={M}", rounded=(x, c.W()) if M > 32 else None)
    buf.fill_(0xFF)   # NaN patterns in the workspace must not leak into the result
    y2 = b.bf16_bits(b.gemm(w, xt, workspace=ws))
    torch.cuda.synchronize()
    assert np.array_equal(y1, y2)
    if M > 32 or (M > 16 and kinds != ["narrow"]):   # a smaller workspace is rejected
        with pytest.raises(b.CcqError) as ei:
            b.gemm(w, xt, workspace=buf[band:band + need - 16])
        assert ei.value.status == -5
    else:
        # the 16-row kernels (32 rows on the narrow format) take fewer, longer shares of K when the workspace is smaller; where K does not split that
        # way the call is either served by the general kernel or rejected, never wrong
        buf.fill_(0xFF)
        try:
            y3 = b.bf16_bits(b.gemm(w, xt, workspace=buf[band:band + need // 2]))
        except b.CcqError as e:
            assert e.status == -5 and kinds != ["narrow"]
        else:
            torch.cuda.synchronize()
            assert_gemm_close(y3, o.matmul(x, c.W()), f"half the workspace {kinds} M={M}")
            assert bool((buf[:band] == 0xFF).all()) and bool((buf[band + need // 2:] == 0xFF).all()), "wrote outside the smaller workspace"


@pytest.mark.parametrize("n_narrow,n_wide,what", [(0, 16, "wide, shares of two k-tiles"), (0, 8 * 5, "wide, five shares of one"), (96, 64, "(4,2)"),
                                                  (72, 80, "(2,2)"), (96, 56, "(4,1)"), (36, 80, "(1,2)"), (20, 8, "(1,1)"), (24, 8, "(2,1)"),
                                                  (108, 8, "27 narrow k-tiles: no split into 16 shares, general kernel")])
@pytest.mark.parametrize("mode", [0, 1])
def test_one_row_kernel_every_share_shape(n_narrow, n_wide, what, mode):
    """One activation row on wide-format and mixed weights: every (narrow share, wide share) pair the one-row kernel is
    built for, both scale modes; decoded weights bit-exact (one-hot rows, one per call) and the product within tolerance."""
    G = n_narrow + n_wide
    K, N = 64 * G, 48
    kinds = ["wide"] if n_narrow == 0 else ["narrow", "wide"]
    rng = synth.rng(17, G + mode)
    gf = synth.group_format_map(G, n_wide, rng) if n_narrow else None
    ofmt = o.F275 if n_narrow == 0 else (o.F2, o.F275)
    bfmt = [b.WIDE] if n_narrow == 0 else [b.NARROW, b.WIDE]
    codes = synth.random_codes(N, o.row_bytes(K, ofmt, gf), rng)
    alpha, beta = synth.cluster_params(N, rng)
    if mode == 0:
        scales = synth.scales_log_uniform_fp16(N, G, rng)
        W = o.decode(K, N, ofmt, codes, scales, alpha, beta, gf)
        w = b.Weight.from_canonical(K, N, bfmt, codes, scales, alpha, beta, gf, device=DEV)
    else:
        nb = o.sq_row_bytes(K, ofmt, gf)
        sq = rng.integers(0, 256, size=(N, max(nb, 1)), dtype=np.uint8)[:, :nb]
        ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
        W = o.decode_cs(K, N, ofmt, codes, sq, ssup, alpha, beta, gf)
        w = b.Weight.from_canonical_compressed(K, N, bfmt, codes, sq, ssup, alpha, beta, gf, device=DEV)
    x = synth.activations_bf16(1, K, synth.rng(17, 900 + G))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, W), f"one row, {what}, scale mode {mode}")
    ks = np.concatenate([[0, 17, 59, 60, 61, 62, 63, 64, K - 64, K - 4, K - 1], synth.rng(17, 901).integers(0, K, 21)])
    for k in ks:
        got = _gemm_bits(w, synth.one_hot_bf16([int(k)], K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, [int(k)]].T))), f"{what}: decoded weights differ at column {k}"


@pytest.mark.parametrize("G,N,what", [(172, 96, "43 k-tiles (K = 11008): 15 shares of three, the last of one"),
                                      (68, 40, "17 k-tiles: nine shares of two, the last of one"),
                                      (170, 200, "43 k-tiles, the last one ragged too"),
                                      (296, 64, "74 k-tiles (K = 18944): 13 shares of six, the last of two"),
                                      (344, 32, "86 k-tiles (K = 22016): 15 shares of six, the last of two"),
                                      (432, 32, "108 k-tiles (K = 27648): 16 shares of seven, the last of three"),
                                      (462, 16, "116 k-tiles (K = 29568): 15 shares of eight, the last of four")])
@pytest.mark.parametrize("mode", [0, 1])
def test_one_row_kernel_unequal_shares(G, N, what, mode):
    """One activation row on narrow-format weights whose k-tile count has no split into at most 16 equal shares (the
    K of several common models): the last wavefront's share is shorter.  Product within tolerance, decoded weights bit
    for bit at the ends of K, around the last share and at random columns."""
    K = 64 * G
    rng = synth.rng(21, G + mode)
    codes = synth.random_codes(N, o.row_bytes(K, o.F2), rng)
    alpha, beta = synth.cluster_params(N, rng)
    if mode == 0:
        scales = synth.scales_log_uniform_fp16(N, G, rng)
        W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
        w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    else:
        sq = rng.integers(0, 256, size=(N, o.sq_row_bytes(K, o.F2)), dtype=np.uint8)
        ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
        W = o.decode_cs(K, N, o.F2, codes, sq, ssup, alpha, beta)
        w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=DEV)
    x = synth.activations_bf16(1, K, synth.rng(21, 900 + G))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, W), f"one row, {what}, scale mode {mode}")
    ks = np.concatenate([[0, 63, 64, K - 1, K - 64, K - 65, K - 256, K - 257, K - 512, K - 1024, K - 2048], synth.rng(21, 901).integers(0, K, 13)])
    for k in ks:
        k = int(max(k, 0))
        got = _gemm_bits(w, synth.one_hot_bf16([k], K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, [k]].T))), f"{what}: decoded weights differ at column {k}"


@pytest.mark.parametrize("G,N,what", [(16, 100, "shares of one k-tile"), (15, 40, "shares of one, the last k-tile ragged"),
                                      (128, 400, "16 shares of two"), (110, 1000, "14 shares of two, ragged K and N"),
                                      (84, 72, "7 shares of three"), (128, 8208, "8 shares of four: more wavefronts than the chip holds"),
                                      (132, 64, "33 k-tiles: 11 shares of three"), (144, 64, "36 k-tiles: one workgroup per CU"),
                                      (172, 40, "43 k-tiles (K = 11008): unequal shares, 14 of three and one of one"),
                                      (256, 32, "64 k-tiles: 16 shares of four, 144 KiB of LDS"),
                                      (260, 32, "65 k-tiles: no split into 16 shares, the 16-row kernel")])
@pytest.mark.parametrize("mode", [0, 1])
def test_four_row_kernel_every_share_shape(G, N, what, mode):
    """Two to four activation rows on narrow-format weights (the GEMV operator of Table 4 with M = 4): every share length
    the four-row kernel is built for, both scale modes, strided activations; the product within tolerance and the
    decoded weights bit for bit (one-hot rows, a different column per row)."""
    K = 64 * G
    rng = synth.rng(19, G + mode)
    codes = synth.random_codes(N, o.row_bytes(K, o.F2), rng)
    alpha, beta = synth.cluster_params(N, rng)
    if mode == 0:
        scales = synth.scales_log_uniform_fp16(N, G, rng)
        W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
        w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    else:
        nb = o.sq_row_bytes(K, o.F2)
        sq = rng.integers(0, 256, size=(N, nb), dtype=np.uint8)
        ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
        W = o.decode_cs(K, N, o.F2, codes, sq, ssup, alpha, beta)
        w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=DEV)
    for M in (2, 3, 4):
        x = synth.activations_bf16(M, K, synth.rng(19, 900 + G + M))
        xs = torch.zeros((M, K + 24), dtype=torch.bfloat16, device=DEV)      # rows 24 elements apart from contiguous
        xs[:, :K] = b.bf16_tensor(x, DEV)
        y = torch.full((M + 1, (N + 7) // 8 * 8 + 8), 3.140625, dtype=torch.bfloat16, device=DEV)
        b.gemm(w, xs[:, :K], out=y[:M, :N])
        torch.cuda.synchronize()
        bits = b.bf16_bits(y)
        assert np.all(bits[:M, N:] == 0x4049) and np.all(bits[M] == 0x4049), f"{what} M={M}: written outside the result"
        assert_gemm_close(bits[:M, :N], o.matmul(x, W), f"{M} rows, {what}, scale mode {mode}")
    for k0 in (0, 59, K - 64, K - 4):
        ks = [k0, min(k0 + 1, K - 1), K - 1 - k0, (k0 + 64) % K]
        got = _gemm_bits(w, synth.one_hot_bf16(ks, K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, ks].T))), f"{what}: decoded weights differ at columns {ks}"


@pytest.mark.parametrize("n_narrow,n_wide,cap,what", [(0, 16, 32, "(0,1)"), (0, 16, 1, "(0,2): all of K in one share"), (0, 40, 32, "(0,1), five shares"),
                                                      (64, 32, 32, "(1,1)"), (64, 32, 16, "(2,1)"), (64, 32, 10, "(2,2)"), (64, 32, 8, "(4,1)"),
                                                      (64, 32, 6, "(4,2)"), (36, 80, 16, "(1,2)"), (100, 56, 32, "(1,1), 32 shares")])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("M", [2, 7, 16])
def test_sixteen_row_kernel_wide_and_mixed(n_narrow, n_wide, cap, what, mode, M):
    """Two to sixteen activation rows on wide-format and mixed weights: every (narrow share, wide share) pair of the
    16-row kernel for those formats (the workspace is sized for `cap` shares, which decides the pair), both scale modes,
    N not a multiple of the eight row tiles a workgroup holds; decoded weights bit-exact (one-hot rows) and the product
    within tolerance; rows past M and columns past N untouched."""
    G = n_narrow + n_wide
    K, N = 64 * G, 16 * 11 + 5
    rng = synth.rng(18, G + mode)
    gf = synth.group_format_map(G, n_wide, rng) if n_narrow else None
    ofmt = o.F275 if n_narrow == 0 else (o.F2, o.F275)
    bfmt = [b.WIDE] if n_narrow == 0 else [b.NARROW, b.WIDE]
    codes = synth.random_codes(N, o.row_bytes(K, ofmt, gf), rng)
    alpha, beta = synth.cluster_params(N, rng)
    if mode == 0:
        scales = synth.scales_log_uniform_fp16(N, G, rng)
        W = o.decode(K, N, ofmt, codes, scales, alpha, beta, gf)
        w = b.Weight.from_canonical(K, N, bfmt, codes, scales, alpha, beta, gf, device=DEV)
    else:
        nb = o.sq_row_bytes(K, ofmt, gf)
        sq = rng.integers(0, 256, size=(N, max(nb, 1)), dtype=np.uint8)[:, :nb]
        ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
        W = o.decode_cs(K, N, ofmt, codes, sq, ssup, alpha, beta, gf)
        w = b.Weight.from_canonical_compressed(K, N, bfmt, codes, sq, ssup, alpha, beta, gf, device=DEV)
    ws = torch.empty(cap * M * w.info.padded_N * 4, dtype=torch.uint8, device=DEV)

    def run(x_bits):
        ld = (N + 7) // 8 * 8 + 8
        y = torch.full((M + 1, ld), 3.140625, dtype=torch.bfloat16, device=DEV)
        b.gemm(w, b.bf16_tensor(x_bits, DEV), out=y[:M, :N], workspace=ws)
        torch.cuda.synchronize()
        bits = b.bf16_bits(y)
        assert np.all(bits[:M, N:] == 0x4049) and np.all(bits[M] == 0x4049), "wrote past the output"
        return bits[:M, :N]
    x = synth.activations_bf16(M, K, synth.rng(18, 900 + G + M))
    assert_gemm_close(run(x), o.matmul(x, W), f"{M} rows, {what}, scale mode {mode}")
    ks = np.concatenate([[K - 1, 0, 59, 60, 61, 62, 63, 64, K - 64, K - 4, 17], synth.rng(18, 901).integers(0, K, 21)])
    for i in range(0, len(ks), M):
        kk = [int(k) for k in ks[i:i + M]]
        kk += [kk[-1]] * (M - len(kk))
        got = run(synth.one_hot_bf16(kk, K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, kk].T))), f"{what}: decoded weights differ at columns {kk}"


@pytest.mark.parametrize("G,cap,what", [(64, 32, "shares of one k-tile"), (64, 8, "shares of two"), (64, 4, "shares of four"),
                                        (62, 4, "shares of four, the last k-tile ragged"), (16, 1, "all of K in one share: no partial tiles"),
                                        (172, 32, "43 k-tiles (K = 11008): unequal shares, ten of four and one of three"),
                                        (172, 24, "43 k-tiles: 22 shares of two, the last of one"), (68, 32, "17 k-tiles: unequal shares")])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("M", [5, 16, 17, 25, 32])
def test_sixteen_and_32_row_kernel_narrow(G, cap, what, mode, M):
    """Five to 32 activation rows on narrow-format weights: every share length of the 16-row kernel and of its variant
    that holds two 16-row tiles of activations (17..32 rows); the workspace is sized for `cap` shares, which decides
    the share length; both scale modes, N not a multiple of the eight row tiles a workgroup holds; decoded weights
    bit-exact (one-hot rows), the product within tolerance, rows past M and columns past N untouched."""
    K, N = 64 * G, 16 * 11 + 5
    rng = synth.rng(20, G + mode)
    codes = synth.random_codes(N, o.row_bytes(K, o.F2), rng)
    alpha, beta = synth.cluster_params(N, rng)
    if mode == 0:
        scales = synth.scales_log_uniform_fp16(N, G, rng)
        W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
        w = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=DEV)
    else:
        sq = rng.integers(0, 256, size=(N, o.sq_row_bytes(K, o.F2)), dtype=np.uint8)
        ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
        W = o.decode_cs(K, N, o.F2, codes, sq, ssup, alpha, beta)
        w = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=DEV)
    ws = torch.full((max(cap * M * w.info.padded_N * 4, 16),), 0xFF, dtype=torch.uint8, device=DEV)

    def run(x_bits):
        ld = (N + 7) // 8 * 8 + 8
        y = torch.full((M + 1, ld), 3.140625, dtype=torch.bfloat16, device=DEV)
        b.gemm(w, b.bf16_tensor(x_bits, DEV), out=y[:M, :N], workspace=ws)
        torch.cuda.synchronize()
        bits = b.bf16_bits(y)
        assert np.all(bits[:M, N:] == 0x4049) and np.all(bits[M] == 0x4049), "wrote past the output"
        return bits[:M, :N]
    x = synth.activations_bf16(M, K, synth.rng(20, 900 + G + M))
    assert_gemm_close(run(x), o.matmul(x, W), f"{M} rows, {what}, scale mode {mode}")
    ks = np.concatenate([[K - 1, 0, 63, 64, K - 64, K - 4, 17], synth.rng(20, 901).integers(0, K, 2 * M - 7)])
    for i in range(0, len(ks), M):
        kk = [int(k) for k in ks[i:i + M]]
        kk += [kk[-1]] * (M - len(kk))
        got = run(synth.one_hot_bf16(kk, K))
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(W[:, kk].T))), f"{what}: decoded weights differ at columns {kk}"


@pytest.mark.parametrize("kind", ["wide", "h16"])
@pytest.mark.parametrize("mode", [0, 1])
def test_one_row_kernel_more_wavefronts_than_the_chip_holds(kind, mode):
    """With more one-k-tile shares than the chip holds wavefronts (521 row tiles x 16 k-tiles > 32 x 256) the one-row
    kernel takes shares of two wide k-tiles.  Sampled output channels against the oracle; one-hot rows bit-exact."""
    K, N = 8192, 16 * 521
    G = K // 64
    rng = synth.rng(19, mode + (7 if kind == "h16" else 0))
    rows = np.concatenate([np.arange(16), np.arange(4160, 4176), np.arange(N - 16, N)])
    ssup = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * (0.1 if kind == "wide" else 0.002)).astype(np.float16).view(np.uint16)
    scales = synth.scales_log_uniform_fp16(N, G, rng)
    if kind == "wide":
        codes = synth.random_codes(N, G * 22, rng)
        if mode == 0:
            w = b.Weight.from_canonical(K, N, [b.WIDE], codes, scales, device=DEV)
            W = o.decode(K, len(rows), o.F275, codes[rows], scales[rows])
        else:
            w = b.Weight.from_canonical_compressed(K, N, [b.WIDE], codes, np.zeros((N, 0), np.uint8), ssup, device=DEV)
            W = o.decode_cs(K, len(rows), o.F275, codes[rows], np.zeros((len(rows), 0), np.uint8), ssup[rows])
    else:
        codes = synth.random_codes(N, o.h16_row_bytes(K), rng)
        if mode == 0:
            w = b.Weight.from_canonical(K, N, b.H16, codes, scales, device=DEV)
            W = o.h16_decode(K, len(rows), codes[rows], scales[rows])
        else:
            w = b.Weight.from_canonical_compressed(K, N, b.H16, codes, None, ssup, device=DEV)
            W = o.h16_decode_cs(K, len(rows), codes[rows], ssup[rows])
    x = synth.activations_bf16(1, K, synth.rng(19, 50))
    assert_gemm_close(_gemm_bits(w, x)[:, rows], o.matmul(x, W), f"one row, {kind}, scale mode {mode}, shares of two k-tiles")
    for k in (0, 62, 63, 511, 512, K - 1):
        got = _gemm_bits(w, synth.one_hot_bf16([k], K))[:, rows]
        want = W[:, [k]].T
        if kind == "h16" and mode == 1:
            want = want.astype(np.float32).astype(np.float64)   # the kernel's single fp32 rounding of field x super scale x state
        assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(want))), f"{kind} mode {mode}: decoded weights differ at column {k}"
