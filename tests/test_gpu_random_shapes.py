"""Seeded random shapes, formats, row counts and launch decompositions through ccq_gemm / ccq_gemm_ex against the oracle:
the index arithmetic of every kernel (K shares, ragged row blocks, rows past M, group maps) on cases nobody picked by hand."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close, canon_zero, random_case
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _draw(rng):
    kinds = [["narrow"], ["wide"], ["narrow", "wide"]][int(rng.integers(0, 3))]
    if kinds == ["narrow"]:
        K, n_wide = 256 * int(rng.integers(1, 13)), None
    elif kinds == ["wide"]:
        K, n_wide = 512 * int(rng.integers(1, 7)), None
    else:
        nn, nw = 4 * int(rng.integers(1, 7)), 8 * int(rng.integers(1, 4))
        K, n_wide = 64 * (nn + nw), nw
    N = 16 * int(rng.integers(1, 18))
    M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 20, 31, 32, 33, 48, 64, 65, 100, 129, 140]))
    return kinds, K, N, M, n_wide


def _valid_launch(rng, kinds, M, tiles_min):
    held = min(M, 64)
    for _ in range(50):
        rt = int(rng.integers(1, 3))
        wr, wk = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        s = int(rng.integers(1, 6))
        if wr * wk > 16:
            continue
        if rt == 2 and (held > 32 or "wide" in kinds):
            continue
        if held > 32 and wr * wk > 4:
            continue
        if (held > 16 or held == 1) and wr * wk > 8:
            continue
        return (rt, wr, wk, s)
    return (1, 1, 1, 1)


@pytest.mark.parametrize("seed", range(36))
def test_random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    kinds, K, N, M, n_wide = _draw(rng)
    c = random_case(K, N, kinds, 40 + seed, n_wide=n_wide)
    w = c.device_weight(DEV)
    x = synth.activations_bf16(M, K, synth.rng(40 + seed, 7))
    ref = o.matmul(x, c.W())
    rounded = (x, c.W()) if M > 16 else None
    xt = b.bf16_tensor(x, DEV)
    what = f"seed {seed}: {kinds} K={K} N={N} M={M}"
    y = b.gemm(w, xt)
    torch.cuda.synchronize()
    assert_gemm_close(b.bf16_bits(y), ref, what, rounded=rounded)
    launch = _valid_launch(rng, kinds, M, None)
    try:
        y2 = b.gemm(w, xt, launch=b.ccq_launch(*launch))
    except b.CcqError as e:
        # a shape whose staging area would not fit LDS is turned down with an error code, nothing is launched
        assert e.status == -2 and launch[1] * launch[2] > 4, (what, launch)
    else:
        torch.cuda.synchronize()
        assert_gemm_close(b.bf16_bits(y2), ref, what + f" launch={launch}")
    # decoded weights, exactly, through whatever kernel this row count selects
    ks = rng.integers(0, K, M)
    got = b.bf16_bits(b.gemm(w, b.bf16_tensor(synth.one_hot_bf16(ks, K), DEV)))
    torch.cuda.synchronize()
    assert np.array_equal(canon_zero(got), canon_zero(o.to_bf16_bits(c.W()[:, ks].T))), what + ": decoded weights differ"
