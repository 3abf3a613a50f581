"""Pins for the oracle's encoder (Alg. 1, Eq. 1, Eq. 4): exhaustive search on
tiny inputs, special cases that reduce to element-wise rounding, round trips,
numpy least squares.  CPU only."""
import numpy as np
import pytest

from oracle import ccq_oracle as o
from paper_2507_07145_amd import synth

CFGS = [o.Code(2, 3, 1), o.Code(4, 3, 2), o.Code(3, 3, 2), o.Code(3, 4, 2), o.Code(6, 4, 3)]


def _numpy_argmin(v, s, cfg):
    """Alg. 1's argmin written with the explicit codebook (numpy, independent of the C search)."""
    cb = o.codebook(cfg).astype(np.float64)
    cost = np.zeros(cb.shape[0])
    for i in range(cfg.N):                                       # left-to-right, like the definition
        cost = cost + (v[i] - s * (cb[:, i] - cfg.zero_point)) ** 2
    return int(np.argmin(cost))                                  # first minimum = lowest code


@pytest.mark.parametrize("cfg", CFGS)
def test_search_brute_equals_numpy_codebook_argmin_and_viterbi(cfg):
    rng = np.random.default_rng(cfg.L * 100 + cfg.N)
    s = 0.37
    n = 12 if cfg.T >= 15 else 150
    for t in range(n):
        v = rng.standard_normal(cfg.N) * s * (1 << (cfg.L - 1)) * 0.6
        if t % 5 == 0:                                           # exact ties: midpoints between levels / zeros
            v = (rng.integers(-2, 3, cfg.N) + 0.5) * s
        if t % 7 == 0:
            v[:] = 0.0
        want = _numpy_argmin(v, s, cfg)
        assert o.search(v, s, cfg, "brute") == want
        assert o.search(v, s, cfg, "viterbi") == want


def test_viterbi_equals_brute_many_f2_vectors():
    rng = np.random.default_rng(11)
    for _ in range(40):
        v = rng.standard_normal(4) * 0.02
        s = float(np.float16(np.abs(v).max() / 31 * rng.uniform(0.5, 2.0)))
        assert o.search(v, s, o.F2, "viterbi") == o.search(v, s, o.F2, "brute")


def test_search_no_overlap_is_elementwise_rounding():
    """S = L: every state is free, so the best code rounds each entry on its own."""
    cfg = o.Code(4, 2, 4)
    rng = np.random.default_rng(12)
    for _ in range(200):
        s = rng.uniform(0.1, 1.0)
        v = rng.standard_normal(2) * 6 * s
        st = np.clip(np.rint(v / s + 8), 0, 15).astype(int)
        # (no exact .5 ties with random reals)
        assert o.search(v, s, cfg, "viterbi") == (st[0] << 4 | st[1])


@pytest.mark.parametrize("cfg", CFGS)
def test_fixed_scale_round_trip(cfg):
    """code -> vector is injective, so encoding a decoded vector returns the code."""
    rng = np.random.default_rng(13)
    s = 0.125
    for c in rng.integers(0, 1 << cfg.T, 60):
        v = (np.array(o.states(int(c), cfg), dtype=np.float64) - cfg.zero_point) * s
        assert o.search(v, s, cfg, "viterbi") == int(c)


def test_refit_scale_is_least_squares():
    rng = np.random.default_rng(14)
    wq = rng.integers(-32, 32, 64).astype(np.float64)
    w = wq * 0.013 + rng.standard_normal(64) * 1e-3
    s = o.refit_scale(w, wq)
    ls = np.linalg.lstsq(wq[:, None], w, rcond=None)[0][0]       # Eq. 4 is the normal equation of this
    assert abs(s - ls) < 1e-12
    for t in (0.9, 1.1):
        assert np.sum((w - wq * s) ** 2) <= np.sum((w - wq * s * t) ** 2)
    assert o.refit_scale(w, np.zeros(64), fallback=7.0) == 7.0


def _err(W, fmt, out, gf=None):
    codes, scales, alpha, beta = out
    return float(np.sum((o.decode(W.shape[1], W.shape[0], fmt, codes, scales, alpha, beta, gf) - W) ** 2))


def test_quantize_brute_equals_viterbi_tiny():
    rng = np.random.default_rng(15)
    W = synth.weights_normal(2, 64, rng)
    for fmt in (o.F275, o.F2):
        a = o.quantize(W, fmt, method="brute")
        b = o.quantize(W, fmt, method="viterbi")
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_quantize_f275_round_trip_quality():
    rng = np.random.default_rng(16)
    W = synth.weights_normal(8, 256, rng)
    out = o.quantize(W, o.F275)
    assert out[0].shape == (8, 4 * 22)
    e = _err(W.astype(np.float64), o.F275, out)
    # 8 bits per 3 Gaussian weights: the rate-distortion bound is 2^(-2*8/3) = 2.5 % relative error,
    # a practical code with abs-max scaling lands within a few times that
    assert 0.025 < e / float(np.sum(W.astype(np.float64) ** 2)) < 0.15
    # every stored code is the best one for the stored scale: re-searching a group changes nothing
    codes, scales = out[0], o.fp16_bits_to_f64(out[1])
    for n, g in ((0, 0), (3, 2), (7, 3)):
        for j in range(21):
            v = W[n, 64 * g + 3 * j: 64 * g + 3 * j + 3].astype(np.float64)
            assert o.search(v, scales[n, g], o.F275, "brute") == codes[n, 22 * g + j]


def test_quantize_f2_cluster_properties():
    rng = np.random.default_rng(17)
    W = synth.weights_normal(6, 512, rng)
    plain = o.quantize(W, o.F2, cluster_research=False)
    best = o.quantize(W, o.F2, cluster_research=True)
    W64 = W.astype(np.float64)
    e_plain, e_best = _err(W64, o.F2, plain), _err(W64, o.F2, best)
    assert e_best <= e_plain                                      # Eq. 1's own code is one of the candidates
    assert e_best < float(np.sum(W64 ** 2))                       # better than storing zeros
    for out in (plain, best):
        codes, scales, alpha, beta = out
        assert codes.shape == (6, 512 // 4) and scales.shape == (6, 8)
        assert np.all(beta == np.floor(beta)) and np.all(beta >= 0) and np.all(alpha >= 0)
        assert np.all(255.0 * alpha.astype(np.float64) + beta < 2 ** 15)
        assert np.all(o.fp16_bits_to_f64(scales) > 0)
    # Eq. 1: with the unconstrained codes c, q = round((c - beta)/alpha) spans [0,255] on each row
    assert plain[0].min() == 0 and plain[0].max() == 255


def test_quantize_hybrid_map():
    rng = np.random.default_rng(18)
    W = synth.weights_normal(3, 256, rng)
    gf = np.array([0, 1, 0, 1], dtype=np.uint8)
    out = o.quantize(W, (o.F2, o.F275), gf)
    assert out[0].shape == (3, 2 * 16 + 2 * 22)
    wide_only = o.quantize(W[:, 64:128], o.F275)
    # the wide groups are quantized exactly as they would be on their own
    assert np.array_equal(out[0][:, 16:38], wide_only[0]) and np.array_equal(out[1][:, 1:2], wide_only[1])
    assert _err(W.astype(np.float64), (o.F2, o.F275), out, gf) < float(np.sum(W.astype(np.float64) ** 2))
