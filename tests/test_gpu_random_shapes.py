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


def _ragged_draw(rng):
    family = ["narrow", "wide", "mixed", "h16"][int(rng.integers(0, 4))]
    mode = int(rng.integers(0, 2))
    G = int(rng.integers(2, 41))
    n_wide = int(rng.integers(1, G)) if family == "mixed" else None
    N = int(rng.integers(1, 600)) if rng.random() < 0.8 else int(rng.integers(600, 2600))
    M = int(rng.choice([1, 1, 2, 3, 5, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200]))
    return family, mode, 64 * G, N, M, n_wide


def _ragged_arrays(family, mode, K, N, gf, rng):
    """Canonical arrays of one random matrix in any format and scale mode, and its oracle-decoded weights."""
    G = K // 64
    a = {"scales": None, "sq": None, "ssup": None, "alpha": None, "beta": None}
    if mode == 1:
        a["ssup"] = (o.fp16_bits_to_f64(synth.scales_log_uniform_fp16(N, 1, rng).reshape(N)) * 0.1).astype(np.float16).view(np.uint16)
    else:
        a["scales"] = synth.scales_log_uniform_fp16(N, G, rng)
    if family == "h16":
        a["codes"] = synth.random_codes(N, o.h16_row_bytes(K), rng)
        a["W"] = o.h16_decode(K, N, a["codes"], a["scales"]) if mode == 0 else o.h16_decode_cs(K, N, a["codes"], a["ssup"])
        return a
    ofmt = {"narrow": o.F2, "wide": o.F275, "mixed": (o.F2, o.F275)}[family]
    a["codes"] = synth.random_codes(N, o.row_bytes(K, ofmt, gf), rng)
    if family != "wide":
        a["alpha"], a["beta"] = synth.cluster_params(N, rng)
    if mode == 0:
        a["W"] = o.decode(K, N, ofmt, a["codes"], a["scales"], a["alpha"], a["beta"], gf)
    else:
        nb = o.sq_row_bytes(K, ofmt, gf)
        a["sq"] = rng.integers(0, 256, size=(N, max(nb, 1)), dtype=np.uint8)[:, :nb]
        a["W"] = o.decode_cs(K, N, ofmt, a["codes"], a["sq"], a["ssup"], a["alpha"], a["beta"], gf)
    return a


def _upload(family, mode, K, N, gf, parts):
    """Device weight of one matrix (`parts` = one set of arrays) or of a stack of experts (a list of sets)."""
    bfmt = {"narrow": [b.NARROW], "wide": [b.WIDE], "mixed": [b.NARROW, b.WIDE], "h16": b.H16}[family]
    experts = len(parts) if isinstance(parts, list) else None

    def get(key):
        if experts is None:
            return parts[key]
        return None if parts[0][key] is None else np.stack([p[key] for p in parts])
    if mode == 0:
        return b.Weight.from_canonical(K, N, bfmt, get("codes"), get("scales"), get("alpha"), get("beta"), gf, device=DEV, experts=experts)
    return b.Weight.from_canonical_compressed(K, N, bfmt, get("codes"), get("sq"), get("ssup"), get("alpha"), get("beta"), gf, device=DEV,
                                              experts=experts)


def _ragged_weight(family, mode, K, N, n_wide, seed):
    rng = synth.rng(41, seed)
    gf = synth.group_format_map(K // 64, n_wide, rng) if family == "mixed" else None
    a = _ragged_arrays(family, mode, K, N, gf, rng)
    return _upload(family, mode, K, N, gf, a), a["W"]


@pytest.mark.parametrize("seed", range(160))
def test_random_ragged_case(seed):
    """Any K that is a multiple of the group size (Sec. 3.1), any N, any per-group format map (Sec. 3.3), the hybrid word
    (Sec. 3.2) and both scale modes (Sec. 3.4), drawn at random: the product within tolerance, the decoded weights bit
    for bit, and nothing written outside the M x N result."""
    rng = np.random.default_rng(2000 + seed)
    family, mode, K, N, M, n_wide = _ragged_draw(rng)
    what = f"seed {seed}: {family} scale mode {mode} K={K} N={N} M={M} wide groups {n_wide}"
    print(what, flush=True)
    w, W = _ragged_weight(family, mode, K, N, n_wide, seed)
    ld = (N + 7) // 8 * 8 + 8

    def run(x_bits):
        y = torch.full((M + 1, ld), 3.140625, dtype=torch.bfloat16, device=DEV)
        b.gemm(w, b.bf16_tensor(x_bits, DEV), out=y[:M, :N])
        torch.cuda.synchronize()
        bits = b.bf16_bits(y)
        assert np.all(bits[:M, N:] == 0x4049) and np.all(bits[M] == 0x4049), what + ": written outside the result"
        return bits[:M, :N]

    x = synth.activations_bf16(M, K, synth.rng(41, 1000 + seed))
    assert_gemm_close(run(x), o.matmul(x, W), what, rounded=(x, W) if M > 16 else None)
    ks = rng.integers(0, K, M)
    ks[:min(M, 3)] = [K - 1, 0, K - 64][:min(M, 3)]
    assert np.array_equal(canon_zero(run(synth.one_hot_bf16(ks, K))), canon_zero(o.to_bf16_bits(W[:, ks].T))), what + ": decoded weights differ"


@pytest.mark.parametrize("seed", range(48))
def test_random_ragged_grouped_case(seed):
    """The same through the grouped entry point (Sec. 4.2, Table 5): a random number of experts with random row
    counts, zero included, with and without the host copy of the offsets."""
    from cases import grouped_rounded_weight_sigma
    rng = np.random.default_rng(3000 + seed)
    family = ["narrow", "wide", "mixed", "h16"][int(rng.integers(0, 4))]
    mode = int(rng.integers(0, 2))
    G = int(rng.integers(2, 25))
    K, N, E, T = 64 * G, int(rng.integers(1, 300)), int(rng.integers(2, 9)), 50
    most = int(rng.choice([1, 4, 16, 17, 40, 130]))
    counts = [int(min(most, c)) for c in rng.choice([0, 0, 1, 1, 2, 5, 16, 17, 33, 40, 70, 130], size=E)]
    if sum(counts) == 0:
        counts[0] = 1
    what = f"seed {seed}: grouped {family} scale mode {mode} K={K} N={N} rows per expert {counts}"
    print(what, flush=True)
    wrng = synth.rng(42, seed)
    gf = synth.group_format_map(G, int(rng.integers(1, G)), wrng) if family == "mixed" else None
    parts = [_ragged_arrays(family, mode, K, N, gf, wrng) for _ in range(E)]
    w = _upload(family, mode, K, N, gf, parts)
    x = synth.activations_bf16(T, K, synth.rng(42, 1000 + seed))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    P = int(offs[-1])
    rows = rng.integers(0, T, size=P).astype(np.int32)
    ref = np.concatenate([o.matmul(x[rows[offs[e]:offs[e + 1]]], parts[e]["W"]) for e in range(E) if counts[e] > 0])
    sigma = grouped_rounded_weight_sigma(x, rows, offs, lambda e: parts[e]["W"])
    ld = (N + 7) // 8 * 8 + 8
    for host_offsets in (offs, None):
        y = torch.full((P + 1, ld), 3.140625, dtype=torch.bfloat16, device=DEV)
        b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), host_offsets, out=y[:P, :N])
        torch.cuda.synchronize()
        bits = b.bf16_bits(y)
        assert np.all(bits[:P, N:] == 0x4049) and np.all(bits[P] == 0x4049), what + ": written outside the result"
        assert_gemm_close(bits[:P, :N], ref, what + f", host offsets {'given' if host_offsets is not None else 'absent'}", rounded=sigma)


@pytest.mark.parametrize("family,G,N,counts,what", [("narrow", 8, 7168, [1, 0, 0, 1, 1, 0, 1, 1, 1, 0, 1, 1], "one row per expert, shares of two k-tiles (Table 5, N x K = 7168 x 512)"),
                                             ("narrow", 112, 1000, [0, 1, 1, 0, 1], "one row, 14 shares of two, ragged N"),
                                             ("narrow", 15, 40, [1, 1, 1], "one row, every expert has rows, ragged K"),
                                             ("narrow", 84, 72, [1, 0, 1], "one row, shares of three"),
                                             ("narrow", 112, 1024, [1, 4, 0, 2, 3, 1, 0, 1], "up to four rows (Table 5, 1024 x 7168)"),
                                             ("narrow", 8, 1000, [2, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 1, 0, 0, 3], "up to four rows, most experts without rows"),
                                             ("narrow", 132, 64, [4, 4], "four rows, 11 shares of three"),
                                             ("narrow", 16, 200, [1, 2, 9, 1, 0, 1, 3, 1, 2, 1, 1, 1], "one expert with nine rows: the general kernel"),
                                             ("narrow", 144, 64, [4, 1, 2], "36 k-tiles: one workgroup per CU"),
                                             ("narrow", 268, 32, [3, 1], "67 k-tiles: four rows do not fit the LDS, the general kernel"),
                                             ("wide", 16, 1000, [1, 0, 1, 1, 0, 0, 1], "wide format, one row per expert, shares of two k-tiles"),
                                             ("wide", 13, 40, [1, 1], "wide format, ragged last k-tile, every expert has a row"),
                                             ("mixed", 24, 200, [0, 1, 1, 0, 1], "per-group mix, one row per expert"),
                                             ("mixed", 112, 72, [1, 0, 0, 1], "per-group mix, 14 k-tiles"),
                                             ("h16", 16, 300, [1, 0, 1, 1], "hybrid word, one row per expert"),
                                             ("h16", 17, 40, [1, 1, 0], "hybrid word, ragged last k-tile"),
                                             ("wide", 16, 200, [1, 2, 0, 1], "wide format, two rows on one expert: the general kernel")])
@pytest.mark.parametrize("mode", [0, 1])
def test_grouped_product_with_few_rows_per_expert(family, G, N, counts, what, mode):
    """The Grouped-GEMM operator of Table 5 at one and four tokens: every expert that has rows is a GEMV or a four-row
    product of its own.  With and without the host copy of the offsets (without it the library only knows the total),
    both scale modes, gathered activation rows, experts without rows; products within tolerance and decoded weights
    bit for bit through one-hot rows."""
    K, E, T = 64 * G, len(counts), 9
    wrng = synth.rng(43, G + N + mode)
    gf = synth.group_format_map(G, max(1, G // 3), wrng) if family == "mixed" else None
    parts = [_ragged_arrays(family, mode, K, N, gf, wrng) for _ in range(E)]
    w = _upload(family, mode, K, N, gf, parts)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    P = int(offs[-1])
    rows = synth.rng(43, 7).integers(0, T, size=P).astype(np.int32)
    ld = (N + 7) // 8 * 8 + 8
    x = synth.activations_bf16(T, K, synth.rng(43, 8))
    hot = synth.one_hot_bf16(synth.rng(43, 9).integers(0, K, T), K)
    hot_cols = np.argmax(hot != 0, axis=1)
    for xb, exact in ((x, False), (hot, True)):
        for host_offsets in (offs, None):
            y = torch.full((P + 1, ld), 3.140625, dtype=torch.bfloat16, device=DEV)
            b.grouped_gemm(w, b.bf16_tensor(xb, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), host_offsets, out=y[:P, :N])
            torch.cuda.synchronize()
            bits = b.bf16_bits(y)
            assert np.all(bits[:P, N:] == 0x4049) and np.all(bits[P] == 0x4049), what + ": written outside the result"
            for e in range(E):
                for p in range(offs[e], offs[e + 1]):
                    if exact:
                        want = o.to_bf16_bits(parts[e]["W"][:, hot_cols[rows[p]]])
                        assert np.array_equal(canon_zero(bits[p, :N]), canon_zero(want)), f"{what}: decoded weights of expert {e} differ (row {p})"
                    else:
                        assert_gemm_close(bits[p:p + 1, :N], o.matmul(xb[rows[p]:rows[p] + 1], parts[e]["W"]), f"{what}, expert {e} row {p}")
