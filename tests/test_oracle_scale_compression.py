"""Pins of the oracle's compressed-scale path (Sec. 3.4 "Scale Compression"; first line of Alg. 2 and of Alg. 3).

What fixes it without another implementation: the bit positions the paper states (the spare 4 bits of the 22nd code
of a 64-weight (L=4,N=3,S=2) group; s_q >> s_shift & s_mask), the printed totals 2.75 and 2.06 bpw, values computed by
hand, and the special case of a power-of-two super scale, where the path must agree with the fp16-scale decoder that
the other pins already fix."""
import numpy as np
import pytest

from oracle import ccq_oracle as o
from paper_2507_07145_amd import synth


def _fp16(x: float) -> int:
    return int(np.float16(x).view(np.uint16))


def test_where_the_four_bits_live():
    # Sec. 3.4: 22 codes for 64 weights under (4,3,2); only the first 4 bits of the last one are valid
    assert o.spare_bits(o.F275, 64) == 4
    assert o.group_bytes(o.F275, 64) == 22
    # Code Cluster: "redundant bits cannot be utilized": the scales get an array of their own, 4 bits per group
    assert o.spare_bits(o.F2, 64) == 0
    assert o.sq_row_bytes(8192, o.F2) == 8192 // 64 // 2
    assert o.sq_row_bytes(8192, o.F275) == 0
    gf = np.array([0, 1, 0, 0, 1, 0, 0, 0], dtype=np.uint8)   # 6 narrow groups -> 3 bytes
    assert o.sq_row_bytes(512, (o.F2, o.F275), gf) == 3


def test_equivalent_bit_widths_of_sec_3_4():
    # 2.75 bpw: the scale rides in the spare bits, nothing is added; 2.06 bpw: 2.0 + 4/64
    assert o.bpw(8, 64, 3, 0) == pytest.approx(2.75, abs=0)
    assert o.bpw(8, 64, 4, 4) == pytest.approx(2.0625, abs=0)
    assert (o.group_bytes(o.F2, 64) * 8 + 4) / 64 == 2.0625
    assert round(2.0625, 2) == 2.06


def test_alg2_scale_field_by_hand():
    """One row, one (4,3,2) group.  Byte 21 = 0xB7: weight 63 has state 0xB, the scale field is 7."""
    codes = np.zeros((1, 22), dtype=np.uint8)
    codes[0, 0] = 0b1001_0110      # states (c>>4)&15, (c>>2)&15, c&15 = 9, 5, 6
    codes[0, 21] = 0xB7
    ssup = np.array([_fp16(0.25)], dtype=np.uint16)
    sc = o.expand_scales(64, 1, o.F275, codes, None, ssup)
    assert sc.shape == (1, 1) and sc[0, 0] == 7 * 0.25
    W = o.decode_cs(64, 1, o.F275, codes, None, ssup)
    assert list(W[0, :3]) == [(9 - 8) * 1.75, (5 - 8) * 1.75, (6 - 8) * 1.75]
    assert W[0, 63] == (0xB - 8) * 1.75
    assert W[0, 3] == (0 - 8) * 1.75          # an all-zero code decodes to state 0
    # the field does not leak into the weights: changing it only rescales
    codes2 = codes.copy()
    codes2[0, 21] = 0xB1
    W2 = o.decode_cs(64, 1, o.F275, codes2, None, ssup)
    assert np.array_equal(W2 * 7, W)


def test_alg3_shift_and_mask_by_hand():
    """Two Code Cluster groups of one row share the byte 0xA3 of s_q: fields 3 (s_shift 0) and 10 (s_shift 4)."""
    K = 128
    codes = np.zeros((1, 32), dtype=np.uint8)
    codes[0, 0] = 0x55            # alpha = 128, beta = 0: c = q << 7 = 0x2A80 -> states 21, 21, 16, 0 ... by the shifts 9,6,3,0
    codes[0, 16] = 0xFF           # c = 0x7F80 -> states 63, 62, 48, 0
    sq = np.array([[0xA3]], dtype=np.uint8)
    ssup = np.array([_fp16(0.5)], dtype=np.uint16)
    al, be = np.array([128.0], dtype=np.float32), np.array([0.0], dtype=np.float32)
    sc = o.expand_scales(K, 1, o.F2, codes, sq, ssup)
    assert list(sc[0]) == [3 * 0.5, 10 * 0.5]
    c0, c1 = 0x55 << 7, 0xFF << 7
    st0 = [(c0 >> s) & 63 for s in (9, 6, 3, 0)]
    st1 = [(c1 >> s) & 63 for s in (9, 6, 3, 0)]
    W = o.decode_cs(K, 1, o.F2, codes, sq, ssup, al, be)
    assert list(W[0, :4]) == [(s - 32) * 1.5 for s in st0]
    assert list(W[0, 64:68]) == [(s - 32) * 5.0 for s in st1]


@pytest.mark.parametrize("kinds", [("narrow",), ("wide",), ("narrow", "wide")])
def test_power_of_two_super_scale_reduces_to_fp16_scales(kinds):
    """With s_super = 2^-6 every product field * s_super is an fp16 number, and the compressed-scale decoder must agree
    bit for bit with the fp16-scale decoder fed those numbers."""
    rng = synth.rng(1, 700 + len(kinds))
    K, N = 1024, 24
    G = K // 64
    fm = {"narrow": o.F2, "wide": o.F275}
    fmt = fm[kinds[0]] if len(kinds) == 1 else (o.F2, o.F275)
    gf = None
    if len(kinds) == 2:
        gf = synth.group_format_map(G, 6, rng)
    codes = synth.random_codes(N, o.row_bytes(K, fmt, gf), rng)
    nb = o.sq_row_bytes(K, fmt, gf)
    sq = rng.integers(0, 256, size=(N, max(nb, 1)), dtype=np.uint8)[:, :nb]
    ssup = np.full(N, _fp16(2.0 ** -6), dtype=np.uint16)
    alpha, beta = synth.cluster_params(N, rng)
    sc = o.expand_scales(K, N, fmt, codes, sq, ssup, gf)
    assert np.all(sc * 64 == np.round(sc * 64)) and sc.min() >= 0 and sc.max() <= 15 / 64
    as_fp16 = sc.astype(np.float16)
    assert np.array_equal(as_fp16.astype(np.float64), sc)
    W1 = o.decode_cs(K, N, fmt, codes, sq, ssup, alpha, beta, gf)
    W0 = o.decode(K, N, fmt, codes, as_fp16.view(np.uint16), alpha, beta, gf)
    assert np.array_equal(W1, W0)
    # exact in fp32: 4-bit field x 11-bit super scale x (<= 7-bit state difference)
    assert np.array_equal(W1.astype(np.float32).astype(np.float64), W1)


@pytest.mark.parametrize("fmt", [o.F2, o.F275])
def test_encoder_side(fmt):
    rng = synth.rng(1, 720)
    K, N = 512, 16
    W = synth.weights_normal(N, K, rng)
    W[3] = 0.0                                       # an all-zero row
    codes, scales, alpha, beta = o.quantize(W, fmt)
    c2, sq, ssup = o.compress_scales(W, fmt, codes, scales, alpha, beta)
    s16 = o.fp16_bits_to_f64(scales)
    sup = o.fp16_bits_to_f64(ssup)
    # channel-wise super scale: the largest group scale of the row maps to the largest field
    assert np.array_equal(ssup, (s16.max(axis=1) / 15.0).astype(np.float16).view(np.uint16))
    sc = o.expand_scales(K, N, fmt, c2, sq, ssup)
    fields = np.round(sc / np.where(sup > 0, sup, 1.0)[:, None])
    assert fields.min() >= 0 and fields.max() <= 15 and fields.max() == 15
    nz = sup > 0
    assert np.all(fields[nz] >= 1) and np.all(fields[~nz] == 0) and np.all(s16[~nz] == 0)
    # nearest multiple of the super scale (fields clipped to 1..15)
    want = np.clip(np.rint(s16[nz] / sup[nz][:, None]), 1, 15)
    assert np.array_equal(fields[nz], want)
    # searching again with the stored scales is never worse than keeping the old codes with them
    W_new = o.decode_cs(K, N, fmt, c2, sq, ssup, alpha, beta)
    keep = codes.copy()
    if fmt is o.F275:                                 # old codes, new fields in the spare nibbles
        keep = keep.reshape(N, K // 64, 22)
        keep[:, :, 21] = (keep[:, :, 21] & 0xF0) | (c2.reshape(N, K // 64, 22)[:, :, 21] & 0x0F)
        keep = keep.reshape(N, -1)
    W_keep = o.decode_cs(K, N, fmt, keep, sq, ssup, alpha, beta)
    e_new = ((W_new - W) ** 2).reshape(N, K // 64, 64).sum(axis=2)
    e_keep = ((W_keep - W) ** 2).reshape(N, K // 64, 64).sum(axis=2)
    assert np.all(e_new <= e_keep * (1 + 1e-12) + 1e-30)
    # and the 4-bit scales cost little against fp16 scales
    W_fp16 = o.decode(K, N, fmt, codes, scales, alpha, beta)
    assert np.linalg.norm(W_new - W) <= 1.15 * np.linalg.norm(W_fp16 - W)
    assert np.all(W_new[3] == 0)
