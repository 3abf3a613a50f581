"""Pins of the oracle's hybrid-word format (Sec. 3.2 "Hybrid Encoding"; Table 1 row "(3,3,2)(3,4,2)").

Fixed from outside: Table 1's printed shift list and mask (tests/golden), the printed bit widths 2.28 and 2.5, the
generic single-code routines that the other pins fix (the word is two independent codes side by side), a group decoded
by hand, exhaustive search on tiny inputs."""
import numpy as np
import pytest

from conftest import golden
from oracle import ccq_oracle as o
from paper_2507_07145_amd import synth


def _table1_hybrid():
    for name, wmask, smask, shifts, cluster in golden("table1_shifts.txt"):
        if name == "hybrid":
            return int(wmask, 16), int(smask, 16), [int(v) for v in shifts.split(",")]
    raise AssertionError("fixture row missing")


def test_states_follow_table1_shift_list():
    wmask, smask, shifts = _table1_hybrid()
    assert (wmask, smask, shifts) == (0x7, 0x1FFF, [13, 11, 9, 6, 4, 2, 0])
    rng = np.random.default_rng(11)
    for word in [0, 0xFFFF, 0x8001, 0x1234] + [int(v) for v in rng.integers(0, 1 << 16, 200)]:
        assert o.h16_states(word) == [(word >> s) & wmask for s in shifts]
        # the same seven states from the two single-code definitions
        assert o.h16_states(word) == o.states(word >> 9, o.Code(3, 3, 2)) + o.states(word & 0x1FF, o.Code(3, 4, 2))
    # T = L + (N-1) S of the two codes fills the word exactly
    assert o.T(o.Code(3, 3, 2)) + o.T(o.Code(3, 4, 2)) == 16


def test_bit_widths_of_sec_3_2_and_3_4():
    assert int(16 / 7 * 100) / 100 == 2.28                # seven values in 16 bits (printed truncated)
    assert o.h16_row_bytes(64) == 20                      # 10 words for 64 weights
    assert o.h16_row_bytes(64) * 8 / 64 == 2.5            # "an equivalent bpw of 2.5"
    assert 10 * 16 - (9 * 16 + 3) == 13                   # weight 63 uses 3 bits of the last word: 13 spare bits (scale mask 0x1FFF)


def test_decode_by_hand():
    K = 64
    words = np.zeros(10, dtype=np.uint16)
    words[0] = (0b101 << 13) | (0b01 << 11) | (0b10 << 9) | (0b011 << 6) | (0b00 << 4) | (0b11 << 2) | 0b01
    # code A = 101 01 10 -> states 101, 101 (low bit of 101, then 01) ... written out with the shift list instead:
    want0 = [(int(words[0]) >> s) & 7 for s in (13, 11, 9, 6, 4, 2, 0)]
    words[9] = 0b110 << 13 | 0x1ABC                       # weight 63 = state 6; the 13 spare bits are ignored
    codes = words.view(np.uint8).reshape(1, 20)
    scales = np.array([[np.float16(0.5).view(np.uint16)]], dtype=np.uint16)
    W = o.h16_decode(K, 1, codes, scales)
    assert list(W[0, :7]) == [(s - 4) * 0.5 for s in want0]
    assert W[0, 63] == (6 - 4) * 0.5
    assert np.all(W[0, 7:63] == (0 - 4) * 0.5)
    words[9] = 0b110 << 13                                # spare bits do not matter
    assert np.array_equal(o.h16_decode(K, 1, words.view(np.uint8).reshape(1, 20), scales), W)


def test_quantize_round_trip_and_search():
    rng = synth.rng(1, 800)
    N, K = 8, 256
    W = synth.weights_normal(N, K, rng)
    codes, scales = o.h16_quantize(W)
    codes_b, scales_b = o.h16_quantize(W, method="brute")
    assert np.array_equal(codes, codes_b) and np.array_equal(scales, scales_b)     # dynamic program == exhaustive search
    Wd = o.h16_decode(K, N, codes, scales)
    rel = np.linalg.norm(Wd - W) / np.linalg.norm(W)
    assert 0.1 < rel < 0.6                                                          # 3-bit states at 2.5 bpw: coarse but sane
    # every stored word is the best word for its 7 weights under the stored scale (checked exhaustively on a sample)
    s = o.fp16_bits_to_f64(scales)
    words = codes.view(np.uint16).reshape(N, K // 64, 10)
    for (n, g, j) in [(0, 0, 0), (3, 2, 4), (7, 3, 8)]:
        v = W[n, 64 * g + 7 * j: 64 * g + 7 * j + 7].astype(np.float64)
        best = min(range(1 << 16), key=lambda c: (sum((v[i] - s[n, g] * (st - 4.0)) ** 2 for i, st in enumerate(o.h16_states(c))), c))
        got = int(words[n, g, j])
        err = lambda c: sum((v[i] - s[n, g] * (st - 4.0)) ** 2 for i, st in enumerate(o.h16_states(c)))
        assert err(got) <= err(best) * (1 + 1e-12)
    # an all-zero group gets scale 0 and decodes to zeros
    W[2, 64:128] = 0
    c2, s2 = o.h16_quantize(W)
    assert np.all(o.h16_decode(K, N, c2, s2)[2, 64:128] == 0)


# ---------------------------------------------------------------- Sec. 3.4 on the hybrid word


def _fp16(x: float) -> int:
    return int(np.float16(x).view(np.uint16))


def test_scale_field_by_hand():
    """Alg. 2: s = (last word & 0x1FFF) * s_super; Table 1 gives the mask.  Last word 0xDABC: weight 63 has state 6,
    the field is 0x1ABC = 6844."""
    words = np.zeros(10, dtype=np.uint16)
    words[0] = 0x8000                                     # first weight: state 4 -> value 0; the others state 0 -> -4 s
    words[9] = 0xDABC
    codes = words.view(np.uint8).reshape(1, 20)
    ssup = np.array([_fp16(2.0 ** -10)], dtype=np.uint16)
    sc = o.h16_expand_scales(64, 1, codes, ssup)
    assert sc[0, 0] == 6844 * 2.0 ** -10
    W = o.h16_decode_cs(64, 1, codes, ssup)
    assert W[0, 0] == 0.0 and W[0, 1] == -4 * 6844 * 2.0 ** -10 and W[0, 63] == (6 - 4) * 6844 * 2.0 ** -10
    # the field does not leak into weight 63 and the weight does not leak into the field
    words[9] = 0xC000 | 0x1ABC
    assert o.h16_expand_scales(64, 1, words.view(np.uint8).reshape(1, 20), ssup)[0, 0] == sc[0, 0]
    words[9] = 0xC000 | 0x1001
    assert o.h16_decode_cs(64, 1, words.view(np.uint8).reshape(1, 20), ssup)[0, 63] == (6 - 4) * 0x1001 * 2.0 ** -10


def test_power_of_two_super_scale_reduces_to_fp16_scales():
    """Fields below 2^11 times s_super = 2^-14 are fp16 numbers: the compressed-scale decoder must then agree bit for bit
    with the fp16-scale decoder (pinned above) fed those numbers."""
    rng = synth.rng(1, 810)
    K, N = 512, 12
    codes = synth.random_codes(N, o.h16_row_bytes(K), rng).reshape(N, K // 64, 10, 2)
    codes[:, :, 9, 1] &= 0xE7                              # clear field bits 11 and 12: fields < 2048
    codes = codes.reshape(N, -1)
    ssup = np.full(N, _fp16(2.0 ** -14), dtype=np.uint16)
    sc = o.h16_expand_scales(K, N, codes, ssup)
    assert sc.max() < 2048 * 2.0 ** -14 and np.array_equal(sc.astype(np.float16).astype(np.float64), sc)
    W1 = o.h16_decode_cs(K, N, codes, ssup)
    W0 = o.h16_decode(K, N, codes, sc.astype(np.float16).view(np.uint16))
    assert np.array_equal(W1, W0)


def test_encoder_side_of_scale_compression():
    rng = synth.rng(1, 820)
    N, K = 8, 256
    W = synth.weights_normal(N, K, rng)
    W[5] = 0.0
    codes, scales = o.h16_quantize(W)
    c2, ssup = o.h16_compress_scales(W, codes, scales)
    s16, sup = o.fp16_bits_to_f64(scales), o.fp16_bits_to_f64(ssup)
    assert np.array_equal(ssup, (s16.max(axis=1) / 8191.0).astype(np.float16).view(np.uint16))
    fields = c2.view(np.uint16).reshape(N, K // 64, 10)[:, :, 9] & 0x1FFF
    nz = sup > 0
    assert np.array_equal(fields[nz], np.clip(np.rint(s16[nz] / sup[nz][:, None]), 1, 8191).astype(np.uint16))
    assert np.all(fields[~nz] == 0) and fields.max() >= 8190
    W_new = o.h16_decode_cs(K, N, c2, ssup)
    assert np.all(W_new[5] == 0)
    # 13-bit scales cost next to nothing against fp16 scales
    W_fp16 = o.h16_decode(K, N, codes, scales)
    assert np.linalg.norm(W_new - W) <= 1.001 * np.linalg.norm(W_fp16 - W)
    # searching again with the stored scale is never worse than keeping the old words with it
    keep = codes.view(np.uint16).reshape(N, K // 64, 10).copy()
    keep[:, :, 9] = (keep[:, :, 9] & 0xE000) | fields
    W_keep = o.h16_decode_cs(K, N, keep.view(np.uint8).reshape(N, -1), ssup)
    e_new = ((W_new - W) ** 2).reshape(N, K // 64, 64).sum(axis=2)
    e_keep = ((W_keep - W) ** 2).reshape(N, K // 64, 64).sum(axis=2)
    assert np.all(e_new <= e_keep * (1 + 1e-12) + 1e-30)
