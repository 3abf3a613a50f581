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
