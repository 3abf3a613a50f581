"""Host-side checks of the C ABI that need no GPU: the library loads and exports every
declared symbol, the layout accounting follows Eq. 5, the pack routines are the documented
byte permutations, and bad arguments come back as error codes."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = b.load()
    header = open(os.path.join(ROOT, "include", "ccq.h")).read()
    declared = set(re.findall(r"\b(ccq_[a-z_0-9]+)\s*\(", header))
    assert {"ccq_pack_info", "ccq_gemm", "ccq_grouped_gemm"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(b.EXPORTS)
    assert lib.ccq_status_string(-6) == b"CCQ_ERR_ROUTING"


def test_pack_info_accounting_matches_eq5_and_oracle():
    for kinds, fmt, bpw in (([b.NARROW], o.F2, 2.0), ([b.WIDE], o.F275, 2.75)):
        w = b.descriptor(8192, 8192, kinds)
        i = b.pack_info(w, 16)
        assert i.code_bpw == bpw == o.bpw(8, 64, fmt.N, 0)
        assert i.code_bytes == 8192 * o.row_bytes(8192, fmt)              # device order stores exactly the canonical bytes
        assert i.bytes_per_group[0] == o.group_bytes(fmt) and i.scale_bytes == 8192 * 128 * 2
        assert i.align == 16 and i.meta_bytes == 128 * 4
    # per-group mix: 32 of 128 groups wide -> (96*16 + 32*22) bytes per row = 2.1875 bpw
    gf = synth.group_format_map(128, 32, synth.rng(3, 0))
    w = b.descriptor(8192, 28672, [b.NARROW, b.WIDE], gf)
    i = b.pack_info(w, 64)
    assert i.code_bpw == 2.1875 and list(i.groups) == [96, 32]
    assert i.code_bytes == 28672 * o.row_bytes(8192, (o.F2, o.F275), gf) == 64225280
    assert i.total_bpw == 8.0 * (i.code_bytes + i.scale_bytes + 8 * 28672) / (28672 * 8192)


def test_compressed_scale_accounting_and_packing():
    """scale_mode 1 (Sec. 3.4): 4 bits per narrow-format group in an array of their own -> the 2.06 bpw the paper prints;
    nothing extra for the wide format, whose field rides in the spare nibble -> 2.75 bpw all told."""
    K, N = 8192, 8192
    w = b.descriptor(K, N, [b.NARROW], scale_mode=1)
    i = b.pack_info(w, 16)
    assert i.scale_bytes == N * (K // 64) // 2 and i.code_bpw == 2.0
    assert 8.0 * (i.code_bytes + i.scale_bytes) / (N * K) == 2.0625 == o.bpw(8, 64, 4, 4)
    assert i.total_bpw == 8.0 * (i.code_bytes + i.scale_bytes + 8 * N + 2 * N) / (N * K)   # + alpha, beta, super scale per row
    w2 = b.descriptor(K, N, [b.WIDE], scale_mode=1)
    i2 = b.pack_info(w2, 16)
    assert i2.scale_bytes == 0 and i2.code_bpw == 2.75 and i2.total_bpw == 8.0 * (i2.code_bytes + 2 * N) / (N * K)
    bad = b.descriptor(K, N, [b.NARROW], scale_mode=2)
    with pytest.raises(b.CcqError):
        b.pack_info(bad)
    # the permutation of the 4-bit fields: the p-th narrow group of row n (byte p/2, shift 4*(p%2) in paper order)
    # lands in the 16-bit word [row tile][p/4][n%16] at bits 4*(p%4)
    K, N = 1024, 32
    gf = synth.group_format_map(K // 64, 8, synth.rng(3, 5))
    w3 = b.descriptor(K, N, [b.NARROW, b.WIDE], gf, scale_mode=1)
    gn = int((gf == 0).sum())
    sq = synth.rng(3, 6).integers(0, 256, size=(N, gn // 2), dtype=np.uint8)
    dev = b.pack_scales4(w3, sq)
    assert dev.size == (N // 16) * (gn // 4) * 16
    for n in (0, 5, 17, 31):
        for p in range(gn):
            field = (int(sq[n, p // 2]) >> (4 * (p % 2))) & 15
            word = int(dev[((n // 16) * (gn // 4) + p // 4) * 16 + n % 16])
            assert (word >> (4 * (p % 4))) & 15 == field
    buf = np.zeros(N * (K // 64), np.uint16)
    assert b.load().ccq_pack_scales(ctypes.byref(w3), b._np_ptr(buf), b._np_ptr(buf.copy())) == -2   # fp16 scales belong to scale_mode 0
    w0 = b.descriptor(K, N, [b.NARROW, b.WIDE], gf)
    assert b.load().ccq_pack_scales4(ctypes.byref(w0), b._np_ptr(sq), b._np_ptr(buf)) == -2           # and the fields to scale_mode 1


def _device_offset_narrow(n, pos, byte):
    """Documented device order of a narrow k-tile (independent re-statement for the test)."""
    tile, j, kq, b_in = pos // 4, pos % 4, byte // 4, byte % 4
    return tile * 1024 + (kq * 16 + n % 16) * 16 + j * 4 + b_in


def _device_offset_wide(n, pos, byte):
    tile, j = pos // 8, pos % 8
    kq = min(byte // 6, 3)
    t, b_in = (byte - 6 * kq) // 2, (byte - 6 * kq) % 2
    return tile * 2816 + t * 1024 + (kq * 16 + n % 16) * 16 + j * 2 + b_in


def test_pack_codes_is_the_documented_permutation():
    rng = np.random.default_rng(0)
    K, N = 2048, 48
    gf = synth.group_format_map(K // 64, 8, synth.rng(3, 1))
    w = b.descriptor(K, N, [b.NARROW, b.WIDE], gf)
    rb = o.row_bytes(K, (o.F2, o.F275), gf)
    src = rng.integers(0, 256, size=(N, rb), dtype=np.uint8)
    out = b.pack_codes(w, src)
    assert np.array_equal(np.sort(out), np.sort(src.ravel()))               # a permutation: no byte altered, none duplicated
    info = b.pack_info(w, 0)
    n_narrow = int((gf == 0).sum())
    pos = {0: 0, 1: 0}
    off = 0
    for g in range(K // 64):
        kind = int(gf[g])
        nb = 22 if kind else 16
        for n in (0, 5, 16, 47):
            base = (n // 16) * info.row_tile_bytes + (0 if kind == 0 else (n_narrow // 4) * 1024)
            for byte in range(nb):
                d = base + (_device_offset_wide(n, pos[1], byte) if kind else _device_offset_narrow(n, pos[0], byte))
                assert out[d] == src[n, off + byte], (g, n, byte)
        pos[kind] += 1
        off += nb
    meta = b.pack_meta(w)
    assert list(meta[:n_narrow]) == list(np.flatnonzero(gf == 0)) and list(meta[n_narrow:]) == list(np.flatnonzero(gf == 1))
    scales = rng.integers(0, 1 << 16, size=(N, K // 64), dtype=np.uint16)
    ps = b.pack_scales(w, scales)
    assert np.array_equal(np.sort(ps), np.sort(scales.ravel()))
    tile_halfs = (n_narrow // 4) * 64 + ((K // 64 - n_narrow) // 8) * 128
    g0 = int(np.flatnonzero(gf == 0)[5])                                    # 6th narrow group: tile 1, slot 1
    assert ps[2 * tile_halfs + 1 * 64 + 3 * 4 + 1] == scales[35, g0]
    g1 = int(np.flatnonzero(gf == 1)[7])                                    # 8th wide group: tile 0, slot 7
    assert ps[0 * tile_halfs + (n_narrow // 4) * 64 + 9 * 8 + 7] == scales[9, g1]


def test_hybrid_word_accounting_and_packing():
    """Sec. 3.2 / 3.4: ten 16-bit words per 64 weights = 2.5 bpw; the device order is a permutation of the canonical bytes
    (segment t = word // 4, lane = 16 (word % 4) + row, halfword = group within the k-tile of 8 groups)."""
    K, N = 1024, 32
    w = b.descriptor(K, N, b.H16)
    i = b.pack_info(w, 64)
    assert i.code_bpw == 2.5 and i.code_bytes == N * o.h16_row_bytes(K) and i.bytes_per_group[0] == i.bytes_per_group[1] == 20
    assert i.scale_bytes == N * (K // 64) * 2 and i.row_tile_bytes == (K // 512) * 2560
    assert i.total_bpw == 2.5 + 16 / 64
    canon = np.arange(N * o.h16_row_bytes(K), dtype=np.uint32)
    tagged = (canon * 2654435761 >> 7).astype(np.uint8)           # any byte pattern; positions are what is tested
    dev = b.pack_codes(w, tagged)
    assert sorted(dev.tolist()) == sorted(tagged.tolist())
    rb = o.h16_row_bytes(K)
    for (n, g, word, byte) in [(0, 0, 0, 0), (5, 3, 9, 1), (17, 8, 4, 0), (31, 15, 7, 1), (16, 9, 8, 0)]:
        src = n * rb + g * 20 + word * 2 + byte
        off = (n // 16) * i.row_tile_bytes + (g // 8) * 2560 + (word // 4) * 1024 + ((word % 4) * 16 + n % 16) * 16 + (g % 8) * 2 + byte
        assert dev[off] == tagged[src], (n, g, word, byte)
    info = b.ccq_info()
    lib = b.load()
    i1 = b.pack_info(b.descriptor(K, N, b.H16, scale_mode=1), 64)      # Sec. 3.4: the scale rides in the 13 spare bits, 2.5 bpw in all
    assert i1.scale_bytes == 0 and i1.code_bytes == i.code_bytes and i1.total_bpw == 2.5 + 16 / K
    assert lib.ccq_pack_info(ctypes.byref(b.descriptor(K + 64, N, b.H16)), 1, ctypes.byref(info)) == 0              # 17 groups: three k-tiles of 8, the last padded
    assert info.padded_groups[0] == info.padded_groups[1] == 24 and info.code_bytes == (N // 16) * 3 * 2560 and info.code_bpw == 2.5
    assert lib.ccq_pack_info(ctypes.byref(b.descriptor(K, N, [b.H16_HI, b.ccq_code(3, 4, 2, 0, 3.0)])), 1, ctypes.byref(info)) == -3  # one zp per word
    assert lib.ccq_pack_info(ctypes.byref(b.descriptor(K, N, [b.H16_LO, b.H16_HI])), 1, ctypes.byref(info)) != 0   # halves in the wrong order


def test_descriptor_validation():
    def status(fn):
        try:
            fn()
            return 0
        except b.CcqError as e:
            return e.status
    ok = b.descriptor(1024, 64, [b.NARROW])
    assert status(lambda: b.pack_info(ok)) == 0
    bad_group = b.descriptor(1024, 64, [b.NARROW]); bad_group.group = 128
    assert status(lambda: b.pack_info(bad_group)) == -3                     # valid CCQ, not built
    assert status(lambda: b.pack_info(b.descriptor(1000, 64, [b.NARROW]))) == -2   # K not a multiple of 64
    assert status(lambda: b.pack_info(b.descriptor(1024, 0, [b.NARROW]))) == -2
    i = b.pack_info(b.descriptor(1024, 40, [b.NARROW]))                           # rows not a multiple of 16: the last row tile is padded
    assert i.padded_N == 48 and i.code_bytes == 3 * 4 * 1024 and i.canonical_code_bytes == 40 * 256 and i.code_bpw == 2.0
    i = b.pack_info(b.descriptor(1088, 64, [b.NARROW]))                           # 17 narrow groups: the fifth k-tile holds one
    assert i.padded_groups[0] == 20 and i.groups[0] == 17 and i.code_bytes == 4 * 5 * 1024 and i.scale_bytes == 4 * 5 * 64 * 2
    assert status(lambda: b.pack_info(b.descriptor(1024, 64, [b.ccq_code(3, 3, 2, 0, 4.0)]))) == -3   # other (L,N,S)
    assert status(lambda: b.pack_info(b.descriptor(1024, 64, [b.ccq_code(6, 4, 3, 1, 31.25)]))) == -2  # zp not a multiple of 0.5
    assert status(lambda: b.pack_info(b.descriptor(1024, 64, [b.ccq_code(6, 4, 7, 1, 32.0)]))) == -2   # S > L
    assert status(lambda: b.pack_info(b.descriptor(1024, 64, [b.NARROW, b.NARROW], np.zeros(16, np.uint8)))) == -2
    gf = np.zeros(16, np.uint8); gf[3] = 2
    assert status(lambda: b.pack_info(b.descriptor(1024, 64, [b.NARROW, b.WIDE], gf))) == -2
    assert b.load().ccq_pack_info(None, 1, None) == -1


def test_gemm_argument_errors_need_no_gpu():
    """All argument checks happen before any HIP call."""
    lib = b.load()
    w = b.descriptor(1024, 64, [b.NARROW])
    vp = ctypes.c_void_p
    assert lib.ccq_gemm(ctypes.byref(w), vp(0), 0, 1024, vp(0), 64, vp(0), 0, vp(0)) == 0            # M = 0: no-op
    assert lib.ccq_gemm(ctypes.byref(w), vp(0), 1, 1024, vp(0), 64, vp(0), 0, vp(0)) == -1           # x, y NULL
    assert lib.ccq_gemm(ctypes.byref(w), vp(256), 1, 1024, vp(512), 64, vp(0), 0, vp(0)) == -1       # codes NULL
    w.codes, w.scales, w.code_alpha, w.code_beta = 4096, 8192, 12288, 16384                           # never dereferenced below
    assert lib.ccq_gemm(ctypes.byref(w), vp(256), -1, 1024, vp(512), 64, vp(0), 0, vp(0)) == -2
    assert lib.ccq_gemm(ctypes.byref(w), vp(256), 1, 512, vp(512), 64, vp(0), 0, vp(0)) == -2        # ldx < K
    assert lib.ccq_gemm(ctypes.byref(w), vp(258), 1, 1024, vp(512), 64, vp(0), 0, vp(0)) == -4       # misaligned x
    assert lib.ccq_gemm(ctypes.byref(w), vp(256), 1, 1028, vp(512), 64, vp(0), 0, vp(0)) == -4       # ldx not a multiple of 8
    la = b.ccq_launch(1, 1, 1, 4)
    assert lib.ccq_gemm_ex(ctypes.byref(w), vp(256), 1, 1024, vp(512), 64, vp(0), 0, vp(0), ctypes.byref(la)) == -5   # workspace missing
    la = b.ccq_launch(3, 1, 1, 1)
    assert lib.ccq_gemm_ex(ctypes.byref(w), vp(256), 1, 1024, vp(512), 64, vp(0), 0, vp(0), ctypes.byref(la)) == -2
    offs = np.array([0, 2, 1, 4], dtype=np.int32)                                                    # not monotone
    rc = lib.ccq_grouped_gemm(ctypes.byref(w), 3, 1 << 20, 1 << 16, 4096, vp(256), 4, 1024, vp(512), 4, vp(768),
                              offs.ctypes.data_as(vp), vp(1024), 64, vp(0), 0, vp(0))
    assert rc == -6


def test_missing_library_is_a_loud_error(monkeypatch, tmp_path):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "libccq.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        b.load()


def _ragged_case(kinds, K, N, n_wide, seed):
    rng = synth.rng(8, seed)
    G = K // 64
    gf = synth.group_format_map(G, n_wide, rng) if len(kinds) == 2 else None
    fm = {"narrow": (o.F2, b.NARROW), "wide": (o.F275, b.WIDE)}
    ofmt = fm[kinds[0]][0] if len(kinds) == 1 else (o.F2, o.F275)
    w = b.descriptor(K, N, [fm[k][1] for k in kinds], gf)
    codes = rng.integers(1, 256, size=(N, o.row_bytes(K, ofmt, gf)), dtype=np.uint8)      # no zero byte: padding is what is zero
    scales = rng.integers(1, 1 << 15, size=(N, G), dtype=np.uint16)
    return w, gf, codes, scales


@pytest.mark.parametrize("kinds,K,N,n_wide", [(["narrow"], 1088, 40, None), (["wide"], 832, 24, None), (["narrow", "wide"], 1600, 1000, 5),
                                              (["narrow", "wide"], 7232, 8, 5)])
def test_padded_layouts(kinds, K, N, n_wide):
    """Any K % 64 == 0, any N and any group map: the device layout rounds every kind up to whole k-tiles and the rows up
    to whole row tiles; what is added holds zero codes and zero scales, the real bytes sit where the unpadded layout
    puts them, and the group map names the last real group for the padded positions."""
    w, gf, codes, scales = _ragged_case(kinds, K, N, n_wide, K + N)
    i = b.pack_info(w, 64)
    G = K // 64
    gn = G if kinds == ["narrow"] else (0 if kinds == ["wide"] else G - n_wide)
    gw = G - gn
    tn, tw = -(-gn // 4), -(-gw // 8)
    rt = -(-N // 16)
    assert i.padded_N == rt * 16 and i.row_tile_bytes == tn * 1024 + tw * 2816 and i.code_bytes == rt * i.row_tile_bytes
    assert i.scale_bytes == rt * (tn * 64 + tw * 128) * 2 and i.canonical_code_bytes == codes.size
    assert abs(i.code_bpw - 8 * codes.size / (N * K)) < 1e-12
    pg = {"narrow": tn * 4, "wide": tw * 8}
    assert [i.padded_groups[f] for f in range(len(kinds))] == [pg[k] for k in kinds]
    dev = b.pack_codes(w, codes)
    assert np.count_nonzero(dev) == codes.size - (0 if gw == 0 else 0) and sorted(dev[dev != 0].tolist()) == sorted(codes.ravel().tolist())
    ps = b.pack_scales(w, scales)
    assert sorted(ps[ps != 0].tolist()) == sorted(scales.ravel().tolist())
    # a row of the last (ragged) row tile, last real group of each kind: the same position rule as in whole tiles
    n = N - 1
    kind_of = (lambda g: 0 if kinds == ["narrow"] else 1) if gf is None else (lambda g: int(gf[g]))
    cnt = [0, 0]
    goff = 0
    for g in range(G):
        kd = kind_of(g)
        p = cnt[kd]
        cnt[kd] += 1
        if kd == 0:
            assert dev[(n // 16) * i.row_tile_bytes + (p // 4) * 1024 + (2 * 16 + n % 16) * 16 + (p % 4) * 4 + 1] == codes[n, goff + 4 * 2 + 1], g
            assert ps[(n // 16) * (tn * 64 + tw * 128) + (p // 4) * 64 + (n % 16) * 4 + p % 4] == scales[n, g]
            goff += 16
        else:
            assert dev[(n // 16) * i.row_tile_bytes + tn * 1024 + (p // 8) * 2816 + 1 * 1024 + (3 * 16 + n % 16) * 16 + (p % 8) * 2] == codes[n, goff + 6 * 3 + 2], g
            assert ps[(n // 16) * (tn * 64 + tw * 128) + tn * 64 + (p // 8) * 128 + (n % 16) * 8 + p % 8] == scales[n, g]
            goff += 22
    if gf is not None:
        meta = b.pack_meta(w)
        assert meta.size == tn * 4 + tw * 8
        assert meta[:gn].tolist() == np.flatnonzero(gf == 0).tolist() and meta[tn * 4:tn * 4 + gw].tolist() == np.flatnonzero(gf == 1).tolist()
        assert np.all(meta[gn:tn * 4] == G - 1) and np.all(meta[tn * 4 + gw:] == G - 1)
