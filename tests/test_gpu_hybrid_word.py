"""GPU parity of the hybrid 16-bit word (Sec. 3.2 "Hybrid Encoding"; Table 1 row "(3,3,2)(3,4,2)") through the C ABI:
decoded weights bit for bit (one-hot activations), products within the tolerance of tests/cases.py, every number of
activation rows the kernels distinguish, explicit launch shapes, the grouped entry point."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close, canon_zero
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class H16Case:
    def __init__(self, K, N, codes, scales):
        self.K, self.N, self.codes, self.scales = K, N, codes, scales
        self._W = None

    def W(self):
        if self._W is None:
            self._W = o.h16_decode(self.K, self.N, self.codes, self.scales)
        return self._W

    def device_weight(self):
        return b.Weight.from_canonical(self.K, self.N, b.H16, self.codes, self.scales, device=DEV)


def random_h16(K, N, seed, stream0=0) -> H16Case:
    """Random words (every bit pattern decodes, the 13 spare bits of a group's last word included) and log-uniform scales."""
    codes = synth.random_codes(N, o.h16_row_bytes(K), synth.rng(seed, stream0))
    scales = synth.scales_log_uniform_fp16(N, K // 64, synth.rng(seed, stream0 + 1))
    return H16Case(K, N, codes, scales)


def encoded_h16(K, N, seed) -> H16Case:
    W = synth.weights_normal(N, K, synth.rng(seed, 0))
    codes, scales = o.h16_quantize(W)
    return H16Case(K, N, codes, scales)


def _gemm_bits(w, x_bits, **kw):
    y = b.gemm(w, b.bf16_tensor(x_bits, DEV), **kw)
    torch.cuda.synchronize()
    return b.bf16_bits(y)


def _check_decode(c, w, ks, fp32_first=False, **kw):
    ks = list(ks)
    got = _gemm_bits(w, synth.one_hot_bf16(ks, c.K), **kw)
    want = c.W()[:, ks].T
    if fp32_first:
        # a 13-bit scale field times an 11-bit super scale times a 3-bit state difference has up to 27 significant
        # bits: the kernels hold that product in fp32 (one rounding) before the bf16 output rounding, and so does
        # the expected value here
        want = want.astype(np.float32).astype(np.float64)
    want = o.to_bf16_bits(want)
    assert np.array_equal(canon_zero(got), canon_zero(want)), f"decoded weights differ at columns {ks[:8]}..."


@pytest.mark.parametrize("K,N", [(512, 16), (1024, 208), (2048, 64)])
def test_decode_bit_exact(K, N):
    c = random_h16(K, N, 21, stream0=K % 97)
    w = c.device_weight()
    # every column of the first group and of the last one (all seven states of every word, the lone weight 63)
    for g in (0, K // 64 - 1):
        for i in range(0, 64, 16):
            _check_decode(c, w, range(64 * g + i, 64 * g + i + 16))
    _check_decode(c, w, [63])                                   # one held row
    _check_decode(c, w, [6, 7, 62])                             # up to four
    _check_decode(c, w, synth.rng(21, 5).integers(0, K, 40))    # more than 16: several passes or the tiled kernel


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 16, 17, 33, 64, 70, 130])
def test_gemm_rows(M):
    c = encoded_h16(1024, 256, 22)
    w = c.device_weight()
    x = synth.activations_bf16(M, c.K, synth.rng(22, 100 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"hybrid word M={M}", rounded=(x, c.W()) if M > 16 else None)


@pytest.mark.parametrize("K,N,M", [(4096, 144, 70), (2048, 16, 65), (8192, 272, 40), (512, 400, 257)])
def test_tiled_kernel_shapes(K, N, M):
    """More than 16 rows go through the 64-row LDS-tiled kernel: K cut into shares, ragged last blocks in M and N."""
    c = random_h16(K, N, 26, stream0=N)
    w = c.device_weight()
    x = synth.activations_bf16(M, K, synth.rng(26, 100 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"K={K} N={N} M={M}", rounded=(x, c.W()))
    ks = synth.rng(26, 200 + M).integers(0, K, M)
    ks[:8] = [0, 6, 7, 62, 63, 64, K - 1, K - 2]
    _check_decode(c, w, ks)


@pytest.mark.parametrize("launch", [(1, 1, 1, 1), (1, 4, 1, 1), (1, 1, 4, 1), (1, 2, 2, 2), (1, 1, 1, 4), (1, 3, 2, 1)])
@pytest.mark.parametrize("M", [1, 4, 16, 40])
def test_launch_shapes(launch, M):
    c = random_h16(2048, 112, 23)
    w = c.device_weight()
    if M > 32 and launch[1] * launch[2] > 4:
        pytest.skip("launch shape not built for this many held rows")
    x = synth.activations_bf16(M, c.K, synth.rng(23, 300 + M))
    assert_gemm_close(_gemm_bits(w, x, launch=b.ccq_launch(*launch)), o.matmul(x, c.W()), f"M={M} launch={launch}")
    _check_decode(c, w, [3, 64 + 20, 2047, 500][:min(M, 4)], launch=b.ccq_launch(*launch))


def test_strided_rows_and_untouched_padding():
    c = random_h16(1024, 48, 24)
    w = c.device_weight()
    M, ldx, ldy = 5, c.K + 64, c.N + 16
    x = synth.activations_bf16(M, c.K, synth.rng(24, 1))
    xt = torch.zeros((M, ldx), dtype=torch.bfloat16, device=DEV)
    xt[:, :c.K] = b.bf16_tensor(x, DEV)
    yt = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device=DEV)
    b.gemm(w, xt[:, :c.K], out=yt[:, :c.N])
    torch.cuda.synchronize()
    assert_gemm_close(b.bf16_bits(yt[:, :c.N]), o.matmul(x, c.W()), "strided")
    assert torch.all(yt[:, c.N:] == 7.0)


def test_grouped():
    E, K, N, T = 4, 512, 64, 12
    cases = [random_h16(K, N, 25, stream0=10 * e) for e in range(E)]
    w = b.Weight.from_canonical(K, N, b.H16, np.stack([c.codes for c in cases]), np.stack([c.scales for c in cases]), device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(25, 99))
    offs = np.array([0, 5, 5, 14, 20], dtype=np.int32)
    rows = synth.rng(25, 98).integers(0, T, 20).astype(np.int32)
    y = b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), offs)
    torch.cuda.synchronize()
    got = b.bf16_bits(y)
    for e in range(E):
        lo, hi = offs[e], offs[e + 1]
        if hi > lo:
            assert_gemm_close(got[lo:hi], o.matmul(x[rows[lo:hi]], cases[e].W()), f"expert {e}")


def test_grouped_many_rows_per_expert():
    """More than 32 rows on an expert: with the host copy of the offsets the 64-row kernel runs, without it the
    per-row-tile kernel; decoded weights bit exact through the 64-row kernel."""
    E, K, N, T = 3, 1024, 80, 50
    cases = [random_h16(K, N, 29, stream0=10 * e) for e in range(E)]
    w = b.Weight.from_canonical(K, N, b.H16, np.stack([c.codes for c in cases]), np.stack([c.scales for c in cases]), device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(29, 99))
    offs = np.array([0, 70, 70, 105], dtype=np.int32)
    rows = synth.rng(29, 98).integers(0, T, 105).astype(np.int32)
    for host_offsets in (offs, None):
        y = b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), host_offsets)
        torch.cuda.synchronize()
        got = b.bf16_bits(y)
        for e in range(E):
            lo, hi = offs[e], offs[e + 1]
            if hi > lo:
                xe = x[rows[lo:hi]]
                assert_gemm_close(got[lo:hi], o.matmul(xe, cases[e].W()), f"expert {e}", rounded=(xe, cases[e].W()))
    ks = synth.rng(29, 97).integers(0, K, 40)
    ks[:4] = [0, 62, 63, K - 1]
    offs2 = (np.arange(E + 1) * len(ks)).astype(np.int32)
    rows2 = np.tile(np.arange(len(ks), dtype=np.int32), E)
    y2 = b.grouped_gemm(w, b.bf16_tensor(synth.one_hot_bf16(ks, K), DEV), torch.from_numpy(rows2).to(DEV), torch.from_numpy(offs2).to(DEV), offs2)
    torch.cuda.synchronize()
    got = b.bf16_bits(y2).reshape(E, len(ks), N)
    for e in range(E):
        assert np.array_equal(canon_zero(got[e]), canon_zero(o.to_bf16_bits(cases[e].W()[:, ks].T))), f"expert {e}"


# ---------------------------------------------------------------- compressed scales (Sec. 3.4; Alg. 2 with scale mask 0x1FFF)


class H16CaseCS:
    def __init__(self, K, N, codes, ssup):
        self.K, self.N, self.codes, self.ssup = K, N, codes, ssup
        self._W = None

    def W(self):
        if self._W is None:
            self._W = o.h16_decode_cs(self.K, self.N, self.codes, self.ssup)
        return self._W

    def device_weight(self):
        return b.Weight.from_canonical_compressed(self.K, self.N, b.H16, self.codes, None, self.ssup, device=DEV)


def random_h16_cs(K, N, seed) -> H16CaseCS:
    """Random words (so random 13-bit fields) and log-uniform fp16 super scales."""
    codes = synth.random_codes(N, o.h16_row_bytes(K), synth.rng(seed, 0))
    ssup = synth.scales_log_uniform_fp16(N, 1, synth.rng(seed, 1), lo=1e-5, hi=1e-3).reshape(N)
    return H16CaseCS(K, N, codes, ssup)


@pytest.mark.parametrize("K,N", [(512, 32), (2048, 208)])
def test_compressed_scales_decode_bit_exact(K, N):
    c = random_h16_cs(K, N, 27)
    w = c.device_weight()
    assert w.info.scale_bytes == 0 and w.info.total_bpw == 2.5 + 16 / K
    for ks in (range(48, 64), range(K - 16, K), [63], [0, 62, 63], synth.rng(27, 5).integers(0, K, 40)):
        _check_decode(c, w, ks, fp32_first=True)


@pytest.mark.parametrize("M", [1, 3, 16, 17, 64, 130])
def test_compressed_scales_gemm(M):
    Wf = synth.weights_normal(192, 1536, synth.rng(28, 0))
    codes, scales = o.h16_quantize(Wf)
    codes, ssup = o.h16_compress_scales(Wf, codes, scales)
    c = H16CaseCS(1536, 192, codes, ssup)
    w = c.device_weight()
    x = synth.activations_bf16(M, c.K, synth.rng(28, 100 + M))
    assert_gemm_close(_gemm_bits(w, x), o.matmul(x, c.W()), f"hybrid word, compressed scales, M={M}", rounded=(x, c.W()) if M > 16 else None)


def test_compressed_scales_grouped():
    E, K, N, T = 3, 512, 48, 9
    cases = [random_h16_cs(K, N, 29 + e) for e in range(E)]
    w = b.Weight.from_canonical_compressed(K, N, b.H16, np.stack([c.codes for c in cases]), None, np.stack([c.ssup for c in cases]),
                                           device=DEV, experts=E)
    x = synth.activations_bf16(T, K, synth.rng(29, 99))
    offs = np.array([0, 4, 4, 11], dtype=np.int32)
    rows = synth.rng(29, 98).integers(0, T, 11).astype(np.int32)
    y = b.grouped_gemm(w, b.bf16_tensor(x, DEV), torch.from_numpy(rows).to(DEV), torch.from_numpy(offs).to(DEV), offs)
    torch.cuda.synchronize()
    got = b.bf16_bits(y)
    for e in range(E):
        lo, hi = offs[e], offs[e + 1]
        if hi > lo:
            assert_gemm_close(got[lo:hi], o.matmul(x[rows[lo:hi]], cases[e].W()), f"expert {e}")
