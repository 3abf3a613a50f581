"""ctypes front end of the CCQ CPU oracle (oracle/ccq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports this module and
this module never imports the GPU package.

Every function is a thin marshalling layer; the arithmetic lives in the C file,
whose header lists the passage of the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ccq_oracle.c")
_LIB = os.path.join(_HERE, "libccq_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Code(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("N", ctypes.c_int32), ("S", ctypes.c_int32),
                ("code_cluster", ctypes.c_int32), ("zp", ctypes.c_double)]


@dataclass(frozen=True)
class Code:
    """A convolutional-code configuration (L, N, S) of Sec. 3.1 plus the
    Code Cluster switch of Sec. 3.3 and the weight zero-point of Alg. 2/3."""
    L: int
    N: int
    S: int
    code_cluster: bool = False
    zp: float | None = None

    @property
    def T(self) -> int:
        return self.L + (self.N - 1) * self.S

    @property
    def zero_point(self) -> float:
        return float(2 ** (self.L - 1)) if self.zp is None else float(self.zp)

    def c(self) -> _Code:
        return _Code(self.L, self.N, self.S, int(self.code_cluster), self.zero_point)


# the two inference formats of Table 1 used by the GPU library
F2 = Code(6, 4, 3, code_cluster=True)     # 2.0 bpw codes (2.06 with 4-bit scales)
F275 = Code(4, 3, 2)                      # 2.75 bpw

_lib = None


def lib():
    global _lib
    if _lib is None:
        # CCQ_ORACLE_LIBRARY names another build of ccq_oracle.c (the host-sanitizer test points it at an instrumented one)
        L = ctypes.CDLL(os.environ.get("CCQ_ORACLE_LIBRARY") or build())
        u8p = ctypes.POINTER(ctypes.c_uint8)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        cp = ctypes.POINTER(_Code)
        I = ctypes.c_int
        L.cco_fp16_to_double.restype = ctypes.c_double
        L.cco_fp16_to_double.argtypes = [ctypes.c_uint16]
        L.cco_bf16_to_double.restype = ctypes.c_double
        L.cco_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.cco_double_to_bf16.restype = ctypes.c_uint16
        L.cco_double_to_bf16.argtypes = [ctypes.c_double]
        L.cco_double_to_fp16.restype = ctypes.c_uint16
        L.cco_double_to_fp16.argtypes = [ctypes.c_double]
        L.cco_double_to_bf16_array.restype = None
        L.cco_double_to_bf16_array.argtypes = [ctypes.c_int64, f64p, u16p]
        L.cco_fp16_to_double_array.restype = None
        L.cco_fp16_to_double_array.argtypes = [ctypes.c_int64, u16p, f64p]
        L.cco_T.restype = I
        L.cco_T.argtypes = [I, I, I]
        L.cco_states.restype = None
        L.cco_states.argtypes = [ctypes.c_uint32, I, I, I, u32p]
        L.cco_bpw.restype = ctypes.c_double
        L.cco_bpw.argtypes = [I, I, I, I]
        L.cco_codes_per_group.restype = I
        L.cco_codes_per_group.argtypes = [I, I]
        L.cco_code_bytes.restype = I
        L.cco_code_bytes.argtypes = [cp]
        L.cco_group_bytes.restype = I
        L.cco_group_bytes.argtypes = [cp, I]
        L.cco_cluster_expand.restype = ctypes.c_uint32
        L.cco_cluster_expand.argtypes = [ctypes.c_uint32, ctypes.c_float, ctypes.c_float]
        L.cco_row_bytes.restype = ctypes.c_int64
        L.cco_row_bytes.argtypes = [I, I, cp, u8p]
        L.cco_decode.restype = I
        L.cco_decode.argtypes = [I, I, I, cp, u8p, u8p, u16p, f32p, f32p, f64p]
        L.cco_decode_f64scales.restype = I
        L.cco_decode_f64scales.argtypes = [I, I, I, cp, u8p, u8p, f64p, f32p, f32p, f64p]
        L.cco_spare_bits.restype = I
        L.cco_spare_bits.argtypes = [cp, I]
        L.cco_sq_row_bytes.restype = ctypes.c_int64
        L.cco_sq_row_bytes.argtypes = [I, I, cp, u8p]
        L.cco_expand_scales.restype = I
        L.cco_expand_scales.argtypes = [I, I, I, cp, u8p, u8p, u8p, u16p, f64p]
        L.cco_compress_scales.restype = I
        L.cco_compress_scales.argtypes = [I, I, I, cp, u8p, f32p, I, u8p, u16p, f32p, f32p, u8p, u16p]
        L.cco_h16_states.restype = None
        L.cco_h16_states.argtypes = [ctypes.c_uint32, u32p]
        L.cco_h16_words_per_group.restype = I
        L.cco_h16_words_per_group.argtypes = [I]
        L.cco_h16_decode.restype = I
        L.cco_h16_decode.argtypes = [I, I, I, ctypes.c_double, u8p, u16p, f64p]
        L.cco_h16_quantize.restype = I
        L.cco_h16_quantize.argtypes = [I, I, I, ctypes.c_double, f32p, I, u8p, u16p]
        L.cco_h16_expand_scales.restype = I
        L.cco_h16_expand_scales.argtypes = [I, I, I, u8p, u16p, f64p]
        L.cco_h16_decode_cs.restype = I
        L.cco_h16_decode_cs.argtypes = [I, I, I, ctypes.c_double, u8p, u16p, f64p]
        L.cco_h16_compress_scales.restype = I
        L.cco_h16_compress_scales.argtypes = [I, I, I, ctypes.c_double, f32p, I, u8p, u16p, u16p]
        L.cco_matmul.restype = None
        L.cco_matmul.argtypes = [I, I, I, u16p, ctypes.c_int64, f64p, f64p]
        L.cco_num_threads.restype = I
        L.cco_num_threads.argtypes = []
        L.cco_search_brute.restype = ctypes.c_uint32
        L.cco_search_brute.argtypes = [f64p, ctypes.c_double, ctypes.c_double, I, I, I]
        L.cco_search_viterbi.restype = ctypes.c_uint32
        L.cco_search_viterbi.argtypes = [f64p, ctypes.c_double, ctypes.c_double, I, I, I]
        L.cco_refit_scale.restype = ctypes.c_double
        L.cco_refit_scale.argtypes = [f64p, f64p, I, ctypes.c_double]
        L.cco_quantize.restype = I
        L.cco_quantize.argtypes = [I, I, I, cp, u8p, f32p, I, I, u8p, u16p, f32p, f32p]
        _lib = L
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty)) if a is not None else None


def _fmts(fmt):
    if isinstance(fmt, Code):
        fmt = (fmt, fmt)
    arr = (_Code * 2)(fmt[0].c(), fmt[1].c())
    return arr, fmt


def T(code: Code) -> int:
    return lib().cco_T(code.L, code.N, code.S)


def states(code_value: int, cfg: Code) -> list[int]:
    out = (ctypes.c_uint32 * cfg.N)()
    lib().cco_states(int(code_value), cfg.L, cfg.N, cfg.S, out)
    return list(out)


def codebook(cfg: Code) -> np.ndarray:
    """The virtual codebook C in Z^(2^T x N) of Sec. 3.1 (row = code value)."""
    return np.array([states(c, cfg) for c in range(1 << cfg.T)], dtype=np.int64)


def bpw(T_store: int, g: int, N: int, scale_bits: int) -> float:
    return lib().cco_bpw(T_store, g, N, scale_bits)


def group_bytes(cfg: Code, g: int = 64) -> int:
    c = cfg.c()
    return lib().cco_group_bytes(ctypes.byref(c), g)


def cluster_expand(q: int, alpha: float, beta: float) -> int:
    return lib().cco_cluster_expand(int(q), float(np.float32(alpha)), float(np.float32(beta)))


def fp16_bits_to_f64(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float64)
    lib().cco_fp16_to_double_array(h.size, _p(h, ctypes.c_uint16), _p(out, ctypes.c_double))
    return out


def to_bf16_bits(y: np.ndarray) -> np.ndarray:
    """Round fp64 values to bfloat16 (nearest even); returns uint16 bit patterns."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    out = np.empty(y.shape, dtype=np.uint16)
    lib().cco_double_to_bf16_array(y.size, _p(y, ctypes.c_double), _p(out, ctypes.c_uint16))
    return out


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    b = np.asarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def row_bytes(K: int, fmt, group_fmt=None, g: int = 64) -> int:
    arr, _ = _fmts(fmt)
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    return lib().cco_row_bytes(K, g, arr, _p(gf, ctypes.c_uint8))


def decode(K, N, fmt, codes, scales_fp16, alpha=None, beta=None, group_fmt=None, g=64) -> np.ndarray:
    """Alg. 2 / Alg. 3: canonical codes -> W fp64 [N][K] (exact values)."""
    arr, _ = _fmts(fmt)
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales_fp16, dtype=np.uint16)
    assert codes.size == N * row_bytes(K, fmt, gf, g), "codes size does not match canonical layout"
    assert scales.size == N * (K // g)
    al = None if alpha is None else np.ascontiguousarray(alpha, dtype=np.float32)
    be = None if beta is None else np.ascontiguousarray(beta, dtype=np.float32)
    W = np.empty((N, K), dtype=np.float64)
    rc = lib().cco_decode(K, N, g, arr, _p(gf, ctypes.c_uint8), _p(codes, ctypes.c_uint8),
                          _p(scales, ctypes.c_uint16), _p(al, ctypes.c_float), _p(be, ctypes.c_float),
                          _p(W, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_decode failed with {rc}")
    return W


def spare_bits(cfg: Code, g: int = 64) -> int:
    """Unused low bits of a group's last stored code (Sec. 3.4): 4 for (L=4,N=3,S=2) at g=64."""
    return lib().cco_spare_bits(ctypes.byref(cfg.c()), g)


def sq_row_bytes(K: int, fmt, group_fmt=None, g: int = 64) -> int:
    """Bytes per row of the packed 4-bit scale array s_q (groups without spare bits, two per byte)."""
    arr, _ = _fmts(fmt)
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    return lib().cco_sq_row_bytes(K, g, arr, _p(gf, ctypes.c_uint8))


def expand_scales(K, N, fmt, codes, sq_packed, s_super_fp16, group_fmt=None, g=64) -> np.ndarray:
    """Sec. 3.4 / first line of Alg. 2 and Alg. 3: fp64 group scales [N][K/g] = 4-bit field * s_super."""
    arr, _ = _fmts(fmt)
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    nb = sq_row_bytes(K, fmt, gf, g)
    sq = np.zeros((N, max(nb, 1)), dtype=np.uint8) if sq_packed is None else np.ascontiguousarray(sq_packed, dtype=np.uint8)
    assert sq_packed is None or sq.size == N * nb
    ssup = np.ascontiguousarray(s_super_fp16, dtype=np.uint16)
    assert ssup.size == N and codes.size == N * row_bytes(K, fmt, gf, g)
    out = np.empty((N, K // g), dtype=np.float64)
    rc = lib().cco_expand_scales(K, N, g, arr, _p(gf, ctypes.c_uint8), _p(codes, ctypes.c_uint8), _p(sq, ctypes.c_uint8),
                                 _p(ssup, ctypes.c_uint16), _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_expand_scales failed with {rc}")
    return out


def decode_cs(K, N, fmt, codes, sq_packed, s_super_fp16, alpha=None, beta=None, group_fmt=None, g=64) -> np.ndarray:
    """Alg. 2 / Alg. 3 with compressed scales: canonical codes -> W fp64 [N][K] (exact values)."""
    arr, _ = _fmts(fmt)
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sc = expand_scales(K, N, fmt, codes, sq_packed, s_super_fp16, gf, g)
    al = None if alpha is None else np.ascontiguousarray(alpha, dtype=np.float32)
    be = None if beta is None else np.ascontiguousarray(beta, dtype=np.float32)
    W = np.empty((N, K), dtype=np.float64)
    rc = lib().cco_decode_f64scales(K, N, g, arr, _p(gf, ctypes.c_uint8), _p(codes, ctypes.c_uint8), _p(sc, ctypes.c_double),
                                    _p(al, ctypes.c_float), _p(be, ctypes.c_float), _p(W, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_decode_f64scales failed with {rc}")
    return W


def compress_scales(W, fmt, codes, scales_fp16, alpha=None, beta=None, group_fmt=None, method: str = "viterbi", g: int = 64):
    """Sec. 3.4 Scale Compression on the output of quantize(): returns (codes, sq_packed uint8 [N][sq_row_bytes],
    s_super fp16 bits [N]).  Codes are searched again with the scales that will be stored."""
    arr, _ = _fmts(fmt)
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    codes = np.array(codes, dtype=np.uint8, copy=True, order="C")
    scales = np.ascontiguousarray(scales_fp16, dtype=np.uint16)
    al = np.ones(N, dtype=np.float32) if alpha is None else np.ascontiguousarray(alpha, dtype=np.float32)
    be = np.zeros(N, dtype=np.float32) if beta is None else np.ascontiguousarray(beta, dtype=np.float32)
    nb = sq_row_bytes(K, fmt, gf, g)
    sq = np.zeros((N, max(nb, 1)), dtype=np.uint8)
    ssup = np.zeros(N, dtype=np.uint16)
    rc = lib().cco_compress_scales(K, N, g, arr, _p(gf, ctypes.c_uint8), _p(W, ctypes.c_float), 0 if method == "brute" else 1,
                                   _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16), _p(al, ctypes.c_float), _p(be, ctypes.c_float),
                                   _p(sq, ctypes.c_uint8), _p(ssup, ctypes.c_uint16))
    if rc != 0:
        raise ValueError(f"cco_compress_scales failed with {rc}")
    return codes, sq[:, :nb], ssup


# ---- Sec. 3.2 hybrid word: (3,3,2) + (3,4,2) in 16 bits, 2.28 bpw per word, 2.5 bpw at g = 64
H16_ZP = 4.0


def h16_states(word: int) -> list[int]:
    st = (ctypes.c_uint32 * 7)()
    lib().cco_h16_states(int(word), st)
    return list(st)


def h16_row_bytes(K: int, g: int = 64) -> int:
    return (K // g) * lib().cco_h16_words_per_group(g) * 2


def h16_decode(K, N, codes, scales_fp16, zp: float = H16_ZP, g: int = 64) -> np.ndarray:
    """Alg. 2 on hybrid words: canonical bytes (little-endian uint16 words, 10 per 64-weight group) -> W fp64 [N][K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales_fp16, dtype=np.uint16)
    assert codes.size == N * h16_row_bytes(K, g) and scales.size == N * (K // g)
    W = np.empty((N, K), dtype=np.float64)
    rc = lib().cco_h16_decode(K, N, g, float(zp), _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16), _p(W, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_h16_decode failed with {rc}")
    return W


def h16_quantize(W: np.ndarray, method: str = "viterbi", zp: float = H16_ZP, g: int = 64):
    """Alg. 1 on hybrid words: returns (codes uint8 [N][h16_row_bytes], scales fp16 bits [N][K/g])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    codes = np.zeros((N, h16_row_bytes(K, g)), dtype=np.uint8)
    scales = np.zeros((N, K // g), dtype=np.uint16)
    rc = lib().cco_h16_quantize(K, N, g, float(zp), _p(W, ctypes.c_float), 0 if method == "brute" else 1, _p(codes, ctypes.c_uint8),
                                _p(scales, ctypes.c_uint16))
    if rc != 0:
        raise ValueError(f"cco_h16_quantize failed with {rc}")
    return codes, scales


def h16_expand_scales(K, N, codes, s_super_fp16, g: int = 64) -> np.ndarray:
    """Alg. 2, first lines, scale mask 0x1FFF (Table 1): group scales fp64 [N][K/g] from the last word of every group."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    ssup = np.ascontiguousarray(s_super_fp16, dtype=np.uint16)
    out = np.empty((N, K // g), dtype=np.float64)
    rc = lib().cco_h16_expand_scales(K, N, g, _p(codes, ctypes.c_uint8), _p(ssup, ctypes.c_uint16), _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_h16_expand_scales failed with {rc}")
    return out


def h16_decode_cs(K, N, codes, s_super_fp16, zp: float = H16_ZP, g: int = 64) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    ssup = np.ascontiguousarray(s_super_fp16, dtype=np.uint16)
    assert codes.size == N * h16_row_bytes(K, g) and ssup.size == N
    W = np.empty((N, K), dtype=np.float64)
    rc = lib().cco_h16_decode_cs(K, N, g, float(zp), _p(codes, ctypes.c_uint8), _p(ssup, ctypes.c_uint16), _p(W, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"cco_h16_decode_cs failed with {rc}")
    return W


def h16_compress_scales(W, codes, scales_fp16, method: str = "viterbi", zp: float = H16_ZP, g: int = 64):
    """Encoder side of Sec. 3.4 on the hybrid word: returns (codes with the 13-bit fields in place, s_super fp16 bits [N])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    codes = np.array(codes, dtype=np.uint8, copy=True).reshape(N, -1)
    scales = np.ascontiguousarray(scales_fp16, dtype=np.uint16)
    ssup = np.zeros(N, dtype=np.uint16)
    rc = lib().cco_h16_compress_scales(K, N, g, float(zp), _p(W, ctypes.c_float), 0 if method == "brute" else 1, _p(codes, ctypes.c_uint8),
                                       _p(scales, ctypes.c_uint16), _p(ssup, ctypes.c_uint16))
    if rc != 0:
        raise ValueError(f"cco_h16_compress_scales failed with {rc}")
    return codes, ssup


def matmul(x_bf16: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X W^T in fp64; x_bf16 is uint16 bf16 bit patterns [M][K]."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.float64)
    M, K = x.shape
    N = W.shape[0]
    assert W.shape[1] == K
    Y = np.empty((M, N), dtype=np.float64)
    lib().cco_matmul(M, K, N, _p(x, ctypes.c_uint16), K, _p(W, ctypes.c_double), _p(Y, ctypes.c_double))
    return Y


def grouped_matmul(x_bf16, sorted_rows, expert_offsets, W_of_expert) -> np.ndarray:
    """Grouped GEMM as E independent GEMMs: output row p (in expert e's range
    expert_offsets[e]..expert_offsets[e+1]) = x[sorted_rows[p]] @ W_e^T.
    W_of_expert(e) returns the decoded fp64 matrix of expert e (streamed so
    that only one expert's weights are held at a time)."""
    x = np.asarray(x_bf16, dtype=np.uint16)
    E = len(expert_offsets) - 1
    out = None
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        W = W_of_expert(e)
        if out is None:
            out = np.zeros((int(expert_offsets[-1]), W.shape[0]), dtype=np.float64)
        out[lo:hi] = matmul(x[np.asarray(sorted_rows[lo:hi], dtype=np.int64)], W)
    return out


def num_threads() -> int:
    return lib().cco_num_threads()


def search(v, s: float, cfg: Code, method: str = "viterbi") -> int:
    v = np.ascontiguousarray(v, dtype=np.float64)
    assert v.size == cfg.N
    f = lib().cco_search_brute if method == "brute" else lib().cco_search_viterbi
    return f(_p(v, ctypes.c_double), float(s), cfg.zero_point, cfg.L, cfg.N, cfg.S)


def refit_scale(w, wq, fallback: float = 1.0) -> float:
    w = np.ascontiguousarray(w, dtype=np.float64)
    wq = np.ascontiguousarray(wq, dtype=np.float64)
    return lib().cco_refit_scale(_p(w, ctypes.c_double), _p(wq, ctypes.c_double), w.size, fallback)


def quantize(W: np.ndarray, fmt, group_fmt=None, method: str = "viterbi", cluster_research: bool = True, g: int = 64):
    """Alg. 1 (+ Code Cluster, + Eq. 4): fp32 W [N][K] -> canonical codes.
    Returns (codes uint8 [N][row_bytes], scales_fp16 uint16 [N][K/g], alpha, beta)."""
    arr, fm = _fmts(fmt)
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    gf = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    rb = row_bytes(K, fmt, gf, g)
    codes = np.zeros((N, rb), dtype=np.uint8)
    scales = np.zeros((N, K // g), dtype=np.uint16)
    alpha = np.ones(N, dtype=np.float32)
    beta = np.zeros(N, dtype=np.float32)
    rc = lib().cco_quantize(K, N, g, arr, _p(gf, ctypes.c_uint8), _p(W, ctypes.c_float),
                            0 if method == "brute" else 1, int(cluster_research),
                            _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16),
                            _p(alpha, ctypes.c_float), _p(beta, ctypes.c_float))
    if rc != 0:
        raise ValueError(f"cco_quantize failed with {rc}")
    return codes, scales, alpha, beta
