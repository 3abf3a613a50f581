"""Thin ctypes binding of libccq.so (include/ccq.h): argument marshalling only.

Every step of the fused dequantize-and-multiply runs inside the HIP library;
PyTorch is used for device memory and streams.  The functions carry the names
of the C entry points (pack_info, pack_codes, pack_scales, pack_meta, gemm,
gemm_ex, grouped_gemm).  If the library has not been built this module raises
on first use -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# CCQ_LIBRARY names another build of the same library (the host-sanitizer test points it at an instrumented one)
LIB_PATH = os.environ.get("CCQ_LIBRARY") or os.path.join(_HERE, "libccq.so")

CCQ_OK = 0
STATUS = {0: "CCQ_OK", -1: "CCQ_ERR_NULL", -2: "CCQ_ERR_BAD_PARAM", -3: "CCQ_ERR_UNSUPPORTED", -4: "CCQ_ERR_ALIGN",
          -5: "CCQ_ERR_WORKSPACE", -6: "CCQ_ERR_ROUTING", -7: "CCQ_ERR_HIP"}


class CcqError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where} failed: {STATUS.get(status, status)}")
        self.status = status


class ccq_code(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("N", ctypes.c_int32), ("S", ctypes.c_int32), ("code_cluster", ctypes.c_int32),
                ("zp", ctypes.c_float)]


class ccq_weight(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("N", ctypes.c_int32), ("group", ctypes.c_int32), ("n_formats", ctypes.c_int32),
                ("fmt", ccq_code * 2), ("group_fmt", ctypes.c_void_p), ("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("code_alpha", ctypes.c_void_p), ("code_beta", ctypes.c_void_p), ("meta", ctypes.c_void_p),
                ("scale_mode", ctypes.c_int32), ("scale_super", ctypes.c_void_p)]


class ccq_info(ctypes.Structure):
    _fields_ = [("code_bytes", ctypes.c_int64), ("scale_bytes", ctypes.c_int64), ("meta_bytes", ctypes.c_int64),
                ("workspace_bytes", ctypes.c_int64), ("row_tile_bytes", ctypes.c_int64), ("bytes_per_group", ctypes.c_int32 * 2),
                ("groups", ctypes.c_int32 * 2), ("align", ctypes.c_int32), ("code_bpw", ctypes.c_double), ("total_bpw", ctypes.c_double),
                ("canonical_code_bytes", ctypes.c_int64), ("padded_N", ctypes.c_int32), ("padded_groups", ctypes.c_int32 * 2)]


class ccq_launch(ctypes.Structure):
    _fields_ = [("rows_per_wave_tiles", ctypes.c_int32), ("waves_rows", ctypes.c_int32), ("waves_k", ctypes.c_int32),
                ("splits_k", ctypes.c_int32)]


# the two code configurations of Table 1 the kernels are built for
NARROW = ccq_code(6, 4, 3, 1, 32.0)   # (L=6,N=4,S=3) + Code Cluster, 2.0 bpw
WIDE = ccq_code(4, 3, 2, 0, 8.0)      # (L=4,N=3,S=2), 2.75 bpw
# the two halves of the hybrid 16-bit word of Sec. 3.2 (pass both, in this order, without a group map)
H16_HI = ccq_code(3, 3, 2, 0, 4.0)    # (L=3,N=3,S=2): top 7 bits of the word
H16_LO = ccq_code(3, 4, 2, 0, 4.0)    # (L=3,N=4,S=2): low 9 bits; 10 words per 64 weights, 2.5 bpw
H16 = [H16_HI, H16_LO]

EXPORTS = ["ccq_pack_info", "ccq_pack_codes", "ccq_pack_scales", "ccq_pack_scales4", "ccq_pack_meta", "ccq_gemm", "ccq_gemm_ex",
           "ccq_grouped_gemm", "ccq_grouped_workspace_bytes", "ccq_quantize", "ccq_quantize_workspace_bytes", "ccq_status_string",
           "ccq_probe_stream_read", "ccq_probe_mfma_bf16", "ccq_gemm_workspace_bytes",
           "ccq_gemm_static", "ccq_gemm_static_max_workspace"]

_lib = None


def load() -> ctypes.CDLL:
    """Load libccq.so; raises if it has not been built (python -m paper_2507_07145_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_07145_amd.build` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    wp = ctypes.POINTER(ccq_weight)
    L.ccq_pack_info.restype = ctypes.c_int
    L.ccq_pack_info.argtypes = [wp, i32, ctypes.POINTER(ccq_info)]
    for name in ("ccq_pack_codes", "ccq_pack_scales", "ccq_pack_scales4"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [wp, vp, vp]
    L.ccq_pack_meta.restype = ctypes.c_int
    L.ccq_pack_meta.argtypes = [wp, vp]
    L.ccq_gemm.restype = ctypes.c_int
    L.ccq_gemm.argtypes = [wp, vp, i32, i64, vp, i64, vp, i64, vp]
    L.ccq_gemm_ex.restype = ctypes.c_int
    L.ccq_gemm_ex.argtypes = [wp, vp, i32, i64, vp, i64, vp, i64, vp, ctypes.POINTER(ccq_launch)]
    L.ccq_grouped_gemm.restype = ctypes.c_int
    L.ccq_grouped_gemm.argtypes = [wp, i32, i64, i64, i64, vp, i32, i64, vp, i32, vp, vp, vp, i64, vp, i64, vp]
    L.ccq_gemm_workspace_bytes.restype = i64
    L.ccq_gemm_workspace_bytes.argtypes = [wp, i32]
    L.ccq_gemm_static.restype = ctypes.c_int
    L.ccq_gemm_static.argtypes = [wp, vp, i32, i64, vp, i64, vp]
    L.ccq_gemm_static_max_workspace.restype = i64
    L.ccq_gemm_static_max_workspace.argtypes = []
    L.ccq_grouped_workspace_bytes.restype = i64
    L.ccq_grouped_workspace_bytes.argtypes = [wp, i32, i32]
    L.ccq_quantize_workspace_bytes.restype = i64
    L.ccq_quantize_workspace_bytes.argtypes = [wp]
    L.ccq_quantize.restype = ctypes.c_int
    L.ccq_quantize.argtypes = [wp, vp, i64, vp, vp, vp, vp, vp, vp, i64, vp]
    L.ccq_probe_stream_read.restype = ctypes.c_int
    L.ccq_probe_stream_read.argtypes = [vp, i64, i32, i32, vp, vp]
    L.ccq_probe_mfma_bf16.restype = ctypes.c_int
    L.ccq_probe_mfma_bf16.argtypes = [vp, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    L.ccq_status_string.restype = ctypes.c_char_p
    L.ccq_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != CCQ_OK:
        raise CcqError(status, where)


def _np_ptr(a) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _t_ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream_ptr(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def descriptor(K: int, N: int, fmts, group_fmt: np.ndarray | None = None, scale_mode: int = 0) -> ccq_weight:
    """A ccq_weight with shape/format fields set and all DEVICE pointers NULL."""
    w = ccq_weight()
    w.K, w.N, w.group, w.n_formats, w.scale_mode = K, N, 64, len(fmts), scale_mode
    for i, f in enumerate(fmts):
        w.fmt[i] = f
    w.group_fmt = group_fmt.ctypes.data if group_fmt is not None else None
    return w


def pack_info(w: ccq_weight, M_max: int = 64) -> ccq_info:
    info = ccq_info()
    _check(load().ccq_pack_info(ctypes.byref(w), M_max, ctypes.byref(info)), "ccq_pack_info")
    return info


def pack_codes(w: ccq_weight, canonical: np.ndarray) -> np.ndarray:
    info = pack_info(w, 0)
    src = np.ascontiguousarray(canonical, dtype=np.uint8)
    if src.size != info.canonical_code_bytes:
        raise ValueError(f"canonical code stream has {src.size} bytes, layout needs {info.canonical_code_bytes}")
    out = np.empty(info.code_bytes, dtype=np.uint8)
    _check(load().ccq_pack_codes(ctypes.byref(w), _np_ptr(src), _np_ptr(out)), "ccq_pack_codes")
    return out


def pack_scales(w: ccq_weight, canonical_fp16_bits: np.ndarray) -> np.ndarray:
    info = pack_info(w, 0)
    src = np.ascontiguousarray(canonical_fp16_bits, dtype=np.uint16)
    if src.size != w.N * (w.K // 64):
        raise ValueError("scale array size does not match the layout")
    out = np.empty(info.scale_bytes // 2, dtype=np.uint16)
    _check(load().ccq_pack_scales(ctypes.byref(w), _np_ptr(src), _np_ptr(out)), "ccq_pack_scales")
    return out


def pack_scales4(w: ccq_weight, canonical_sq: np.ndarray) -> np.ndarray:
    """scale_mode 1: canonical packed 4-bit scale fields of the narrow-format groups -> device order (uint16 words)."""
    info = pack_info(w, 0)
    src = np.ascontiguousarray(canonical_sq, dtype=np.uint8)
    out = np.zeros(max(info.scale_bytes // 2, 1), dtype=np.uint16)
    _check(load().ccq_pack_scales4(ctypes.byref(w), _np_ptr(src), _np_ptr(out)), "ccq_pack_scales4")
    return out[:info.scale_bytes // 2]


def pack_meta(w: ccq_weight) -> np.ndarray:
    info = pack_info(w, 0)
    out = np.empty(info.meta_bytes // 4, dtype=np.int32)
    _check(load().ccq_pack_meta(ctypes.byref(w), _np_ptr(out)), "ccq_pack_meta")
    return out


def bf16_tensor(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns (numpy) -> torch bf16 tensor on `device`."""
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """torch bf16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _per_row(values: np.ndarray, E: int, N: int, n_pad: int, dtype) -> np.ndarray:
    """[E][N] per-row parameters in rows of n_pad entries (the experts of a stack then start 16-byte aligned whatever N is)."""
    out = np.zeros((E, n_pad), dtype=dtype)
    out[:, :N] = np.ascontiguousarray(values, dtype=dtype).reshape(E, N)
    return out


class Weight:
    """Device-resident quantized weights of one matrix, or of E same-shaped experts stacked along a leading axis."""

    def __init__(self):
        self.desc = None
        self.info = None
        self.E = 1
        self.codes = self.scales = self.alpha = self.beta = self.meta = self.ssup = None
        self._group_fmt = None

    @classmethod
    def from_canonical(cls, K, N, fmts, codes, scales_fp16, alpha=None, beta=None, group_fmt=None, device="cuda:0", experts: int | None = None):
        """Permute canonical (paper order) arrays into device order with the library's pack routines and upload.
        With `experts` = E the arrays carry a leading expert axis."""
        self = cls()
        self._group_fmt = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
        w = descriptor(K, N, fmts, self._group_fmt)
        info = pack_info(w, 64)
        E = 1 if experts is None else int(experts)
        codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(E, -1)
        scales = np.ascontiguousarray(scales_fp16, dtype=np.uint16).reshape(E, -1)
        pc = np.stack([pack_codes(w, codes[e]) for e in range(E)])
        ps = np.stack([pack_scales(w, scales[e]) for e in range(E)])
        self.codes = torch.from_numpy(pc).to(device)
        self.scales = torch.from_numpy(ps.view(np.int16)).to(device)
        needs_ab = any(f.code_cluster for f in fmts)
        if needs_ab:
            self.alpha = torch.from_numpy(_per_row(alpha, E, N, info.padded_N, np.float32)).to(device)
            self.beta = torch.from_numpy(_per_row(beta, E, N, info.padded_N, np.float32)).to(device)
        if group_fmt is not None:
            self.meta = torch.from_numpy(pack_meta(w)).to(device)
        w.codes, w.scales = self.codes.data_ptr(), self.scales.data_ptr()
        w.code_alpha = self.alpha.data_ptr() if needs_ab else None
        w.code_beta = self.beta.data_ptr() if needs_ab else None
        w.meta = self.meta.data_ptr() if self.meta is not None else None
        self.desc, self.info, self.E = w, info, E
        return self

    @classmethod
    def from_canonical_compressed(cls, K, N, fmts, codes, sq_packed, s_super_fp16, alpha=None, beta=None, group_fmt=None, device="cuda:0",
                                  experts: int | None = None):
        """The same for compressed scales (scale_mode 1): `sq_packed` holds the 4-bit fields of the narrow-format
        groups (uint8 [N][ceil(narrow groups / 2)], may be empty), `s_super_fp16` the fp16 bits of the per-row super
        scale; wide-format groups carry their field inside `codes`."""
        self = cls()
        self._group_fmt = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
        w = descriptor(K, N, fmts, self._group_fmt, scale_mode=1)
        info = pack_info(w, 64)
        E = 1 if experts is None else int(experts)
        codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(E, -1)
        self.codes = torch.from_numpy(np.stack([pack_codes(w, codes[e]) for e in range(E)])).to(device)
        if info.scale_bytes > 0:
            sq = np.ascontiguousarray(sq_packed, dtype=np.uint8).reshape(E, N, -1)
            self.scales = torch.from_numpy(np.stack([pack_scales4(w, sq[e]) for e in range(E)]).view(np.int16)).to(device)
        self.ssup = torch.from_numpy(_per_row(s_super_fp16, E, N, info.padded_N, np.uint16).view(np.int16)).to(device)
        needs_ab = any(f.code_cluster for f in fmts)
        if needs_ab:
            self.alpha = torch.from_numpy(_per_row(alpha, E, N, info.padded_N, np.float32)).to(device)
            self.beta = torch.from_numpy(_per_row(beta, E, N, info.padded_N, np.float32)).to(device)
        if group_fmt is not None:
            self.meta = torch.from_numpy(pack_meta(w)).to(device)
        w.codes = self.codes.data_ptr()
        w.scales = self.scales.data_ptr() if self.scales is not None else None
        w.scale_super = self.ssup.data_ptr()
        w.code_alpha = self.alpha.data_ptr() if needs_ab else None
        w.code_beta = self.beta.data_ptr() if needs_ab else None
        w.meta = self.meta.data_ptr() if self.meta is not None else None
        self.desc, self.info, self.E = w, info, E
        return self

    @property
    def K(self):
        return self.desc.K

    @property
    def N(self):
        return self.desc.N

    @property
    def device(self):
        return self.codes.device

    def strides(self):
        """(codes, scales, alpha/beta) byte strides between consecutive experts."""
        ab = self.alpha.stride(0) * 4 if self.alpha is not None else (self.ssup.stride(0) * 4 if self.ssup is not None else 0)
        return (self.codes.stride(0), self.scales.stride(0) * 2 if self.scales is not None else 0, ab)


def quantize(W: torch.Tensor, fmt, scale_mode: int = 0, group_fmt=None, stream=None, prefill_byte: int | None = None) -> Weight:
    """Quantize fp32 W [N][K] on the GPU through ccq_quantize; the result is ready for gemm().  `fmt`: NARROW, WIDE, H16, or
    [NARROW, WIDE] with `group_fmt` (uint8 [K/64], 0 = narrow, 1 = wide).  `prefill_byte`: every byte of the code and scale
    arrays is set to it before the call (a test's way of showing that the call leaves none of them unwritten)."""
    assert W.dtype == torch.float32 and W.dim() == 2 and W.stride(1) == 1 and W.is_cuda
    N, K = W.shape
    self = Weight()
    fmts = list(fmt) if isinstance(fmt, (list, tuple)) else [fmt]
    self._group_fmt = None if group_fmt is None else np.ascontiguousarray(group_fmt, dtype=np.uint8)
    d = descriptor(K, N, fmts, self._group_fmt, scale_mode=scale_mode)
    info = pack_info(d, 64)
    if self._group_fmt is not None:
        self.meta = torch.from_numpy(pack_meta(d)).to(W.device)
        d.meta = self.meta.data_ptr()
    self.codes = torch.empty(info.code_bytes, dtype=torch.uint8, device=W.device)
    if info.scale_bytes > 0:
        self.scales = torch.empty(info.scale_bytes // 2, dtype=torch.int16, device=W.device)
    if scale_mode == 1:
        self.ssup = torch.empty(N, dtype=torch.int16, device=W.device)
    if any(f.code_cluster for f in fmts):
        self.alpha = torch.empty(N, dtype=torch.float32, device=W.device)
        self.beta = torch.empty(N, dtype=torch.float32, device=W.device)
    if prefill_byte is not None:
        self.codes.fill_(prefill_byte)
        if self.scales is not None:
            self.scales.view(torch.uint8).fill_(prefill_byte)
    need = int(load().ccq_quantize_workspace_bytes(ctypes.byref(d)))
    if need < 0:
        raise CcqError(-3, "ccq_quantize_workspace_bytes")
    ws = _workspace(need, W.device)
    rc = load().ccq_quantize(ctypes.byref(d), _t_ptr(W), W.stride(0), _t_ptr(self.codes), _t_ptr(self.scales), _t_ptr(self.alpha),
                             _t_ptr(self.beta), _t_ptr(self.ssup), _t_ptr(ws), need, _stream_ptr(stream))
    _check(rc, "ccq_quantize")
    torch.cuda.current_stream().synchronize() if stream is None else stream.synchronize()   # the workspace is released on return
    d.codes = self.codes.data_ptr()
    d.scales = self.scales.data_ptr() if self.scales is not None else None
    d.scale_super = self.ssup.data_ptr() if self.ssup is not None else None
    d.code_alpha = self.alpha.data_ptr() if self.alpha is not None else None
    d.code_beta = self.beta.data_ptr() if self.beta is not None else None
    self.codes = self.codes.reshape(1, -1)
    if self.scales is not None:
        self.scales = self.scales.reshape(1, -1)
    if self.ssup is not None:
        self.ssup = self.ssup.reshape(1, -1)
    if self.alpha is not None:
        self.alpha, self.beta = self.alpha.reshape(1, -1), self.beta.reshape(1, -1)
    self.desc, self.info, self.E = d, info, 1
    return self


def _workspace(nbytes: int, device) -> torch.Tensor | None:
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes > 0 else None


def _new_output(rows: int, N: int, device) -> torch.Tensor:
    """bf16 [rows][N] whose row stride is a multiple of 8 elements, as the entry points require."""
    ld = (N + 7) // 8 * 8
    y = torch.empty((rows, ld), dtype=torch.bfloat16, device=device)
    return y if ld == N else y[:, :N]


def gemm(w: Weight, x: torch.Tensor, out: torch.Tensor | None = None, workspace: torch.Tensor | None = None, stream=None,
         launch: ccq_launch | None = None) -> torch.Tensor:
    """y = x W_dq^T through ccq_gemm (or ccq_gemm_ex when `launch` is given).  x: bf16 [M][K] on the GPU."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1 and x.is_cuda
    M = x.shape[0]
    y = out if out is not None else _new_output(M, w.N, x.device)
    if workspace is None:
        need = launch.splits_k * min(M, 64) * w.info.padded_N * 4 if (launch is not None and launch.splits_k > 1) else gemm_workspace_bytes(w.desc, M)
        workspace = _workspace(need, x.device)
        if workspace is not None and stream is not None:
            workspace.record_stream(stream)   # the temporary returns to the allocator at once; its memory must outlive the kernels
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    L = load()
    if launch is None:
        rc = L.ccq_gemm(ctypes.byref(w.desc), _t_ptr(x), M, x.stride(0), _t_ptr(y), y.stride(0), _t_ptr(workspace), ws_bytes, _stream_ptr(stream))
    else:
        rc = L.ccq_gemm_ex(ctypes.byref(w.desc), _t_ptr(x), M, x.stride(0), _t_ptr(y), y.stride(0), _t_ptr(workspace), ws_bytes,
                           _stream_ptr(stream), ctypes.byref(launch))
    _check(rc, "ccq_gemm")
    return y


def gemm_static(w: Weight, x: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
    """y = x W_dq^T through ccq_gemm_static: no workspace, nothing allocated (the caller passes `out`)."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1 and x.is_cuda
    assert out.dtype == torch.bfloat16 and out.shape == (x.shape[0], w.N) and out.stride(1) == 1
    _check(load().ccq_gemm_static(ctypes.byref(w.desc), _t_ptr(x), x.shape[0], x.stride(0), _t_ptr(out), out.stride(0), _stream_ptr(stream)),
           "ccq_gemm_static")
    return out


def gemm_workspace_bytes(desc: ccq_weight, M: int) -> int:
    need = int(load().ccq_gemm_workspace_bytes(ctypes.byref(desc), M))
    if need < 0:
        raise CcqError(-2, "ccq_gemm_workspace_bytes")
    return need


def grouped_workspace_bytes(w: Weight, P: int) -> int:
    return int(load().ccq_grouped_workspace_bytes(ctypes.byref(w.desc), w.E, P))


def grouped_gemm(w: Weight, x: torch.Tensor, sorted_rows: torch.Tensor, expert_offsets: torch.Tensor,
                 expert_offsets_host: np.ndarray | None = None, out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                 stream=None) -> torch.Tensor:
    """y[p] = x[sorted_rows[p]] W_dq(e)^T for p in expert e's range, through ccq_grouped_gemm."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1 and x.is_cuda
    assert sorted_rows.dtype == torch.int32 and expert_offsets.dtype == torch.int32
    P = sorted_rows.numel()
    y = out if out is not None else _new_output(P, w.N, x.device)
    if workspace is None:
        workspace = _workspace(max(grouped_workspace_bytes(w, P), 0), x.device)
        if workspace is not None and stream is not None:
            workspace.record_stream(stream)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    cs, ss, abs_ = w.strides()
    host = None
    if expert_offsets_host is not None:
        host = np.ascontiguousarray(expert_offsets_host, dtype=np.int32)
    rc = load().ccq_grouped_gemm(ctypes.byref(w.desc), w.E, cs, ss, abs_, _t_ptr(x), x.shape[0], x.stride(0), _t_ptr(sorted_rows), P,
                                 _t_ptr(expert_offsets), _np_ptr(host), _t_ptr(y), y.stride(0), _t_ptr(workspace), ws_bytes,
                                 _stream_ptr(stream))
    _check(rc, "ccq_grouped_gemm")
    return y


def probe_stream_read(src: torch.Tensor, sink: torch.Tensor, loads_per_thread: int = 4, block_threads: int = 512, stream=None) -> None:
    """Read `src` (uint8, a multiple of 16 bytes) once through ccq_probe_stream_read."""
    nbytes = src.numel() * src.element_size()
    _check(load().ccq_probe_stream_read(_t_ptr(src), nbytes, loads_per_thread, block_threads, _t_ptr(sink), _stream_ptr(stream)),
           "ccq_probe_stream_read")


def probe_mfma_bf16(operands: torch.Tensor, sink: torch.Tensor, workgroups: int, iters: int, stream=None) -> float:
    """Back-to-back bf16 MFMAs through ccq_probe_mfma_bf16; returns the floating-point operations of the launch."""
    assert operands.numel() * operands.element_size() >= 8 * 64 * 16 and sink.numel() >= workgroups * 256
    flop = ctypes.c_double(0.0)
    _check(load().ccq_probe_mfma_bf16(_t_ptr(operands), workgroups, iters, _t_ptr(sink), _stream_ptr(stream), ctypes.byref(flop)),
           "ccq_probe_mfma_bf16")
    return float(flop.value)
