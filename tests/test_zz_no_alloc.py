"""ccq_gemm_static, the entry point for callers that cannot allocate: its output must equal ccq_gemm's bit for
bit (same kernels, the library's own scratch array in place of the caller's workspace) and stay within the GEMM
tolerance of the oracle, on two calls in a row that share the array, the second one smaller."""
import numpy as np
import pytest
import torch

from cases import assert_gemm_close, random_case
from oracle import ccq_oracle as o
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(case, w, M, seed):
    x_bits = synth.activations_bf16(M, case.K, synth.rng(31, seed))
    x = b.bf16_tensor(x_bits, DEV)
    need = b.gemm_workspace_bytes(w.desc, M)
    assert 0 < need <= b.load().ccq_gemm_static_max_workspace(), (M, need)   # the case must really use the scratch array
    ref = b.bf16_bits(b.gemm(w, x))
    out = torch.full((M, case.N), float("nan"), dtype=torch.bfloat16, device=DEV)
    got = b.bf16_bits(b.gemm_static(w, x, out))
    torch.cuda.synchronize()
    assert np.array_equal(got, ref), f"M={M}: ccq_gemm_static differs from ccq_gemm"
    assert_gemm_close(got, o.matmul(x_bits, case.W()), f"ccq_gemm_static M={M}")


def test_static_entry_matches_gemm_on_two_calls_in_a_row():
    big = random_case(2048, 1024, ["narrow"], 31)
    wb = big.device_weight(DEV)
    small = random_case(1024, 512, ["wide"], 31, stream0=10)
    wsm = small.device_weight(DEV)
    _both(big, wb, 64, 1)      # 64-row kernel, K cut into shares: 1 MiB of partial tiles in the array
    _both(big, wb, 16, 2)      # per-row-tile kernel, smaller input, same array
    _both(small, wsm, 8, 3)    # another matrix and format, smaller again
    _both(big, wb, 24, 4)      # the 32-row variant of the per-row-tile kernel
    _both(big, wb, 64, 1)      # and the first call again, after the others have left their partials behind


def test_static_entry_rejects_what_exceeds_the_array():
    # wide format, 128 rows, N = 16384: two K shares of 128 x 16384 fp32 = 16 MiB of partial tiles
    d = b.descriptor(2048, 16384, [b.WIDE])
    M = 128
    assert b.gemm_workspace_bytes(d, M) > b.load().ccq_gemm_static_max_workspace()
    x = torch.zeros((M, 2048), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((M, 16384), dtype=torch.bfloat16, device=DEV)
    import ctypes
    rc = b.load().ccq_gemm_static(ctypes.byref(d), b._t_ptr(x), M, 2048, b._t_ptr(y), 16384, b._stream_ptr(None))
    assert rc == -5   # CCQ_ERR_WORKSPACE, before anything is enqueued (the descriptor's device pointers are still NULL)
    torch.cuda.synchronize()
    assert not bool(y.any())
