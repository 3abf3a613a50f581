"""The ceiling probes (ccq_probe_stream_read, ccq_probe_mfma_bf16) run, reject bad arguments and do what they say:
the MFMA loop's result is the product its operands define, repeated `iters` times."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_stream_read_runs_for_every_shape_and_rejects_bad_arguments():
    src = torch.randint(0, 256, (3 * 1024 * 1024 + 16,), dtype=torch.uint8, device=DEV)
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    for lpt in (1, 2, 4, 8):
        for bt in (64, 256, 512):
            b.probe_stream_read(src, sink, lpt, bt)
    torch.cuda.synchronize()
    L = b.load()
    assert L.ccq_probe_stream_read(b._t_ptr(src), 1000, 4, 256, b._t_ptr(sink), None) == -2      # not a multiple of 16
    assert L.ccq_probe_stream_read(b._t_ptr(src), 1024, 3, 256, b._t_ptr(sink), None) == -2      # loads per thread
    assert L.ccq_probe_stream_read(b._t_ptr(src), 1024, 4, 100, b._t_ptr(sink), None) == -2      # block size
    assert L.ccq_probe_stream_read(None, 1024, 4, 256, b._t_ptr(sink), None) == -1
    assert L.ccq_probe_stream_read(ctypes.c_void_p(src.data_ptr() + 8), 1024, 4, 256, b._t_ptr(sink), None) == -4


def test_mfma_loop_accumulates_what_its_operands_define():
    # operands that are small integers: every partial sum is exact in fp32, so the sum over a wavefront's 4 accumulator
    # tiles after `iters` steps is iters * sum_i sum(A_i B_i^T), whatever the operand-to-lane layout is
    vals = synth.rng(90, 0).integers(-2, 3, size=(8 * 64, 8)).astype(np.float32)
    ops = b.bf16_tensor(synth.f32_to_bf16_bits(vals), DEV)
    sink = torch.zeros(2 * 256, dtype=torch.float32, device=DEV)
    iters = 5
    flop = b.probe_mfma_bf16(ops, sink, 2, iters)
    torch.cuda.synchronize()
    assert flop == 2.0 * 32 * 32 * 16 * 4 * iters * 4 * 2
    got = sink.cpu().numpy().reshape(2 * 4, 64).sum(axis=1)            # per wavefront: all elements of its 4 tiles
    v = vals.reshape(8, 64, 8)                                           # [operand][lane][k-slot]
    want = 0.0
    for i in range(4):
        # sum over all (row, column) of A B^T = sum_k (sum_rows A[:, k]) (sum_cols B[:, k]); lane l holds k-slots
        # 8 (l / 32) .. 8 (l / 32) + 7 of row (column) l % 32
        A, B = v[2 * i], v[2 * i + 1]
        for half in range(2):
            want += float(np.dot(A[32 * half:32 * half + 32].sum(axis=0), B[32 * half:32 * half + 32].sum(axis=0)))
    assert np.all(got == iters * want), (got, iters * want)
