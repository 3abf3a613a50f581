"""The entry points under HIP graph capture: the library enqueues kernels only (no memset node, no allocation, no
synchronisation), so a captured call must give, on every replay, exactly the bits of the eager call -- with other work
of the program and synchronisations between the replays, and with new activations written into the captured input
buffer before each replay (the decode step of generation replays one graph per token)."""
import numpy as np
import pytest
import torch

from cases import random_case
from paper_2507_07145_amd import binding as b
from paper_2507_07145_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("kinds,K,N,M,n_wide,static", [(["narrow"], 2048, 1024, 1, None, False), (["narrow"], 2048, 1024, 8, None, False),
                                                       (["narrow"], 2048, 1024, 16, None, True), (["wide"], 2048, 512, 1, None, False),
                                                       (["narrow", "wide"], 4096, 256, 16, 16, False), (["narrow"], 2048, 1024, 64, None, False),
                                                       (["wide"], 1024, 256, 40, None, True), (["narrow"], 512, 768, 300, None, False)])
def test_captured_calls_replay_bit_exactly(kinds, K, N, M, n_wide, static):
    c = random_case(K, N, kinds, 21, stream0=M + N % 7, n_wide=n_wide)
    w = c.device_weight(DEV)
    xs = [b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(21, 10 * M + i)), DEV) for i in range(4)]
    need = b.gemm_workspace_bytes(w.desc, M)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    call = (lambda x, y, s=None: b.gemm_static(w, x, y, stream=s)) if static else (lambda x, y, s=None: b.gemm(w, x, out=y, workspace=ws, stream=s))
    if static and need > b.load().ccq_gemm_static_max_workspace():
        pytest.skip("more partial tiles than the static array holds")
    eager = []
    for x in xs:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        call(x, y)
        torch.cuda.synchronize()
        eager.append(b.bf16_bits(y).copy())
    # capture one call on a side stream, reading x_in and writing y_out
    x_in = xs[0].clone()
    y_out = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call(x_in, y_out, side)          # warm the code path on this stream before capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call(x_in, y_out, side)
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(6):
        i = rep % len(xs)
        x_in.copy_(xs[i])
        y_out.fill_(1.0)                                  # a replay must overwrite every element
        ws.fill_(0xFF)                                    # and must not depend on what the workspace held
        scratch.normal_()                                 # unrelated work of the program between the replays
        _ = (scratch * 2).sum().item()                    # with a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(b.bf16_bits(y_out), eager[i]), f"replay {rep} differs from the eager call ({kinds} M={M})"
