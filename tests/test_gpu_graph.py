"""The library under HIP graph capture: calls enqueue kernels only (no allocation, no
synchronisation, no memset nodes), so a captured sequence must replay to the eager result
every time.  Replays are separated by eager work and synchronisations of the program."""
import sys

import numpy as np
import pytest
import torch

from paper_2511_13764_amd import binding as B
from paper_2511_13764_amd import workloads as W

import gpu_helpers as H

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def test_captured_calls_replay_to_the_eager_result(oracle):
    assert torch.cuda.is_available()
    B.load()
    # a split shape (partial sums in the caller's workspace / the library's own buffer) and an unsplit one
    M1, N1, K1 = 16, 2048, 4096
    M2, N2, K2 = 512, 768, 512
    A1, W1 = H.dev(W.normal_bf16(96, 0, (M1, K1))), H.dev(W.normal_bf16(96, 1, (N1, K1), sigma=0.05))
    A2, B2 = H.dev(W.normal_bf16(96, 2, (M2, K2))), H.dev(W.normal_bf16(96, 3, (K2, N2)))
    bias = H.dev(W.normal_f32(96, 4, (N2,)))
    ws = torch.empty(B.gemm_workspace_bytes(B.DTYPE_BF16, M1, N1, K1), dtype=torch.uint8, device="cuda")
    C1 = torch.zeros((M1, N1), dtype=torch.float32, device="cuda")
    C1n = torch.zeros((M1, N1), dtype=torch.float32, device="cuda")
    C2 = torch.zeros((M2, N2), dtype=torch.int16, device="cuda")

    def sequence(stream):
        B.gemm_bf16(0, 1, M1, N1, K1, A1, K1, W1, K1, 0.0, C1, N1, 1, workspace=ws, stream=stream)
        B.gemm_bf16_noalloc(0, 1, M1, N1, K1, A1, K1, W1, K1, 0.0, C1n, N1, 1, stream=stream)
        B.brgemm_fused(B.DTYPE_BF16, 0, 0, M2, N2, K2, 1, A2, None, K2, B2, None, N2, 0.0, C2, N2, 0, bias,
                       B.EPI_BIAS | B.EPI_RELU, stream=stream)

    sequence(None)                       # eager: also the first call of gemm_bf16_noalloc on this device
    torch.cuda.synchronize()
    assert B.gemm_last_variant() >= 0
    want = [C1.clone(), C1n.clone(), C2.clone()]
    assert torch.equal(want[0], want[1])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sequence(side)                   # warm the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            sequence(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        say(f"graph replay {rep}")
        for c in (C1, C1n, C2):
            c.fill_(-3 if c.dtype == torch.int16 else float("nan"))
        x = torch.randn(1 << 20, device="cuda")           # the program's own eager work between replays
        (x * 2).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C1, want[0]) and torch.equal(C1n, want[1]) and torch.equal(C2, want[2]), rep
    ref = oracle.gemm_ref(W.normal_bf16(96, 0, (M1, K1)), K1, W.normal_bf16(96, 1, (N1, K1), sigma=0.05), K1,
                          M1, N1, K1, transB=1)
    assert H.rel_fro(C1.cpu().numpy(), ref) <= H.TOL_BF16_F32OUT
