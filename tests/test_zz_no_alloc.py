"""gemm_bf16_noalloc (the entry point for callers that cannot allocate) against gemm_bf16
with a full caller workspace: two calls in a row on shapes whose plan splits the
reduction, the second smaller than the first, then the refusal of a plan that does not
fit the built-in buffer.  Collected last: a failure here must not hide other tests."""
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


def _both_ways(oracle, seed, M, N, K, c_f32):
    A = W.normal_bf16(seed, 0, (M, K))
    Wt = W.normal_bf16(seed, 1, (N, K), sigma=0.02)
    dA, dB = H.dev(A), H.dev(Wt)
    ws = torch.empty(B.gemm_workspace_bytes(B.DTYPE_BF16, M, N, K), dtype=torch.uint8, device="cuda")
    dt = torch.float32 if c_f32 else torch.int16
    c_ref = torch.full((M, N), -1, dtype=dt, device="cuda")
    c_new = torch.full((M, N), -2, dtype=dt, device="cuda")
    say(f"noalloc {M}x{N}x{K} c_f32={c_f32}: gemm_bf16 with workspace")
    B.gemm_bf16(0, 1, M, N, K, dA, K, dB, K, 0.0, c_ref, N, c_f32, workspace=ws)
    torch.cuda.synchronize()
    plan = (B.gemm_last_variant(), B.gemm_last_split())
    free_before = torch.cuda.mem_get_info()[0]
    say(f"noalloc {M}x{N}x{K} c_f32={c_f32}: gemm_bf16_noalloc")
    B.gemm_bf16_noalloc(0, 1, M, N, K, dA, K, dB, K, 0.0, c_new, N, c_f32)
    torch.cuda.synchronize()
    assert (B.gemm_last_variant(), B.gemm_last_split()) == plan
    assert plan[1] > 1, "the case is meant to exercise the built-in partial-sum buffer"
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated by the call"
    assert torch.equal(c_ref, c_new), "same plan, fixed-order reduction: results must be identical"
    got = c_new.cpu().numpy()
    got = H.widen(got.view(np.uint16)) if not c_f32 else got.astype(np.float64)
    ref = oracle.gemm_ref(A, K, Wt, K, M, N, K, transB=1)
    err = H.rel_fro(got, ref)
    say(f"   split={plan[1]} rel_fro={err:.3e}")
    assert err <= (H.TOL_BF16_F32OUT if c_f32 else H.TOL_BF16)


def test_noalloc_twice_then_refusal(oracle):
    assert torch.cuda.is_available()
    B.load()
    # one call first: the first call on a device looks the buffer's address up
    z = torch.zeros((64, 64), dtype=torch.int16, device="cuda")
    B.gemm_bf16_noalloc(0, 1, 64, 64, 64, z, 64, z, 64, 0.0, z.clone(), 64, 0)
    torch.cuda.synchronize()
    _both_ways(oracle, 90, 128, 11008, 4096, False)      # 2 x 128 x 11008 x 4 B = 11 MiB of partial sums
    _both_ways(oracle, 91, 16, 2048, 4096, True)         # smaller, right after: stale partial sums around it
    # a plan that cannot fit: forced split 16 of a 1024 x 1024 C needs 64 MiB
    M = N = K = 1024
    a = torch.zeros((M, K), dtype=torch.int16, device="cuda")
    c = torch.full((M, N), 7, dtype=torch.int16, device="cuda")
    B.gemm_force_variant(-1, 16)
    try:
        rc = B.gemm_bf16_noalloc(0, 1, M, N, K, a, K, a, K, 0.0, c, N, 0, check=False)
    finally:
        B.gemm_force_variant(-1, 0)
    torch.cuda.synchronize()
    assert rc == B.SCRATCH_TOO_SMALL and "scratch" in B.strerror(rc)
    assert (c == 7).all().item(), "a refused call must launch nothing"
    # unsplit problems need no scratch and are accepted whatever their size
    B.gemm_bf16_noalloc(0, 1, M, N, K, a, K, a, K, 0.0, c, N, 0)
    torch.cuda.synchronize()
    assert (c == 0).all().item()
