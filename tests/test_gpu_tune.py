"""gemm_tune: tile selection by measurement (Section 5(a)).  The plan it finds must be one the
library can run, later calls of the same shape must take it and still agree with the
oracle, and it must not be slower than the rule table's plan by more than noise."""
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


def _time(fn, n=30):
    for _ in range(10):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


@pytest.mark.parametrize("M,N,K,tB,c_f32", [(512, 512, 4096, 0, True), (128, 4096, 4096, 1, False),
                                            (1536, 1536, 1536, 0, False)])
def test_tune_then_call(oracle, M, N, K, tB, c_f32):
    assert torch.cuda.is_available()
    B.load()
    B.gemm_tune_reset()
    A = W.normal_bf16(95, 0, (M, K))
    Bm = W.normal_bf16(95, 1, (N, K) if tB else (K, N), sigma=0.05)
    ldb = K if tB else N
    dA, dB = H.dev(A), H.dev(Bm)
    dC = torch.empty((M, N), dtype=torch.float32 if c_f32 else torch.int16, device="cuda")
    ws = torch.empty(B.gemm_workspace_bytes(B.DTYPE_BF16, M, N, K), dtype=torch.uint8, device="cuda")

    def call():
        B.gemm_bf16(0, tB, M, N, K, dA, K, dB, ldb, 0.0, dC, N, c_f32, workspace=ws)

    call()
    torch.cuda.synchronize()
    rule_plan = (B.gemm_variant_name(B.gemm_last_variant()), B.gemm_last_split())
    t_rule = _time(call)
    say(f"tune {M}x{N}x{K} tB={tB}: rule table -> {rule_plan} {t_rule:.2f} us")
    name, split, us = B.gemm_tune(B.DTYPE_BF16, 0, tB, M, N, K, dA, K, dB, ldb, dC, N, c_f32, workspace=ws)
    say(f"   measured best -> ({name}, {split}) {us:.2f} us")
    assert name in B.variants() and 1 <= split <= 16 and us > 0
    dC.zero_()
    call()
    torch.cuda.synchronize()
    assert (B.gemm_variant_name(B.gemm_last_variant()), B.gemm_last_split()) == (name, split)
    got = dC.cpu().numpy()
    got = got.astype(np.float64) if c_f32 else H.widen(got.view(np.uint16))
    ref = oracle.gemm_ref(A, K, Bm, ldb, M, N, K, transB=tB)
    assert H.rel_fro(got, ref) <= (H.TOL_BF16_F32OUT if c_f32 else H.TOL_BF16)
    t_tuned = _time(call)
    say(f"   tuned plan in use: {t_tuned:.2f} us")
    assert t_tuned <= 1.15 * t_rule, "the measured plan must not lose to the rule table's beyond noise"
    # without a workspace a tuned split cannot run: the call falls back to the rules
    B.gemm_bf16(0, tB, M, N, K, dA, K, dB, ldb, 0.0, dC, N, c_f32)
    torch.cuda.synchronize()
    assert B.gemm_last_split() == 1
    B.gemm_tune_reset()
    call()
    torch.cuda.synchronize()
    assert (B.gemm_variant_name(B.gemm_last_variant()), B.gemm_last_split()) == rule_plan
