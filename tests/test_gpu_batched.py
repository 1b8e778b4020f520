"""GPU parity of the batched (non-reduce) matmul entry points (Section 5(d)): every
matrix of the batch against the oracle's plain product."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from paper_2511_13764_amd import binding as B
from paper_2511_13764_amd import workloads as W

import gpu_helpers as H

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def run_batched(dtype, tA, tB, M, N, K, nmat, *, share_b=False, beta=0.0, c_f32=True, pad=0, seed=90):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    lda, ldb, ldc = ca + pad, cb + pad, N + pad
    sA, sC = ra * lda + 8 * pad, M * ldc + 8 * pad
    sB = 0 if share_b else rb * ldb + 8 * pad
    A = np.full((nmat, sA), np.nan, np.float32)
    Bm = np.full((1 if share_b else nmat, rb * ldb + 8 * pad), np.nan, np.float32)
    As, Bs = [], []
    for z in range(nmat):
        a = W.normal_f32(seed, 10 * z, (ra, ca))
        A[z, :ra * lda].reshape(ra, lda)[:, :ca] = a
        As.append(a)
    for z in range(1 if share_b else nmat):
        b = W.normal_f32(seed, 10 * z + 1, (rb, cb))
        Bm[z, :rb * ldb].reshape(rb, ldb)[:, :cb] = b
        Bs.append(b)
    C0 = W.normal_f32(seed, 5, (nmat, M, N))
    if dtype == "bf16":
        A, Bm = W.to_bf16_bits(A), W.to_bf16_bits(Bm)
        As = [W.to_bf16_bits(a) for a in As]
        Bs = [W.to_bf16_bits(b) for b in Bs]
    Cbuf = np.full((nmat, sC), H.SENTINEL_F32 if c_f32 else H.SENTINEL_BF16, dtype=np.float32 if c_f32 else np.uint16)
    C0s = C0 if c_f32 else W.to_bf16_bits(C0)
    for z in range(nmat):
        live = Cbuf[z, :M * ldc].reshape(M, ldc)[:, :N]
        live[...] = C0s[z] if beta != 0.0 else (np.float32(np.nan) if c_f32 else W.BF16_NAN)
    dA, dB, dC = H.dev(A), H.dev(Bm), H.dev(Cbuf)
    if dtype == "bf16":
        B.gemm_bf16_batched(tA, tB, M, N, K, nmat, dA, lda, sA, dB, ldb, sB, beta, dC, ldc, sC, c_f32)
    else:
        B.gemm_f32_batched(tA, tB, M, N, K, nmat, dA, lda, sA, dB, ldb, sB, beta, dC, ldc, sC)
    torch.cuda.synchronize()
    out = H.host(dC, as_uint16=not c_f32)
    return out, As, Bs, C0s, (ldc, sC)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,nmat,pad", [(512, 512, 64, 6, 0), (256, 384, 128, 3, 8), (100, 72, 40, 5, 3),
                                            (128, 1024, 256, 4, 0), (1, 1, 1, 2, 0)])
def test_batched_matches_per_matrix_oracle(oracle, dtype, tA, tB, M, N, K, nmat, pad):
    beta = -0.5
    out, As, Bs, C0s, (ldc, sC) = run_batched(dtype, tA, tB, M, N, K, nmat, beta=beta, pad=pad)
    say(f"batched {dtype} t{tA}{tB} {M}x{N}x{K} x{nmat} pad={pad} -> {B.gemm_variant_name(B.gemm_last_variant())}")
    for z in range(nmat):
        ref = oracle.gemm_ref(As[z], As[z].shape[1], Bs[z], Bs[z].shape[1], M, N, K, transA=tA, transB=tB,
                              beta=beta, C0=C0s[z], ldc0=N)
        full = out[z, :M * ldc].reshape(M, ldc)
        H.check_padding(full, N, True)
        got = H.widen(full[:, :N])
        assert np.isfinite(got).all(), "padding (NaN) leaked into the result"
        assert H.rel_fro(got, ref) <= 1e-5, z
        if sC > M * ldc:
            assert (out[z, M * ldc:] == H.SENTINEL_F32).all(), "wrote between the C matrices"


def test_batched_shared_b_bf16_out_and_large_grid(oracle):
    """One weight matrix for all products (strideB = 0), bf16 results, enough tiles for the
    256x256 kernel; and a batch whose tile count selects it only through the batch."""
    M, N, K, nmat = 512, 768, 256, 24           # 24 tiles of 128x128 per matrix: 576 in all
    out, As, Bs, _, (ldc, sC) = run_batched("bf16", 0, 1, M, N, K, nmat, share_b=True, c_f32=False)
    used = B.gemm_variant_name(B.gemm_last_variant())
    say(f"batched shared-B -> {used}")
    assert used == "bf16_pingpong_256x256x64"
    for z in range(nmat):
        ref = oracle.gemm_ref(As[z], K, Bs[0], K, M, N, K, transA=0, transB=1)
        got = H.widen(out[z, :M * ldc].reshape(M, ldc)[:, :N])
        assert H.rel_fro(got, ref) <= H.TOL_BF16, z


def test_batched_equals_separate_calls_bit_for_bit():
    """The same kernel runs each matrix: a batched call and nmat single calls agree exactly."""
    M, N, K, nmat = 256, 256, 512, 4
    A = torch.randn((nmat, M, K), device="cuda").to(torch.bfloat16)
    Bm = torch.randn((nmat, K, N), device="cuda").to(torch.bfloat16)
    C1 = torch.empty((nmat, M, N), device="cuda", dtype=torch.float32)
    C2 = torch.empty_like(C1)
    B.gemm_bf16_batched(0, 0, M, N, K, nmat, A, K, M * K, Bm, N, K * N, 0.0, C1, N, M * N, 1)
    v = B.gemm_last_variant()
    B.gemm_force_variant(v, 1)
    try:
        for z in range(nmat):
            B.gemm_bf16(0, 0, M, N, K, A[z], K, Bm[z], N, 0.0, C2[z], N, 1)
    finally:
        B.gemm_force_variant(-1, 0)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)
