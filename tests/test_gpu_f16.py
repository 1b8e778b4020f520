"""GPU parity of the binary16 (FP16) operand path against the oracle: same kernels as
bf16 with the f16 matrix instruction and f16 narrowing in the epilogue."""
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

TOL_F16_OUT = 2.5e-4        # one rounding to 11 significant bits: 2^-12 / sqrt(3) * ~1.4 relative RMS
TOL_F32_OUT = 1e-5


def say(msg):
    print(f"[case] {msg}", flush=True)


def widen16(bits):
    return bits.view(np.float16).astype(np.float64)


def run_f16(A, lda, Bm, ldb, M, N, K, tA, tB, *, beta=0.0, C0=None, c_f32=True, ldc=None, workspace_bytes=0,
            force=None, bias=None, relu=False):
    """A, Bm, C0: numpy float16 arrays (C0 float32 when c_f32).  Returns the live part of C."""
    ldc = ldc or N
    if c_f32:
        cbuf = np.full((M, ldc), H.SENTINEL_F32, dtype=np.float32)
        cbuf[:, :N] = C0 if beta != 0.0 else np.float32(np.nan)
    else:
        cbuf = np.full((M, ldc), np.float16(-7777.0), dtype=np.float16)
        cbuf[:, :N] = C0 if beta != 0.0 else np.float16(np.nan)
    dA = torch.from_numpy(A.view(np.int16)).cuda()
    dB = torch.from_numpy(Bm.view(np.int16)).cuda()
    dC = torch.from_numpy(cbuf if c_f32 else cbuf.view(np.int16)).cuda()
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    dbias = H.dev(bias) if bias is not None else None
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        if bias is not None or relu:
            epi = (B.EPI_BIAS if bias is not None else 0) | (B.EPI_RELU if relu else 0)
            B.brgemm_fused(B.DTYPE_F16, tA, tB, M, N, K, 1, dA, None, lda, dB, None, ldb, beta, dC, ldc, c_f32,
                           dbias, epi, workspace=ws)
        else:
            B.gemm_f16(tA, tB, M, N, K, dA, lda, dB, ldb, beta, dC, ldc, c_f32, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = dC.cpu().numpy()
    if c_f32:
        assert (full[:, N:] == H.SENTINEL_F32).all()
        return full[:, :N].astype(np.float64)
    full = full.view(np.float16)
    assert (full[:, N:] == np.float16(-7777.0)).all()
    return full[:, :N].astype(np.float64)


def operands(seed, M, N, K, tA, tB, pad=0, scale_b=1.0):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((ra, ca + pad), np.nan, np.float16)
    Bm = np.full((rb, cb + pad), np.nan, np.float16)
    A[:, :ca] = W.normal_f32(seed, 0, (ra, ca)).astype(np.float16)
    Bm[:, :cb] = (W.normal_f32(seed, 1, (rb, cb)) * scale_b).astype(np.float16)
    return A, Bm


def test_f16_every_variant_all_transposes(oracle):
    M, N, K = 512, 768, 512
    ws = B.gemm_workspace_bytes(B.DTYPE_F16, M, N, K)
    for tA, tB in [(0, 0), (0, 1), (1, 0), (1, 1)]:
        A, Bm = operands(95, M, N, K, tA, tB)
        ref = oracle.gemm_ref(A, A.shape[1], Bm, Bm.shape[1], M, N, K, transA=tA, transB=tB)
        ran = set()
        for v, name in enumerate(B.variants()):
            for split in (1, 2):
                say(f"f16 t{tA}{tB} variant={name} split={split}")
                try:
                    out = run_f16(A, A.shape[1], Bm, Bm.shape[1], M, N, K, tA, tB, workspace_bytes=ws,
                                  force=(v, split))
                except B.BrgemmError as e:
                    assert e.code == B.INVALID_ARG
                    continue
                ran.add(name)
                assert H.rel_fro(out, ref) <= TOL_F32_OUT, (name, split)
        assert {"generic_64x64x16_f32mfma", "bf16_128x128x64", "bf16_pingpong_256x256x64",
                "bf16_stream_128x128x64"} <= ran


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (257, 131, 67), (33, 520, 1000), (16, 384, 1024)])
def test_f16_small_integers_bit_exact(oracle, M, N, K, tA, tB):
    Al = W.small_int_matrix(96, (M, K)).astype(np.float16)
    Bl = W.small_int_matrix(97, (K, N)).astype(np.float16)
    A = np.ascontiguousarray(Al.T if tA else Al)
    Bm = np.ascontiguousarray(Bl.T if tB else Bl)
    want = (Al.astype(np.int64) @ Bl.astype(np.int64)).astype(np.float64)
    out = run_f16(A, A.shape[1], Bm, Bm.shape[1], M, N, K, tA, tB)
    assert (out == want).all()
    if np.abs(want).max() <= 2048:           # exactly representable in binary16 as well
        out16 = run_f16(A, A.shape[1], Bm, Bm.shape[1], M, N, K, tA, tB, c_f32=False)
        assert (out16 == want).all()


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,pad", [(300, 260, 520, 8), (129, 1000, 64, 16), (100, 72, 24, 3), (1024, 1024, 1024, 0)])
def test_f16_ragged_padded_beta_f16_out(oracle, M, N, K, pad, tA, tB):
    """binary16 C with beta != 0 (widened, scaled and rounded once), padded leading dimensions
    with NaN in the padding; the narrowing is checked bit for bit against the oracle's rounding."""
    A, Bm = operands(98, M, N, K, tA, tB, pad=pad)
    C0 = W.normal_f32(98, 2, (M, N)).astype(np.float16)
    say(f"f16 ragged {M}x{N}x{K} t{tA}{tB} pad={pad}")
    ref = oracle.gemm_ref(A, A.shape[1], Bm, Bm.shape[1], M, N, K, transA=tA, transB=tB, beta=-0.75, C0=C0, ldc0=N)
    out = run_f16(A, A.shape[1], Bm, Bm.shape[1], M, N, K, tA, tB, beta=-0.75, C0=C0, c_f32=False, ldc=N + pad,
                  workspace_bytes=B.gemm_workspace_bytes(B.DTYPE_F16, M, N, K))
    assert np.isfinite(out).all()
    assert H.rel_fro(out, ref) <= TOL_F16_OUT
    # the GPU rounds an fp32 sum, the oracle an fp64 one: they may differ only where the
    # exact value sits within the fp32 summation error of a rounding boundary
    want_bits = oracle.round_to_out(ref, 2).view(np.uint16)
    got_bits = out.astype(np.float16).view(np.uint16)
    assert (want_bits == got_bits).mean() >= 0.995


def test_f16_subnormal_and_overflow_results(oracle):
    """Results in the binary16 subnormal range keep their subnormal bits; results beyond
    65504 become infinity (the oracle's rounding, bit for bit: every sum here is exact)."""
    M, N, K = 32, 128, 64
    A = np.zeros((M, K), np.float16)
    Bm = np.zeros((K, N), np.float16)
    A[:, 0] = np.float16(2.0 ** -10)
    Bm[0, :] = (np.arange(N) * 2.0 ** -18).astype(np.float16)       # products k * 2^-28: subnormal range
    A[5, 1] = np.float16(300.0)
    Bm[1, 7] = np.float16(300.0)                                     # 90000 > 65504
    ref = oracle.gemm_ref(A, K, Bm, N, M, N, K)
    out = run_f16(A, K, Bm, N, M, N, K, 0, 0, c_f32=False)
    want = oracle.round_to_out(ref, 2)
    assert np.isinf(want[5, 7]) and (want[0, 1:40] != 0).any()
    assert (out.astype(np.float16).view(np.uint16) == want.view(np.uint16)).all()


def test_f16_fused_bias_relu_and_scattered_batch(oracle):
    M, N, K = 192, 520, 256
    A, Bm = operands(99, M, N, K, 0, 1)
    bias = W.normal_f32(99, 3, (N,))
    ref = oracle.gemm_ref(A, K, Bm, K, M, N, K, transB=1, bias=bias, relu=True)
    out = run_f16(A, K, Bm, K, M, N, K, 0, 1, bias=bias, relu=True, workspace_bytes=B.gemm_workspace_bytes(2, M, N, K))
    assert H.rel_fro(out, ref) <= TOL_F32_OUT and (out >= 0).all()
    # batch-reduce over scattered tiles of one pool (NaN between the tiles)
    m, n, k, batch = 128, 256, 64, 9
    rng = np.random.default_rng(5)
    pool = np.full(1 << 20, np.nan, np.float16)
    slots = rng.permutation(64)[: 2 * batch] * 16384
    a_off, b_off = slots[:batch].astype(np.int64), slots[batch:].astype(np.int64)
    for i in range(batch):
        pool[a_off[i]: a_off[i] + m * k] = W.normal_f32(99, 10 + i, (m * k,)).astype(np.float16)
        pool[b_off[i]: b_off[i] + k * n] = W.normal_f32(99, 40 + i, (k * n,)).astype(np.float16)
    ref = oracle.brgemm_ref(pool, a_off, k, pool, b_off, n, m, n, k)
    dpool = torch.from_numpy(pool.view(np.int16)).cuda()
    dC = torch.full((m, n), float("nan"), device="cuda")
    B.brgemm_fused(B.DTYPE_F16, 0, 0, m, n, k, batch, dpool, torch.from_numpy(a_off).cuda(), k, dpool,
                   torch.from_numpy(b_off).cuda(), n, 0.0, dC, n, 1, None, 0,
                   workspace=torch.empty(B.gemm_workspace_bytes(2, m, n, k, batch), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert H.rel_fro(dC.cpu().numpy().astype(np.float64), ref) <= TOL_F32_OUT


@pytest.mark.parametrize("M", [16, 128, 4096])
def test_f16_mlp_up_shape_sampled(oracle, M):
    """The MLP up-projection shape with binary16 operands and results (weights N(0, 0.02))."""
    N, K = 11008, 4096
    A, Bm = operands(94, M, N, K, 0, 1, scale_b=0.02)
    rows = H.sample_rows(M, 16) if M > 128 else list(range(M))
    ref = oracle.gemm_ref(A, K, Bm, K, M, N, K, transB=1, rows=rows)
    out = run_f16(A, K, Bm, K, M, N, K, 0, 1, c_f32=False, workspace_bytes=B.gemm_workspace_bytes(2, M, N, K))
    say(f"f16 mlp up M={M} -> {B.gemm_variant_name(B.gemm_last_variant())} split={B.gemm_last_split()}")
    assert H.rel_fro(out[rows], ref) <= TOL_F16_OUT
