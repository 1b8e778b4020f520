"""GPU parity of the FP8 (E4M3) operand path: the oracle widens the same bytes exactly
(its own decoder) and multiplies them in fp64."""
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

# The 128-deep FP8 matrix instruction does not add its 128 products one by one in fp32: it
# aligns them to the largest exponent of the group and keeps a fixed number of bits, so the
# relative Frobenius error against the exact result is ~1.3e-5 on N(0,1) operands (measured;
# the general kernel, which widens to fp32 first, stays below 1e-6).  The bound used here
# leaves a factor of 4 over the measurement and is still 30x tighter than one bf16 rounding.
TOL_F32_OUT = 5e-5


def say(msg):
    print(f"[case] {msg}", flush=True)


def f8_bytes(seed, tensor, shape, scale=1.0):
    """N(0, scale) values rounded to E4M3 by the library conversion (input generation only)."""
    x = torch.from_numpy(W.normal_f32(seed, tensor, shape) * np.float32(scale))
    return x.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()


def run_f8(A, Bm, M, N, K, tA, tB, *, beta=0.0, C0=None, c_f32=True, ldc=None, workspace_bytes=0, force=None):
    ldc = ldc or N
    cbuf = H.make_c(M, N, ldc, c_f32, C0, beta)
    dA, dB, dC = torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), H.dev(cbuf)
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        B.gemm_f8(tA, tB, M, N, K, dA, A.shape[1], dB, Bm.shape[1], beta, dC, ldc, c_f32, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = H.host(dC, as_uint16=not c_f32)
    H.check_padding(full, N, c_f32)
    return H.widen(full[:, :N])


def ref_f8(oracle, A, Bm, M, N, K, tA, tB, **kw):
    Aw, Bw = oracle.f8e4m3_widen(A), oracle.f8e4m3_widen(Bm)
    return oracle.gemm_ref(Aw, Aw.shape[1], Bw, Bw.shape[1], M, N, K, transA=tA, transB=tB, **kw)


def test_f8_every_variant_nt(oracle):
    M, N, K = 512, 768, 512
    A, Bm = f8_bytes(300, 0, (M, K)), f8_bytes(300, 1, (N, K))
    ref = ref_f8(oracle, A, Bm, M, N, K, 0, 1)
    ws = B.gemm_workspace_bytes(1, M, N, K)
    ran = set()
    for v, name in enumerate(B.variants()):
        for split in (1, 2):
            say(f"f8 variant={name} split={split}")
            try:
                out = run_f8(A, Bm, M, N, K, 0, 1, workspace_bytes=ws, force=(v, split))
            except B.BrgemmError as e:
                assert e.code == B.INVALID_ARG
                continue
            ran.add(name)
            err = H.rel_fro(out, ref)
            say(f"   rel. Frobenius error {err:.2e}")
            assert err <= (1e-6 if name.startswith("generic") else TOL_F32_OUT), (name, split)
    assert {"generic_64x64x16_f32mfma", "bf16_pingpong_256x256x64", "bf16_stream_32x128x64",
            "bf16_stream_64x128x64", "bf16_stream_128x128x64"} <= ran
    assert "bf16_128x128x64" not in ran


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,pad", [(257, 131, 67, 3), (360, 520, 1024, 16), (16, 384, 2048, 0), (128, 256, 128, 0)])
def test_f8_all_layouts_ragged_beta_bf16_out(oracle, M, N, K, pad, tA, tB):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((ra, ca + pad), 0x7F, np.uint8)          # NaN in the padding
    Bm = np.full((rb, cb + pad), 0x7F, np.uint8)
    A[:, :ca] = f8_bytes(301, 0, (ra, ca))
    Bm[:, :cb] = f8_bytes(301, 1, (rb, cb))
    C0 = W.to_bf16_bits(W.normal_f32(301, 2, (M, N)))
    say(f"f8 {M}x{N}x{K} t{tA}{tB} pad={pad}")
    ref = ref_f8(oracle, A, Bm, M, N, K, tA, tB, beta=-0.5, C0=C0, ldc0=N)
    out = run_f8(A, Bm, M, N, K, tA, tB, beta=-0.5, C0=C0, c_f32=False, ldc=N + pad,
                 workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
    assert np.isfinite(out).all()
    assert H.rel_fro(out, ref) <= H.TOL_BF16, B.gemm_variant_name(B.gemm_last_variant())


def test_f8_small_integers_and_extremes_bit_exact(oracle):
    """Integer-valued E4M3 operands (every partial sum exact in fp32) and the extreme codes."""
    M, N, K = 256, 384, 1024
    codes = np.array([0x00, 0x38, 0xB8, 0x40, 0xC0, 0x44, 0xC4, 0x48, 0xC8], np.uint8)    # 0, +-1, +-2, +-3, +-4
    rng = np.random.default_rng(8)
    A, Bm = rng.choice(codes, (M, K)), rng.choice(codes, (N, K))
    ref = ref_f8(oracle, A, Bm, M, N, K, 0, 1)
    out = run_f8(A, Bm, M, N, K, 0, 1)
    assert (out == ref).all()
    A[:] = 0x7E                                                     # 448
    Bm[:] = 0xFE                                                    # -448
    Bm[::2] = 0x01                                                  # 2^-9, the smallest subnormal
    ref = ref_f8(oracle, A, Bm, M, N, K, 0, 1)
    out = run_f8(A, Bm, M, N, K, 0, 1)
    assert (out == ref).all() and out[0, 1] == -448.0 * 448.0 * K and out[0, 0] == 448.0 * 2.0 ** -9 * K


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 4096), (16, 11008, 4096), (128, 4096, 11008)])
def test_f8_full_size_sampled_rows(oracle, M, N, K):
    A, Bm = f8_bytes(302, 0, (M, K)), f8_bytes(302, 1, (N, K), scale=0.05)
    rows = H.sample_rows(M, 16) if M > 128 else list(range(M))
    ref = ref_f8(oracle, A, Bm, M, N, K, 0, 1, rows=rows)
    out = run_f8(A, Bm, M, N, K, 0, 1, workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
    say(f"f8 {M}x{N}x{K} -> {B.gemm_variant_name(B.gemm_last_variant())} split={B.gemm_last_split()}")
    assert H.rel_fro(out[rows], ref) <= TOL_F32_OUT
