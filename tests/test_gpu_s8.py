"""GPU parity of the int8 path: int8 x int8 -> int32, bit for bit against the oracle's
exact integer product (integer work has no tolerance)."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from paper_2511_13764_amd import binding as B

pytestmark = pytest.mark.gpu

CANARY = np.int32(-1234567)


def say(msg):
    print(f"[case] {msg}", flush=True)


def make(seed, M, N, K, tA, tB, pad=0):
    rng = np.random.default_rng(seed)
    Al = rng.integers(-128, 128, (M, K)).astype(np.int8)
    Bl = rng.integers(-128, 128, (K, N)).astype(np.int8)
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = rng.integers(-128, 128, (ra, ca + pad)).astype(np.int8)       # padding holds junk that must not be read as data
    Bm = rng.integers(-128, 128, (rb, cb + pad)).astype(np.int8)
    A[:, :ca] = Al.T if tA else Al
    Bm[:, :cb] = Bl.T if tB else Bl
    return A, Bm


def run_s8(A, Bm, M, N, K, tA, tB, *, C0=None, ldc=None, force=None):
    ldc = ldc or N
    cbuf = np.full((M, ldc), CANARY, np.int32)
    if C0 is not None:
        cbuf[:, :N] = C0
    dA, dB, dC = torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), torch.from_numpy(cbuf).cuda()
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        B.gemm_s8(tA, tB, M, N, K, dA, A.shape[1], dB, Bm.shape[1], C0 is not None, dC, ldc)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = dC.cpu().numpy()
    assert (full[:, N:] == CANARY).all(), "wrote outside the N live columns"
    return full[:, :N]


def as_i32(x):
    """int64 reference -> the int32 the hardware keeps (wrap-around, never hit in these tests)."""
    assert np.abs(x).max() < 2 ** 31
    return x.astype(np.int32)


def test_s8_every_variant_nt(oracle):
    M, N, K = 512, 768, 512
    A, Bm = make(1, M, N, K, 0, 1)
    ref = as_i32(oracle.gemm_s8_ref(A, K, Bm, K, M, N, K, transB=1))
    ran = set()
    for v, name in enumerate(B.variants()):
        say(f"s8 variant={name}")
        try:
            out = run_s8(A, Bm, M, N, K, 0, 1, force=(v, 1))
        except B.BrgemmError as e:
            assert e.code == B.INVALID_ARG
            continue
        ran.add(name)
        assert (out == ref).all(), name
    assert {"generic_64x64x16_f32mfma", "bf16_128x128x64", "bf16_pingpong_256x256x64", "bf16_stream_32x128x64",
            "bf16_stream_64x128x64", "bf16_stream_128x128x64"} <= ran
    # a split of the integer sum is refused rather than done in floating point
    with pytest.raises(B.BrgemmError):
        run_s8(A, Bm, M, N, K, 0, 1, force=(B.variants().index("bf16_128x128x64"), 2))


MFMA_VARIANTS = {"bf16_128x128x64", "bf16_pingpong_256x256x64", "bf16_stream_32x128x64", "bf16_stream_64x128x64",
                 "bf16_stream_128x128x64"}


@pytest.mark.parametrize("tA,tB", [(0, 0), (1, 0), (1, 1)])
def test_s8_every_variant_other_layouts(oracle, tA, tB):
    """Operands contiguous in m / n (read out of LDS with the transposing one-byte read) through
    every matrix-instruction kernel; the 32- and 64-row tiles need a k-contiguous A."""
    M, N, K = 512, 768, 512
    A, Bm = make(11 + 2 * tA + tB, M, N, K, tA, tB)
    ref = as_i32(oracle.gemm_s8_ref(A, A.shape[1], Bm, Bm.shape[1], M, N, K, transA=tA, transB=tB))
    ran = set()
    for v, name in enumerate(B.variants()):
        say(f"s8 t{tA}{tB} variant={name}")
        try:
            out = run_s8(A, Bm, M, N, K, tA, tB, force=(v, 1))
        except B.BrgemmError as e:
            assert e.code == B.INVALID_ARG
            continue
        ran.add(name)
        assert (out == ref).all(), name
    expect = set(MFMA_VARIANTS) if tA == 0 else MFMA_VARIANTS - {"bf16_stream_32x128x64", "bf16_stream_64x128x64"}
    assert ran == expect | {"generic_64x64x16_f32mfma"}


@pytest.mark.parametrize("tA,tB", [(0, 0), (1, 0), (1, 1)])
@pytest.mark.parametrize("name", ["bf16_pingpong_256x256x64", "bf16_stream_128x128x64", "bf16_128x128x64"])
def test_s8_edge_tiles_other_layouts(oracle, name, tA, tB):
    """Tiles that overhang the matrix by whole 16-byte chunks in the contiguous direction, padded rows."""
    M, N, K = 256 + 112, 512 + 16, 1024
    A, Bm = make(21 + 2 * tA + tB, M, N, K, tA, tB, pad=16)
    ref = as_i32(oracle.gemm_s8_ref(A, A.shape[1], Bm, Bm.shape[1], M, N, K, transA=tA, transB=tB))
    out = run_s8(A, Bm, M, N, K, tA, tB, force=(B.variants().index(name), 1))
    assert (out == ref).all()


def test_s8_nn_full_size_takes_the_pingpong_kernel(oracle):
    M = N = K = 4096
    A, Bm = make(7, M, N, K, 0, 0)
    rng = np.random.default_rng(8)
    rows = sorted(set([0, 1, 15, 16, 127, 128, 255, 256, M - 1] + rng.integers(0, M, 12).tolist()))
    out = run_s8(A, Bm, M, N, K, 0, 0)
    assert B.gemm_variant_name(B.gemm_last_variant()) == "bf16_pingpong_256x256x64"
    ref = oracle.gemm_s8_ref(np.ascontiguousarray(A[rows]), K, Bm, N, len(rows), N, K)
    assert (out[rows] == as_i32(ref)).all()


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,pad", [(257, 131, 67, 3), (1, 1, 1, 0), (360, 520, 1024, 16), (16, 384, 2048, 0),
                                       (100, 72, 128, 5), (128, 256, 0, 0), (368, 528, 1024, 16), (1040, 2064, 256, 0)])
def test_s8_all_layouts_ragged_accumulate(oracle, M, N, K, pad, tA, tB):
    A, Bm = make(2 + M + K, M, N, K, tA, tB, pad=pad)
    if K == 0:
        A, Bm = np.zeros((max(A.shape[0], 1), 16), np.int8), np.zeros((max(Bm.shape[0], 1), 16), np.int8)
    rng = np.random.default_rng(3)
    C0 = rng.integers(-10 ** 6, 10 ** 6, (M, N)).astype(np.int32)
    ref = oracle.gemm_s8_ref(A, A.shape[1], Bm, Bm.shape[1], M, N, K, transA=tA, transB=tB)
    say(f"s8 {M}x{N}x{K} t{tA}{tB} pad={pad}")
    out = run_s8(A, Bm, M, N, K, tA, tB, ldc=N + pad)
    assert (out == as_i32(ref)).all(), B.gemm_variant_name(B.gemm_last_variant())
    out = run_s8(A, Bm, M, N, K, tA, tB, C0=C0, ldc=N + pad)
    assert (out == as_i32(ref + C0)).all(), B.gemm_variant_name(B.gemm_last_variant())


def test_s8_edge_tiles_pingpong(oracle):
    """Tiles that overhang the matrix, whole wave-loads skipped, 256x256 kernel forced."""
    M, N, K = 256 + 104, 512 + 8, 1024
    A, Bm = make(4, M, N, K, 0, 1)
    ref = as_i32(oracle.gemm_s8_ref(A, K, Bm, K, M, N, K, transB=1))
    out = run_s8(A, Bm, M, N, K, 0, 1, force=(B.variants().index("bf16_pingpong_256x256x64"), 1))
    assert (out == ref).all()


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 4096), (16, 11008, 4096), (128, 4096, 11008)])
def test_s8_full_size_sampled_rows(oracle, M, N, K):
    """Headline-size launches; complete rows of C checked (each row is an exact 1 x K x N product)."""
    A, Bm = make(5, M, N, K, 0, 1)
    rng = np.random.default_rng(6)
    rows = sorted(set([0, 1, 15, 16, 127, 128, 255, 256, M - 1] + rng.integers(0, M, 12).tolist()))
    rows = [r for r in rows if r < M]
    out = run_s8(A, Bm, M, N, K, 0, 1)
    say(f"s8 {M}x{N}x{K} -> {B.gemm_variant_name(B.gemm_last_variant())}")
    ref = oracle.gemm_s8_ref(np.ascontiguousarray(A[rows]), K, Bm, K, len(rows), N, K, transB=1)
    assert (out[rows] == as_i32(ref)).all()


def test_s8_extreme_values_no_saturation(oracle):
    """-128 * -128 summed over K = 4096 stays exact (no saturating arithmetic anywhere)."""
    M, N, K = 128, 128, 4096
    A = np.full((M, K), -128, np.int8)
    Bm = np.full((N, K), -128, np.int8)
    Bm[::2] = 127
    out = run_s8(A, Bm, M, N, K, 0, 1)
    ref = as_i32(oracle.gemm_s8_ref(A, K, Bm, K, M, N, K, transB=1))
    assert (out == ref).all() and out[0, 1] == 16384 * K and out[0, 0] == -128 * 127 * K
