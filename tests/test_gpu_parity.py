"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Bars (relative Frobenius error against the fp64 oracle): fp32 <= 1e-5; bf16-in /
fp32-accumulate / bf16-out <= 2e-3; bf16-in / fp32-out <= 1e-5.  Integer-valued
inputs must match bit for bit (every partial sum is exact in fp32, whatever the
order of summation).
"""
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


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    B.load()


def _abs_bits(x):
    return x & np.uint16(0x7FFF)


def _tol(case):
    if case.dtype == "f32":
        return H.TOL_F32
    return H.TOL_BF16_F32OUT if case.c_is_f32 else H.TOL_BF16


# ------------------------------------------------------------------ the named configurations

def test_config1_f32_256(oracle):
    case = W.config1_f32_256()
    say(case.name)
    out, _ = H.run_gemm_case(case)
    ref = H.oracle_gemm_case(oracle, case)
    err = H.rel_fro(H.widen(out), ref)
    say(f"{case.name} rel_fro={err:.3e}")
    assert err <= H.TOL_F32


def test_config2_f32_2048_beta(oracle):
    case = W.config2_f32_2048()
    say(case.name)
    out, _ = H.run_gemm_case(case, workspace_bytes=B.gemm_workspace_bytes(0, case.M, case.N, case.K))
    ref = H.oracle_gemm_case(oracle, case)
    err = H.rel_fro(H.widen(out), ref)
    worst = H.check_f32_case_elementwise(oracle, case, out, ref)
    say(f"{case.name} rel_fro={err:.3e}, every element within {worst:.3f} of the fp32 summation bound")
    assert err <= H.TOL_F32


def test_f32_4096_sampled(oracle):
    """fp32 at the size the metric names (4096^3, beta = 0.5), launched as the benchmark times
    it; the oracle computes sampled complete rows (first / last / interior tiles, both halves
    of every wave tile)."""
    case = W.config2_f32_2048(size=4096)
    say(case.name)
    out, _ = H.run_gemm_case(case, workspace_bytes=B.gemm_workspace_bytes(0, case.M, case.N, case.K))
    assert B.gemm_variant_name(B.gemm_last_variant()) == "f32_128x128x32"
    rows = H.sample_rows(4096, 64, tile=128)
    ref = H.oracle_gemm_case(oracle, case, rows=rows)
    err = H.rel_fro(H.widen(out[rows]), ref)
    H.check_f32_case_elementwise(oracle, case, out[rows], ref, rows=rows)
    say(f"{case.name} rows={len(rows)} rel_fro={err:.3e}")
    assert err <= H.TOL_F32


@pytest.mark.parametrize("size", [1024, 2048])
def test_config3_bf16_square_full(oracle, size):
    case = W.config3_bf16_square(size)
    say(case.name)
    out, _ = H.run_gemm_case(case, workspace_bytes=B.gemm_workspace_bytes(1, size, size, size))
    ref = H.oracle_gemm_case(oracle, case)
    err = H.rel_fro(H.widen(out), ref)
    # second figure: against the oracle rounded once to bf16 (isolates kernel error)
    err_out = H.rel_fro(H.widen(out), H.widen(oracle.round_to_out(ref, 1)))
    say(f"{case.name} rel_fro={err:.3e} vs_rounded_oracle={err_out:.3e}")
    assert err <= H.TOL_BF16
    assert err_out <= 1e-3
    abs_ref = oracle.gemm_ref(_abs_bits(case.A), case.lda, _abs_bits(case.B), case.ldb, size, size, size)
    H.check_bf16_out_elementwise(oracle, out, ref, abs_ref, size, what=case.name)
    # fp32-out variant of the same problem
    case.c_is_f32 = True
    out32, _ = H.run_gemm_case(case)
    err32 = H.rel_fro(H.widen(out32), ref)
    say(f"{case.name} fp32-out rel_fro={err32:.3e}")
    assert err32 <= H.TOL_BF16_F32OUT


@pytest.mark.parametrize("size", [4096, 8192])
def test_config3_bf16_square_sampled(oracle, size):
    """Full-size launch as the benchmark times it; the oracle computes sampled complete rows."""
    case = W.config3_bf16_square(size)
    say(case.name)
    out, _ = H.run_gemm_case(case, workspace_bytes=B.gemm_workspace_bytes(1, size, size, size))
    rows = H.sample_rows(size, 96 if size == 4096 else 48)
    ref = H.oracle_gemm_case(oracle, case, rows=rows)
    err = H.rel_fro(H.widen(out[rows]), ref)
    say(f"{case.name} rows={len(rows)} rel_fro={err:.3e}")
    assert err <= H.TOL_BF16
    # column sample: every row, a few full columns, via the transposed problem (A B)^T = B^T A^T
    cols = [0, 1, 255, 256, size // 2, size - 257, size - 1]
    refT = oracle.gemm_ref(case.B, case.ldb, case.A, case.lda, size, size, size, transA=1, transB=1, rows=cols)
    errc = H.rel_fro(H.widen(out[:, cols]).T, refT)
    say(f"{case.name} cols={len(cols)} rel_fro={errc:.3e}")
    assert errc <= H.TOL_BF16


@pytest.mark.parametrize("which", ["square4096", "mlp_up4096"])
def test_whole_c_elementwise_at_full_size(oracle, which):
    """The benchmark's headline problem (bf16 4096^3 NN, bf16 out) and the M = 4096
    up-projection (NT), launched as the benchmark launches them, with EVERY element of C
    compared with the oracle: a per-element bound (one bf16 rounding plus the fp32
    summation bound, see check_bf16_out_elementwise), at most one bf16 step from the
    oracle's own rounding, and the Frobenius gate."""
    case = W.config3_bf16_square(4096) if which == "square4096" else W.config4_mlp(4096, "up")
    say(case.name)
    ws = min(B.gemm_workspace_bytes(1, case.M, case.N, case.K), 1 << 30)
    out, _ = H.run_gemm_case(case, workspace_bytes=ws)
    assert B.gemm_variant_name(B.gemm_last_variant()) == "bf16_pingpong_256x256x64"
    ref = H.oracle_gemm_case(oracle, case)
    abs_ref = oracle.gemm_ref(_abs_bits(case.A), case.lda, _abs_bits(case.B), case.ldb, case.M, case.N, case.K,
                              transA=case.transA, transB=case.transB)
    err = H.rel_fro(H.widen(out), ref)
    worst, frac = H.check_bf16_out_elementwise(oracle, out, ref, abs_ref, case.K, what=case.name)
    say(f"{case.name} all {case.M * case.N} elements: rel_fro={err:.3e} worst |err|/bound={worst:.3f} "
        f"differ from the oracle's rounding: {frac:.2e}")
    assert err <= H.TOL_BF16


@pytest.mark.parametrize("which", ["up", "down"])
@pytest.mark.parametrize("M", [16, 128, 4096])
def test_config4_mlp_shapes(oracle, which, M):
    case = W.config4_mlp(M, which)
    say(case.name)
    ws = B.gemm_workspace_bytes(1, case.M, case.N, case.K)
    out, _ = H.run_gemm_case(case, workspace_bytes=min(ws, 1 << 30))
    rows = None if M <= 128 else H.sample_rows(M, 40)
    if M == 128:
        rows = H.sample_rows(M, 48, seed=6)
    ref = H.oracle_gemm_case(oracle, case, rows=rows)
    got = H.widen(out if rows is None else out[rows])
    err = H.rel_fro(got, ref)
    say(f"{case.name} variant={B.gemm_variant_name(B.gemm_last_variant())} split={B.gemm_last_split()} "
        f"rel_fro={err:.3e}")
    assert err <= H.TOL_BF16
    if M == 16:                      # fp32-out variant on the small one
        case.c_is_f32 = True
        out32, _ = H.run_gemm_case(case, workspace_bytes=ws)
        assert H.rel_fro(H.widen(out32), ref) <= H.TOL_BF16_F32OUT


def test_config5_brgemm_scattered_pool(oracle):
    case = W.config5_brgemm()
    say(case.name)
    ws = B.gemm_workspace_bytes(1, case.M, case.N, case.K, case.batch)
    out = H.run_brgemm_case(case, workspace_bytes=ws)
    assert np.isfinite(out).all(), "a read strayed into the NaN canary between the tiles"
    ref = H.oracle_brgemm_case(oracle, case)
    err = H.rel_fro(out, ref)
    say(f"{case.name} variant={B.gemm_variant_name(B.gemm_last_variant())} split={B.gemm_last_split()} "
        f"rel_fro={err:.3e}")
    assert err <= H.TOL_BF16_F32OUT
    # without a workspace the library must still be right (no split possible)
    out2 = H.run_brgemm_case(case, workspace_bytes=0)
    assert H.rel_fro(out2, ref) <= H.TOL_BF16_F32OUT


# ------------------------------------------------------------------ exactness on integer-valued inputs

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (257, 131, 67), (512, 768, 192), (33, 520, 1000)])
def test_small_integer_bit_exact(oracle, dtype, tA, tB, M, N, K):
    Al = W.small_int_matrix(10 + M, (M, K))
    Bl = W.small_int_matrix(20 + N, (K, N))
    As = np.ascontiguousarray(Al.T if tA else Al)
    Bs = np.ascontiguousarray(Bl.T if tB else Bl)
    if dtype == "bf16":
        As, Bs = W.to_bf16_bits(As), W.to_bf16_bits(Bs)
    case = W.GemmCase(f"int_{dtype}_{M}x{N}x{K}_t{tA}{tB}", dtype, M, N, K, tA, tB, 0.0, As, Bs, None, True)
    say(case.name)
    out, _ = H.run_gemm_case(case, ldc=N + 8)
    ref = H.oracle_gemm_case(oracle, case)
    assert np.array_equal(out.astype(np.float64), ref)


# ------------------------------------------------------------------ ragged shapes, padded leading dimensions, misalignment

@pytest.mark.parametrize("dtype,c_f32", [("f32", True), ("bf16", False), ("bf16", True)])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,pad", [(257, 131, 67, 3), (1, 1, 1, 0), (64, 64, 8, 8), (300, 260, 520, 8),
                                       (129, 1000, 64, 16)])
def test_ragged_and_padded(oracle, dtype, c_f32, tA, tB, M, N, K, pad):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((ra, ca + pad), np.nan, np.float32)
    Bm = np.full((rb, cb + pad), np.nan, np.float32)
    A[:, :ca] = W.normal_f32(61, 0, (ra, ca))
    Bm[:, :cb] = W.normal_f32(61, 1, (rb, cb))
    C0 = W.normal_f32(61, 2, (M, N))
    if dtype == "bf16":
        A, Bm = W.to_bf16_bits(A), W.to_bf16_bits(Bm)
    if not c_f32:
        C0 = W.to_bf16_bits(C0)
    case = W.GemmCase(f"ragged_{dtype}_{M}x{N}x{K}_t{tA}{tB}_pad{pad}", dtype, M, N, K, tA, tB, -0.75,
                      A, Bm, C0, c_f32)
    say(case.name)
    out, _ = H.run_gemm_case(case, ldc=N + pad)
    ref = H.oracle_gemm_case(oracle, case)
    assert np.isfinite(H.widen(out)).all(), "padding (NaN) leaked into the result"
    assert H.rel_fro(H.widen(out), ref) <= _tol(case)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_misaligned_bases(oracle, dtype):
    """Operands that start one element into an allocation (2- or 4-byte alignment only)."""
    M, N, K = 130, 260, 136
    A = W.normal_f32(62, 0, (M * K + 1,))
    Bm = W.normal_f32(62, 1, (K * N + 1,))
    if dtype == "bf16":
        A, Bm = W.to_bf16_bits(A), W.to_bf16_bits(Bm)
    dA, dB = H.dev(A), H.dev(Bm)
    dC = torch.full((M * N + 1,), float("nan"), dtype=torch.float32, device="cuda")
    say(f"misaligned_{dtype}")
    if dtype == "f32":
        B.gemm_f32(0, 0, M, N, K, dA[1:], K, dB[1:], N, 0.0, dC[1:], N)
    else:
        B.gemm_bf16(0, 0, M, N, K, dA[1:], K, dB[1:], N, 0.0, dC[1:], N, 1)
    torch.cuda.synchronize()
    out = dC[1:].cpu().numpy().reshape(M, N)
    ref = oracle.gemm_ref(A[1:].reshape(M, K), K, Bm[1:].reshape(K, N), N, M, N, K)
    assert H.rel_fro(out, ref) <= 1e-5
    assert np.isnan(dC[0].item())


# ------------------------------------------------------------------ beta, NaN handling, empty problems

def test_beta_zero_never_reads_c_and_nan_row(oracle):
    M, N, K = 192, 320, 128
    A = W.normal_bf16(63, 0, (M, K))
    Bm = W.normal_bf16(63, 1, (K, N))
    A[77, 5] = W.BF16_NAN
    case = W.GemmCase("nan_row", "bf16", M, N, K, 0, 0, 0.0, A, Bm, None, True)
    say(case.name)
    out, _ = H.run_gemm_case(case)           # C pre-filled with NaN: beta == 0 must ignore it
    assert np.isnan(out[77]).all()
    assert np.isfinite(np.delete(out, 77, axis=0)).all()


@pytest.mark.parametrize("beta", [1.0, 0.5, -2.0])
@pytest.mark.parametrize("c_f32", [True, False])
def test_beta_values(oracle, beta, c_f32):
    M, N, K = 256, 384, 320
    A = W.normal_bf16(64, 0, (M, K))
    Bm = W.normal_bf16(64, 1, (N, K))
    C0 = W.normal_f32(64, 2, (M, N), sigma=10.0)
    if not c_f32:
        C0 = W.to_bf16_bits(C0)
    case = W.GemmCase(f"beta{beta}_cf32{c_f32}", "bf16", M, N, K, 0, 1, beta, A, Bm, C0, c_f32)
    say(case.name)
    out, _ = H.run_gemm_case(case)
    ref = H.oracle_gemm_case(oracle, case)
    assert H.rel_fro(H.widen(out), ref) <= _tol(case)


def test_k_zero_and_batch_zero_scale_c(oracle):
    M, N = 70, 90
    C0 = W.normal_f32(65, 0, (M, N))
    dC = H.dev(C0.copy())
    dummy = torch.zeros(16, dtype=torch.float32, device="cuda")
    say("k_zero")
    B.gemm_f32(0, 0, M, N, 0, dummy, 1, dummy, N, 0.5, dC, N)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), (np.float32(0.5) * C0))
    B.gemm_f32(0, 0, M, N, 0, dummy, 1, dummy, N, 0.0, dC, N)
    torch.cuda.synchronize()
    assert (dC.cpu().numpy() == 0).all()
    dC = H.dev(C0.copy())
    off = torch.zeros(1, dtype=torch.int64, device="cuda")
    B.brgemm_bf16(0, 0, M, N, 8, 0, dummy, off, 8, dummy, off, N, 2.0, dC, N)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.float32(2.0) * C0)


# ------------------------------------------------------------------ batch-reduce: small scattered cases, split, equivalence

@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,batch", [(32, 192, 32, 4), (64, 64, 64, 2), (100, 72, 24, 7), (128, 256, 64, 9)])
def test_brgemm_small_scattered(oracle, tA, tB, M, N, K, batch):
    # first two shapes: the bf16 listings of the paper (Section 2.2 listing; appendix bf16 kernels)
    rng = np.random.default_rng(1234 + M + N + K + batch)
    lda = (M if tA else K) + 8
    ldb = (K if tB else N) + 8
    a_rows, b_rows = (K if tA else M), (N if tB else K)
    a_sz, b_sz = a_rows * lda, b_rows * ldb
    slot = ((max(a_sz, b_sz) + 63) // 64 + 2) * 64
    pool = np.full(slot * 2 * batch + 64, W.BF16_NAN, np.uint16)
    order = rng.permutation(2 * batch)
    A_off = order[:batch].astype(np.int64) * slot + 64
    B_off = order[batch:].astype(np.int64) * slot + 64
    for i in range(batch):
        a = np.full((a_rows, lda), W.BF16_NAN, np.uint16)
        b = np.full((b_rows, ldb), W.BF16_NAN, np.uint16)
        a[:, :lda - 8] = W.normal_bf16(66, i, (a_rows, lda - 8))
        b[:, :ldb - 8] = W.normal_bf16(66, 100 + i, (b_rows, ldb - 8))
        pool[A_off[i]:A_off[i] + a_sz] = a.ravel()
        pool[B_off[i]:B_off[i] + b_sz] = b.ravel()
    C0 = W.normal_f32(66, 999, (M, N))
    case = W.BrgemmCase(f"brgemm_small_{M}x{N}x{K}x{batch}_t{tA}{tB}", M, N, K, batch, tA, tB, 1.0,
                        pool, A_off, B_off, lda, ldb, C0)
    say(case.name)
    ref = H.oracle_brgemm_case(oracle, case)
    out = H.run_brgemm_case(case)
    assert np.isfinite(out).all()
    assert H.rel_fro(out, ref) <= H.TOL_BF16_F32OUT
    # the same through a forced reduction split (partial tiles + fixed-order reduce)
    ws = B.gemm_workspace_bytes(1, M, N, K, batch)
    out_s = H.run_brgemm_case(case, workspace_bytes=ws, force=(0, 3))
    assert H.rel_fro(out_s, ref) <= H.TOL_BF16_F32OUT
    out_s2 = H.run_brgemm_case(case, workspace_bytes=ws, force=(0, 3))
    assert np.array_equal(out_s, out_s2), "split reduction must be deterministic"


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0)])
@pytest.mark.parametrize("odd_tile", [None, 3, 140])
def test_brgemm_more_than_64_tiles_every_variant(oracle, tA, tB, odd_tile):
    """The kernels keep 64 tile offsets at a time in registers: 150 tiles of one k-block each make
    every wave refill that window twice (more often under a split), through every variant.
    odd_tile: one tile starts at an odd element (inside or beyond the first window), which must
    send the kernels to their register-staged loads with identical results."""
    M, N, K, batch = 256, 384, 64, 150
    rng = np.random.default_rng(77 + 2 * tA + tB)
    lda, ldb = (M if tA else K), (K if tB else N)
    a_sz, b_sz = (K if tA else M) * lda, (N if tB else K) * ldb
    slot = max(a_sz, b_sz) + 64
    pool = np.full(slot * 2 * batch + 64, W.BF16_NAN, np.uint16)
    order = rng.permutation(2 * batch)
    A_off = order[:batch].astype(np.int64) * slot + 8 * rng.integers(0, 4, batch)
    B_off = order[batch:].astype(np.int64) * slot + 8 * rng.integers(0, 4, batch)
    if odd_tile is not None:
        A_off[odd_tile] += 3
    for i in range(batch):
        pool[A_off[i]:A_off[i] + a_sz] = W.normal_bf16(67, i, (a_sz,))
        pool[B_off[i]:B_off[i] + b_sz] = W.normal_bf16(67, 1000 + i, (b_sz,))
    case = W.BrgemmCase(f"brgemm_150tiles_t{tA}{tB}_odd{odd_tile}", M, N, K, batch, tA, tB, 0.0,
                        pool, A_off, B_off, lda, ldb, None)
    ref = H.oracle_brgemm_case(oracle, case)
    ws = B.gemm_workspace_bytes(1, M, N, K, batch)
    ran = set()
    for v, name in enumerate(B.variants()):
        for split in (1, 2, 7):
            say(f"{case.name} variant={name} split={split}")
            try:
                out = H.run_brgemm_case(case, workspace_bytes=ws, force=(v, split))
            except B.BrgemmError as e:
                assert e.code == B.INVALID_ARG
                continue
            ran.add(name)
            assert np.isfinite(out).all(), (name, split)
            assert H.rel_fro(out, ref) <= H.TOL_BF16_F32OUT, (name, split)
    want = {"generic_64x64x16_f32mfma", "bf16_128x128x64", "bf16_pingpong_256x256x64", "bf16_stream_128x128x64"}
    if tA == 0:
        want |= {"bf16_stream_32x128x64", "bf16_stream_64x128x64"}
    assert want <= ran, ran


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,batch", [(128, 256, 64, 9), (32, 384, 128, 5), (256, 512, 128, 3)])
def test_brgemm_tile_offsets_not_16_byte_aligned(oracle, tA, tB, M, N, K, batch):
    """Tile offsets live in device memory, so the host cannot route on their alignment: every MFMA
    kernel votes on them and falls back to 2-byte loads staged through registers.  Odd offsets,
    every variant that takes the problem forced in turn, NaN around the tiles."""
    rng = np.random.default_rng(4321 + M + N + K + batch + 2 * tA + tB)
    lda = (M if tA else K) + 8
    ldb = (K if tB else N) + 8
    a_rows, b_rows = (K if tA else M), (N if tB else K)
    a_sz, b_sz = a_rows * lda, b_rows * ldb
    slot = ((max(a_sz, b_sz) + 63) // 64 + 2) * 64
    pool = np.full(slot * 2 * batch + 64, W.BF16_NAN, np.uint16)
    order = rng.permutation(2 * batch)
    jitter = rng.integers(1, 8, size=2 * batch) | 1            # odd: not even 4-byte aligned
    A_off = order[:batch].astype(np.int64) * slot + 32 + jitter[:batch]
    B_off = order[batch:].astype(np.int64) * slot + 32 + jitter[batch:]
    for i in range(batch):
        a = np.full((a_rows, lda), W.BF16_NAN, np.uint16)
        b = np.full((b_rows, ldb), W.BF16_NAN, np.uint16)
        a[:, :lda - 8] = W.normal_bf16(67, i, (a_rows, lda - 8))
        b[:, :ldb - 8] = W.normal_bf16(67, 100 + i, (b_rows, ldb - 8))
        pool[A_off[i]:A_off[i] + a_sz] = a.ravel()
        pool[B_off[i]:B_off[i] + b_sz] = b.ravel()
    C0 = W.normal_f32(67, 999, (M, N))
    case = W.BrgemmCase(f"brgemm_oddoff_{M}x{N}x{K}x{batch}_t{tA}{tB}", M, N, K, batch, tA, tB, 1.0,
                        pool, A_off, B_off, lda, ldb, C0)
    ref = H.oracle_brgemm_case(oracle, case)
    ws = B.gemm_workspace_bytes(1, M, N, K, batch)
    ran = []
    for v, name in enumerate(B.variants()):
        for split in (1, 2):
            say(f"{case.name} variant={name} split={split}")
            try:
                out = H.run_brgemm_case(case, workspace_bytes=ws, force=(v, split))
            except B.BrgemmError as e:
                assert e.code == B.INVALID_ARG          # variant does not take this dtype / layout
                continue
            assert np.isfinite(out).all(), (name, split)
            assert H.rel_fro(out, ref) <= H.TOL_BF16_F32OUT, (name, split)
            ran.append(name)
    assert any("stream" in n for n in ran) and any("pingpong" in n for n in ran) and "bf16_128x128x64" in ran


def test_fused_bias_relu(oracle):
    M, N, K = 200, 328, 264
    for dtype, c_f32, tB in [("bf16", False, 1), ("bf16", True, 0), ("f32", True, 0)]:
        A = W.normal_f32(67, 0, (M, K))
        Bm = W.normal_f32(67, 1, (N, K) if tB else (K, N))
        bias = W.normal_f32(67, 2, (N,))
        if dtype == "bf16":
            A, Bm = W.to_bf16_bits(A), W.to_bf16_bits(Bm)
        case = W.GemmCase(f"bias_relu_{dtype}_cf32{c_f32}", dtype, M, N, K, 0, tB, 0.0, A, Bm, None, c_f32)
        say(case.name)
        out, _ = H.run_gemm_case(case, bias=bias, relu=True)
        ref = H.oracle_gemm_case(oracle, case, bias=bias, relu=True)
        assert (H.widen(out) >= 0).all()
        assert ((H.widen(out) == 0) == (ref <= 0)).mean() > 0.999
        assert H.rel_fro(H.widen(out), ref) <= _tol(case)
        out_b, _ = H.run_gemm_case(case, bias=bias, relu=False)
        ref_b = H.oracle_gemm_case(oracle, case, bias=bias, relu=False)
        assert H.rel_fro(H.widen(out_b), ref_b) <= _tol(case)


@pytest.mark.parametrize("dtype,c_f32", [("bf16", False), ("bf16", True), ("f32", True)])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0)])
def test_fused_epilogue_every_variant(oracle, dtype, c_f32, tA, tB):
    """beta != 0, bias and ReLU (Section 6: the measured kernel is BRGEMM + bias + ReLU)
    through the epilogue of every kernel variant that takes an aligned problem, with and
    without a reduction split; the bias starts one element into its allocation."""
    M, N, K = 512, 768, 512
    Al = W.normal_f32(74, 0, (M, K))
    Bl = W.normal_f32(74, 1, (K, N))
    As = np.ascontiguousarray(Al.T if tA else Al)
    Bs = np.ascontiguousarray(Bl.T if tB else Bl)
    C0 = W.normal_f32(74, 2, (M, N), sigma=8.0)
    bias = W.normal_f32(74, 3, (N,), sigma=8.0)
    if dtype == "bf16":
        As, Bs = W.to_bf16_bits(As), W.to_bf16_bits(Bs)
    if not c_f32:
        C0 = W.to_bf16_bits(C0)
    case = W.GemmCase(f"epilogue_{dtype}_cf32{c_f32}_t{tA}{tB}", dtype, M, N, K, tA, tB, 0.75, As, Bs, C0, c_f32)
    ref = H.oracle_gemm_case(oracle, case, bias=bias, relu=True)
    ref_b = H.oracle_gemm_case(oracle, case, bias=bias, relu=False)
    ws = B.gemm_workspace_bytes(1, M, N, K)
    ran = []
    for v, name in enumerate(B.variants()):
        for split in (1, 2):
            for shift in (0, 1):
                say(f"{case.name} variant={name} split={split} bias_shift={shift}")
                try:
                    out, _ = H.run_gemm_case(case, workspace_bytes=ws, force=(v, split), bias=bias, relu=True,
                                             bias_shift=shift)
                except B.BrgemmError as e:
                    assert e.code == B.INVALID_ARG          # variant does not take this dtype / layout
                    continue
                got = H.widen(out)
                assert (got >= 0).all(), (name, split)
                assert ((got == 0) == (ref <= 0)).mean() > 0.999, (name, split)
                assert H.rel_fro(got, ref) <= _tol(case), (name, split, shift)
                ran.append(name)
            try:
                out_b, _ = H.run_gemm_case(case, workspace_bytes=ws, force=(v, split), bias=bias, relu=False)
            except B.BrgemmError:
                continue
            assert H.rel_fro(H.widen(out_b), ref_b) <= _tol(case), (name, split)
    if dtype == "bf16":
        want = {"bf16_pingpong_256x256x64", "bf16_128x128x64", "bf16_stream_128x128x64", "generic_64x64x16_f32mfma"}
        if tA == 0:
            want |= {"bf16_stream_32x128x64", "bf16_stream_64x128x64"}
    else:
        want = {"f32_128x128x32", "generic_64x64x16_f32mfma"}
    assert want <= set(ran), set(ran)


def test_mlp_up_4096_bias_relu(oracle):
    """The paper's benchmark kernel at the up-projection shape: GEMM + bias + ReLU, bf16
    out, NT, automatic plan (the 256 x 256 kernel's staged epilogue); sampled complete rows."""
    case = W.config4_mlp(4096, "up")
    bias = W.normal_f32(75, 3, (case.N,), sigma=2.0)
    say(case.name + " + bias + relu")
    out, _ = H.run_gemm_case(case, workspace_bytes=1 << 28, bias=bias, relu=True, bias_shift=3)
    assert B.gemm_variant_name(B.gemm_last_variant()) == "bf16_pingpong_256x256x64"
    rows = H.sample_rows(case.M, 64)
    ref = H.oracle_gemm_case(oracle, case, rows=rows, bias=bias, relu=True)
    got = H.widen(out[rows])
    assert (H.widen(out) >= 0).all()
    assert ((got == 0) == (ref <= 0)).mean() > 0.999
    err = H.rel_fro(got, ref)
    say(f"   rel_fro={err:.3e}")
    assert err <= H.TOL_BF16


def test_every_variant_on_an_aligned_problem(oracle):
    """Each kernel variant that accepts the problem, forced in turn, with and without a split."""
    M, N, K = 512, 768, 512
    for dtype in ("bf16", "f32"):
        for tA, tB in [(0, 0), (0, 1), (1, 0), (1, 1)]:
            Al = W.normal_f32(68, 0, (M, K))
            Bl = W.normal_f32(68, 1, (K, N))
            As = np.ascontiguousarray(Al.T if tA else Al)
            Bs = np.ascontiguousarray(Bl.T if tB else Bl)
            if dtype == "bf16":
                As, Bs = W.to_bf16_bits(As), W.to_bf16_bits(Bs)
            case = W.GemmCase(f"variants_{dtype}_t{tA}{tB}", dtype, M, N, K, tA, tB, 0.0, As, Bs, None, True)
            ref = H.oracle_gemm_case(oracle, case)
            ws = B.gemm_workspace_bytes(1, M, N, K)
            for v, name in enumerate(B.variants()):
                for split in (1, 2):
                    say(f"{case.name} variant={name} split={split}")
                    try:
                        out, _ = H.run_gemm_case(case, workspace_bytes=ws, force=(v, split))
                    except B.BrgemmError as e:
                        assert e.code == B.INVALID_ARG      # variant does not take this dtype / layout
                        continue
                    assert H.rel_fro(H.widen(out), ref) <= 1e-5, (name, split)


@pytest.mark.gpu
def test_mfma_probe_counts_what_it_claims():
    """The register-only issue loop really executes iters x 8 matrix instructions per
    wave (x 32 for the 16x16 forms): with all-ones operands every accumulator element
    grows by the reduction depth (16 or 32 for bf16, 2 for fp32, 64 for int8, 128 for
    FP8) per instruction."""
    iters, blocks = 37, 5
    sink = torch.empty(blocks * 512, dtype=torch.float32, device="cuda")
    ones_h = torch.ones(6 * 64 * 8, device="cuda").to(torch.bfloat16)
    fl = B.gemm_mfma_probe(B.DTYPE_BF16, ones_h, iters, blocks, sink)
    assert fl == 2.0 * 32 * 32 * 16 * 8 * iters * 8 * blocks
    assert (sink.cpu().numpy() == 8 * 16 * iters * 16).all()
    # the 16x16x32 form (the 256 x 256 and streaming kernels' instruction): 32 per iteration
    ones_w = torch.ones(12 * 64 * 8, device="cuda").to(torch.bfloat16)
    fl = B.gemm_mfma_probe(B.PROBE_BF16_16X16X32, ones_w, iters, blocks, sink)
    assert fl == 2.0 * 16 * 16 * 32 * 32 * iters * 8 * blocks
    assert (sink.cpu().numpy() == 32 * 4 * iters * 32).all()
    ones_f = torch.ones(6 * 64, device="cuda")
    fl = B.gemm_mfma_probe(B.DTYPE_F32, ones_f, iters, blocks, sink)
    assert fl == 2.0 * 32 * 32 * 2 * 8 * iters * 8 * blocks
    assert (sink.cpu().numpy() == 8 * 16 * iters * 2).all()
    # one-byte operands: 32 instructions of 16x16 per iteration, 4 accumulator elements per lane
    ones_b = torch.ones(12 * 64 * 16, device="cuda", dtype=torch.int8)
    fl = B.gemm_mfma_probe(B.PROBE_S8, ones_b, iters, blocks, sink)
    assert fl == 2.0 * 16 * 16 * 64 * 32 * iters * 8 * blocks
    assert (sink.cpu().numpy() == 32 * 4 * iters * 64).all()
    ones_q = torch.full((12 * 64 * 32,), 0x38, device="cuda", dtype=torch.uint8)     # E4M3 1.0
    fl = B.gemm_mfma_probe(B.PROBE_F8, ones_q, iters, blocks, sink)
    assert fl == 2.0 * 16 * 16 * 128 * 32 * iters * 8 * blocks
    assert (sink.cpu().numpy() == 32 * 4 * iters * 128).all()


@pytest.mark.gpu
@pytest.mark.parametrize("tB", [0, 1])
@pytest.mark.parametrize("M,N,K", [(16, 200, 1024), (100, 392, 640), (33, 128, 64), (128, 264, 2048), (1, 8, 192)])
def test_stream_variants_ragged_edges_and_splits(oracle, M, N, K, tB):
    """The skinny-M streaming kernels, each forced in turn, on shapes whose M and N end
    inside a tile, with padded leading dimensions (NaN in the padding), beta != 0, a
    ring longer and shorter than the k-block count, and with and without a split."""
    pad = 8
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((M, K + pad), np.nan, np.float32)
    Bm = np.full((rb, cb + pad), np.nan, np.float32)
    A[:, :K] = W.normal_f32(71, 0, (M, K))
    Bm[:, :cb] = W.normal_f32(71, 1, (rb, cb))
    # fp32 C: the comparison then sees the kernel's own error only (a bf16 C of a few
    # elements can exceed the bf16 tolerance by rounding alone); bf16 C is covered by
    # the MLP-shape tests, which take these kernels automatically.
    C0 = W.normal_f32(71, 2, (M, N))
    case = W.GemmCase(f"stream_{M}x{N}x{K}_t0{tB}", "bf16", M, N, K, 0, tB, 0.5,
                      W.to_bf16_bits(A), W.to_bf16_bits(Bm), C0, True)
    ref = H.oracle_gemm_case(oracle, case)
    names = B.variants()
    ws = B.gemm_workspace_bytes(1, M, N, K)
    for name in ("bf16_stream_32x128x64", "bf16_stream_64x128x64", "bf16_stream_128x128x64"):
        for split in (1, 3):
            say(f"{case.name} variant={name} split={split}")
            out, _ = H.run_gemm_case(case, ldc=N + pad, workspace_bytes=ws, force=(names.index(name), split))
            assert np.isfinite(H.widen(out)).all(), "padding (NaN) leaked into the result"
            assert H.rel_fro(H.widen(out), ref) <= H.TOL_BF16_F32OUT, (name, split)


@pytest.mark.gpu
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_pingpong_and_f32_edge_tiles_with_skipped_wave_loads(oracle, tA, tB):
    """Tiles that overhang the matrix so far that whole 8-row wave-loads have no live
    lane: the kernels that count outstanding loads must not count those."""
    M, N, K = 256 + 104, 512 + 8, 1024
    names = B.variants()
    for dtype, vname in (("bf16", "bf16_pingpong_256x256x64"), ("f32", "f32_128x128x32")):
        Al = W.normal_f32(72, 0, (M, K))
        Bl = W.normal_f32(72, 1, (K, N))
        As = np.ascontiguousarray(Al.T if tA else Al)
        Bs = np.ascontiguousarray(Bl.T if tB else Bl)
        if dtype == "bf16":
            As, Bs = W.to_bf16_bits(As), W.to_bf16_bits(Bs)
        case = W.GemmCase(f"edge_{dtype}_t{tA}{tB}", dtype, M, N, K, tA, tB, 0.0, As, Bs, None, True)
        say(case.name)
        ref = H.oracle_gemm_case(oracle, case)
        out, _ = H.run_gemm_case(case, force=(names.index(vname), 1))
        assert H.rel_fro(H.widen(out), ref) <= 1e-5, vname


@pytest.mark.gpu
def test_seeded_random_shape_sweep(oracle):
    """120 seeded random problems (all dtypes, transposes, beta, padded leading dimensions,
    sizes chosen around the tile edges 16 / 32 / 64 / 128 / 256 and k-blocks 32 / 64) through
    the automatic plan, each against the oracle."""
    rng = np.random.default_rng(20251113)
    edges = [1, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 136, 200, 255, 256, 257, 264, 384, 520]
    kvals = [1, 8, 31, 32, 33, 64, 96, 128, 192, 320, 448, 640, 1088]
    seen = set()
    for it in range(120):
        dtype = ["bf16", "f32", "bf16"][it % 3]
        tA, tB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        M, N, K = int(rng.choice(edges)), int(rng.choice(edges)), int(rng.choice(kvals))
        if rng.random() < 0.5:          # keep the tuned kernels in play half of the time
            M, N, K = (M + 7) // 8 * 8, (N + 7) // 8 * 8, (K + 63) // 64 * 64
        pad = int(rng.choice([0, 0, 8, 3]))
        beta = float(rng.choice([0.0, 1.0, -0.5]))
        c_f32 = dtype == "f32" or bool(rng.integers(0, 2))
        ra, ca = (K, M) if tA else (M, K)
        rb, cb = (N, K) if tB else (K, N)
        A = np.full((ra, ca + pad), np.nan, np.float32)
        Bm = np.full((rb, cb + pad), np.nan, np.float32)
        A[:, :ca] = W.normal_f32(200 + it, 0, (ra, ca))
        Bm[:, :cb] = W.normal_f32(200 + it, 1, (rb, cb))
        C0 = W.normal_f32(200 + it, 2, (M, N)) if beta != 0.0 else None
        if dtype == "bf16":
            A, Bm = W.to_bf16_bits(A), W.to_bf16_bits(Bm)
        if C0 is not None and not c_f32:
            C0 = W.to_bf16_bits(C0)
        case = W.GemmCase(f"sweep{it}_{dtype}_{M}x{N}x{K}_t{tA}{tB}_pad{pad}_b{beta}", dtype, M, N, K, tA, tB, beta,
                          A, Bm, C0, c_f32)
        say(case.name)
        out, _ = H.run_gemm_case(case, ldc=N + pad, workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
        seen.add(B.gemm_variant_name(B.gemm_last_variant()))
        ref = H.oracle_gemm_case(oracle, case)
        got = H.widen(out)
        assert np.isfinite(got).all(), case.name
        if c_f32:
            assert H.rel_fro(got, ref) <= 1e-5, (case.name, B.gemm_variant_name(B.gemm_last_variant()))
        else:
            # every element within one bf16 rounding of an fp32 evaluation; the Frobenius limit
            # (an RMS figure) only where there are enough elements for it to mean something
            H.check_bf16_case_elementwise(oracle, case, out, ref)
            if M * N >= 4096:
                assert H.rel_fro(got, ref) <= H.TOL_BF16, (case.name, B.gemm_variant_name(B.gemm_last_variant()))
    assert len(seen) >= 5, seen


@pytest.mark.gpu
def test_operand_larger_than_4_gib(oracle):
    """A spans more than 2^32 bytes (2,097,408 x 1024 bf16): rows on both sides of the 4 GiB
    line are checked, so every row offset has to be formed in 64 bits.  A is generated on the
    device (input generation only); the sampled rows are copied back for the oracle."""
    M, N, K = (1 << 21) + 256, 128, 1024
    g = torch.Generator(device="cuda").manual_seed(20251113)
    A = torch.randn((M, K), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    assert A.numel() * 2 > (1 << 32)
    Bm = W.to_bf16_bits(W.normal_f32(73, 1, (N, K)))                 # stored N x K ("NT")
    dB = H.dev(Bm)
    dC = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
    B.gemm_bf16(0, 1, M, N, K, A, K, dB, K, 0.0, dC, N, 1)
    torch.cuda.synchronize()
    used = B.gemm_variant_name(B.gemm_last_variant())
    say(f"4 GiB operand -> {used}")
    rows = [0, 1, 255, 256, M // 2 - 1, M // 2, (1 << 21) - 1, 1 << 21, (1 << 21) + 1, M - 257, M - 256, M - 1]
    idx = torch.tensor(rows, device="cuda")
    A_rows = A[idx].cpu().view(torch.int16).numpy().view(np.uint16)
    got = dC[idx].cpu().numpy().astype(np.float64)
    ref = oracle.gemm_ref(A_rows, K, Bm, K, len(rows), N, K, transB=1)
    assert H.rel_fro(got, ref) <= 1e-5
    assert torch.isfinite(dC).all().item(), "some row of C was never written"
