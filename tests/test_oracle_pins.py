"""Pins of the CPU oracle against things other than itself (CPU only).

Each test checks oracle/brgemm_oracle.c against something the mathematics or
the paper fixes: literal hand-computed products, exact integer arithmetic,
identity / permutation matrices, closed forms, algebraic invariants, the
shapes used in the paper's listings, and the bf16 rounding rule.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2511_13764_amd import workloads as W

F32, BF16 = 0, 1


def bf16_bits(x):
    return W.to_bf16_bits(np.asarray(x, dtype=np.float32))


# ---------------------------------------------------------------- p1: literal / brute force

def test_literal_2x2(oracle):
    # [[1,2],[3,4]] x [[5,6],[7,8]] = [[19,22],[43,50]]  (worked by hand)
    A = np.array([[1, 2], [3, 4]], dtype=np.float32)
    B = np.array([[5, 6], [7, 8]], dtype=np.float32)
    ref = oracle.gemm_ref(A, 2, B, 2, 2, 2, 2)
    assert ref.tolist() == [[19.0, 22.0], [43.0, 50.0]]


def test_literal_2x3x4_nonsquare(oracle):
    # A (2x4) = [[1,0,2,-1],[3,1,0,2]];  B (4x3) = [[1,2,0],[0,1,1],[4,0,-2],[1,1,1]]
    # row0: [1+8-1, 2-1, -4-1] = [8,1,-5];  row1: [3+2, 6+1+2, 1+2] = [5,9,3]
    A = np.array([[1, 0, 2, -1], [3, 1, 0, 2]], dtype=np.float32)
    B = np.array([[1, 2, 0], [0, 1, 1], [4, 0, -2], [1, 1, 1]], dtype=np.float32)
    ref = oracle.gemm_ref(A, 4, B, 3, 2, 3, 4)
    assert ref.tolist() == [[8.0, 1.0, -5.0], [5.0, 9.0, 3.0]]
    # same logical operands, stored transposed
    At, Bt = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
    assert oracle.gemm_ref(At, 2, B, 3, 2, 3, 4, transA=1).tolist() == ref.tolist()
    assert oracle.gemm_ref(A, 4, Bt, 4, 2, 3, 4, transB=1).tolist() == ref.tolist()
    assert oracle.gemm_ref(At, 2, Bt, 4, 2, 3, 4, transA=1, transB=1).tolist() == ref.tolist()


def test_literal_beta_and_batch(oracle):
    # C0 = [[10,20]], beta = 0.5, A_0 = [[1,2]], B_0 = [[1,0],[0,1]], A_1 = [[3,4]], B_1 = [[2,2],[1,1]]
    # sum = [1,2] + [6+4, 6+4] = [11,12];  + 0.5*C0 = [16, 22]
    pool = np.array([1, 2, 3, 4], dtype=np.float32)
    bpool = np.array([1, 0, 0, 1, 2, 2, 1, 1], dtype=np.float32)
    C0 = np.array([[10, 20]], dtype=np.float32)
    ref = oracle.brgemm_ref(pool, [0, 2], 2, bpool, [0, 4], 2, 1, 2, 2, beta=0.5, C0=C0)
    assert ref.tolist() == [[16.0, 22.0]]


def _brute(A, B, M, N, K, tA, tB, lda, ldb, a_off, b_off, beta, C0, ldc0, bias=None, relu=False):
    """Exact rational arithmetic on flat Python lists (independent of the C loops)."""
    out = [[Fraction(0)] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            s = Fraction(0)
            for ao, bo in zip(a_off, b_off):
                for k in range(K):
                    a = A[ao + (k * lda + m if tA else m * lda + k)]
                    b = B[bo + (n * ldb + k if tB else k * ldb + n)]
                    s += Fraction(float(a)) * Fraction(float(b))
            if beta != 0:
                s += Fraction(float(np.float32(beta))) * Fraction(float(C0[m * ldc0 + n]))
            if bias is not None:
                s += Fraction(float(bias[n]))
            if relu and s < 0:
                s = Fraction(0)
            out[m][n] = s
    return out


@pytest.mark.parametrize("M,N,K,batch", [(1, 1, 1, 1), (2, 3, 4, 1), (3, 5, 7, 2), (4, 2, 3, 3)])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_bruteforce_tiny_fractions(oracle, M, N, K, batch, tA, tB):
    rng = np.random.default_rng(7 + M * 100 + N * 10 + K + 2 * tA + tB)
    lda = (M if tA else K) + 2
    ldb = (K if tB else N) + 3
    ldc0 = N + 1
    a_tile = ((K - 1) * lda + M) if tA else ((M - 1) * lda + K)
    b_tile = ((N - 1) * ldb + K) if tB else ((K - 1) * ldb + N)
    a_off = [5 + i * (a_tile + 3) for i in range(batch)][::-1]      # scattered, reversed order
    b_off = [2 + i * (b_tile + 7) for i in range(batch)]
    A = rng.uniform(-1, 1, size=a_off[0] + a_tile + 4).astype(np.float32)
    B = rng.uniform(-1, 1, size=b_off[-1] + b_tile + 4).astype(np.float32)
    C0 = rng.uniform(-1, 1, size=M * ldc0).astype(np.float32)
    bias = rng.uniform(-1, 1, size=N).astype(np.float32)
    for beta, use_bias, relu in [(0.0, False, False), (0.75, False, False), (-1.5, True, True)]:
        ref = oracle.brgemm_ref(A, a_off, lda, B, b_off, ldb, M, N, K, transA=tA, transB=tB,
                                beta=beta, C0=C0, ldc0=ldc0,
                                bias=bias if use_bias else None, relu=relu)
        exact = _brute(A, B, M, N, K, tA, tB, lda, ldb, a_off, b_off, beta, C0, ldc0,
                       bias if use_bias else None, relu)
        for m in range(M):
            for n in range(N):
                e = float(exact[m][n])
                assert abs(ref[m, n] - e) <= 1e-15 * max(1.0, abs(e)) * (K * batch + 2)


# ---------------------------------------------------------------- p2: small integers, exact

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K,tA,tB", [(33, 65, 129, 0, 0), (64, 48, 200, 0, 1),
                                         (17, 31, 257, 1, 0), (40, 24, 96, 1, 1)])
def test_small_integer_exact(oracle, dtype, M, N, K, tA, tB):
    Al = W.small_int_matrix(1000 + M, (M, K))
    Bl = W.small_int_matrix(2000 + N, (K, N))
    expect = Al.astype(np.int64) @ Bl.astype(np.int64)
    As = np.ascontiguousarray(Al.T if tA else Al)
    Bs = np.ascontiguousarray(Bl.T if tB else Bl)
    if dtype == "bf16":
        As, Bs = bf16_bits(As), bf16_bits(Bs)
    ref = oracle.gemm_ref(As, As.shape[1], Bs, Bs.shape[1], M, N, K, transA=tA, transB=tB)
    assert np.array_equal(ref, expect.astype(np.float64))


# ---------------------------------------------------------------- p3: identity / permutation

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identity_and_permutation(oracle, dtype):
    n, m = 37, 21
    X = W.normal_f32(90, 0, (m, n))
    Xs = bf16_bits(X) if dtype == "bf16" else X
    Xv = oracle.bf16_to_f64(Xs) if dtype == "bf16" else X.astype(np.float64)
    eye = np.eye(n, dtype=np.float32)
    perm = np.random.default_rng(3).permutation(n)
    P = eye[perm]                                   # (P @ Y)[i] = Y[perm[i]];  (X @ P)[:, j] = X[:, inv[j]]
    conv = bf16_bits if dtype == "bf16" else (lambda a: a)
    # X * I = X
    assert np.array_equal(oracle.gemm_ref(Xs, n, conv(eye), n, m, n, n), Xv)
    # I * X^T-stored ... left identity on the transposed operand
    eye_m = np.eye(m, dtype=np.float32)
    assert np.array_equal(oracle.gemm_ref(conv(eye_m), m, Xs, n, m, n, m), Xv)
    # X * P permutes columns: column j of the result is column k of X where P[k, j] = 1
    got = oracle.gemm_ref(Xs, n, conv(P), n, m, n, n)
    inv = np.argsort(perm)
    assert np.array_equal(got, Xv[:, inv])
    # P_m * X permutes rows
    pm = np.random.default_rng(4).permutation(m)
    Pm = eye_m[pm]
    assert np.array_equal(oracle.gemm_ref(conv(Pm), m, Xs, n, m, n, m), Xv[pm])


# ---------------------------------------------------------------- p4: closed forms

def test_closed_forms(oracle):
    M, N, K = 19, 23, 301
    ones_a, ones_b = np.ones((M, K), np.float32), np.ones((K, N), np.float32)
    assert np.array_equal(oracle.gemm_ref(ones_a, K, ones_b, N, M, N, K), np.full((M, N), float(K)))
    ramp = np.repeat(np.arange(M, dtype=np.float32)[:, None], K, axis=1)
    assert np.array_equal(oracle.gemm_ref(ramp, K, ones_b, N, M, N, K),
                          np.repeat((np.arange(M) * K).astype(np.float64)[:, None], N, axis=1))
    # rank-1 outer product, K = 1
    u = W.uniform_f32(91, 0, (M, 1))
    v = W.uniform_f32(91, 1, (1, N))
    assert np.array_equal(oracle.gemm_ref(u, 1, v, N, M, N, 1),
                          u.astype(np.float64) * v.astype(np.float64))
    # alternating signs cancel: sum_k (-1)^k = 0 for even K
    alt = np.tile(np.array([1, -1], np.float32), (M, 150))
    assert np.array_equal(oracle.gemm_ref(alt, 300, np.ones((300, N), np.float32), N, M, N, 300),
                          np.zeros((M, N)))


# ---------------------------------------------------------------- p5: associativity

def test_associativity(oracle):
    M, K, N = 96, 160, 72
    A = W.uniform_f32(92, 0, (M, K))
    B = W.uniform_f32(92, 1, (K, N))
    x = W.uniform_f32(92, 2, (N, 1))
    AB = oracle.gemm_ref(A, K, B, N, M, N, K)                       # fp64
    Bx = oracle.gemm_ref(B, N, x, 1, K, 1, N)
    # second products in numpy fp64 (the oracle only takes fp32 / bf16 inputs)
    left = AB @ x.astype(np.float64)
    right = A.astype(np.float64) @ Bx
    assert np.linalg.norm(left - right) <= 1e-12 * np.sqrt(K) * np.linalg.norm(left)


# ---------------------------------------------------------------- p6: transposes and leading dimensions

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_transpose_flags_and_padded_ld(oracle, dtype):
    M, N, K = 29, 43, 57
    Al = W.normal_f32(93, 0, (M, K))
    Bl = W.normal_f32(93, 1, (K, N))
    if dtype == "bf16":
        Al = oracle.bf16_to_f64(bf16_bits(Al)).astype(np.float32)
        Bl = oracle.bf16_to_f64(bf16_bits(Bl)).astype(np.float32)
    results = []
    for tA in (0, 1):
        for tB in (0, 1):
            for pad in (0, 5):
                As = Al.T if tA else Al
                Bs = Bl.T if tB else Bl
                Ap = np.full((As.shape[0], As.shape[1] + pad), np.nan, np.float32)
                Bp = np.full((Bs.shape[0], Bs.shape[1] + pad), np.nan, np.float32)
                Ap[:, :As.shape[1]] = As
                Bp[:, :Bs.shape[1]] = Bs
                if dtype == "bf16":
                    Ap, Bp = bf16_bits(Ap), bf16_bits(Bp)
                r = oracle.gemm_ref(Ap, Ap.shape[1], Bp, Bp.shape[1], M, N, K, transA=tA, transB=tB)
                assert np.isfinite(r).all()
                results.append(r)
    expect = Al.astype(np.float64) @ Bl.astype(np.float64)
    for r in results:
        assert np.allclose(r, expect, rtol=0, atol=1e-12 * K)
    # (A B)^T = B^T A^T : swap operands and flags, result is the transpose
    At, Bt = np.ascontiguousarray(Al.T), np.ascontiguousarray(Bl.T)
    if dtype == "bf16":
        At, Bt = bf16_bits(At), bf16_bits(Bt)
    rT = oracle.gemm_ref(Bt, K, At, M, N, M, K)
    assert np.allclose(rT, expect.T, rtol=0, atol=1e-12 * K)


# ---------------------------------------------------------------- p7: batch-reduce == GEMM over concatenated K

def test_brgemm_equals_concatenated_gemm(oracle):
    M, N, K, batch = 24, 40, 16, 5
    tiles_a = [W.normal_bf16(94, i, (M, K)) for i in range(batch)]
    tiles_b = [W.normal_bf16(94, 50 + i, (K, N)) for i in range(batch)]
    gap = 64
    pool = np.full(batch * (M * K + K * N + 2 * gap) + gap, W.BF16_NAN, np.uint16)
    a_off, b_off, pos = [], [], gap
    for i in range(batch):
        a_off.append(pos)
        pool[pos:pos + M * K] = tiles_a[i].ravel()
        pos += M * K + gap
        b_off.append(pos)
        pool[pos:pos + K * N] = tiles_b[i].ravel()
        pos += K * N + gap
    br = oracle.brgemm_ref(pool, a_off, K, pool, b_off, N, M, N, K)
    assert np.isfinite(br).all()
    Acat = np.concatenate(tiles_a, axis=1)            # M x (K*batch)
    Bcat = np.concatenate(tiles_b, axis=0)            # (K*batch) x N
    g = oracle.gemm_ref(Acat, K * batch, Bcat, N, M, N, K * batch)
    assert np.linalg.norm(br - g) <= 1e-13 * np.linalg.norm(g)
    # batch order does not matter beyond fp64 rounding
    order = [3, 0, 4, 2, 1]
    br2 = oracle.brgemm_ref(pool, [a_off[i] for i in order], K, pool, [b_off[i] for i in order], N, M, N, K)
    assert np.linalg.norm(br - br2) <= 1e-13 * np.linalg.norm(g)
    # mismatched pairing must differ (the pairing of A_i with B_i is part of the definition)
    br3 = oracle.brgemm_ref(pool, a_off, K, pool, b_off[1:] + b_off[:1], N, M, N, K)
    assert np.linalg.norm(br - br3) > 1e-3 * np.linalg.norm(g)
    # batch == 1 is plain GEMM
    one = oracle.brgemm_ref(pool, a_off[:1], K, pool, b_off[:1], N, M, N, K)
    assert np.array_equal(one, oracle.gemm_ref(tiles_a[0], K, tiles_b[0], N, M, N, K))
    # batch == 0 leaves beta*C0
    C0 = W.uniform_f32(94, 99, (M, N))
    zero = oracle.brgemm_ref(pool, [], K, pool, [], N, M, N, K, beta=2.0, C0=C0)
    assert np.array_equal(zero, 2.0 * C0.astype(np.float64))


# ---------------------------------------------------------------- p8: beta

def test_beta_linearity_and_beta_zero_ignores_c(oracle):
    M, N, K = 31, 45, 77
    A = W.uniform_f32(95, 0, (M, K))
    B = W.uniform_f32(95, 1, (K, N))
    C0 = W.uniform_f32(95, 2, (M, N + 3))
    base = oracle.gemm_ref(A, K, B, N, M, N, K)
    for beta in (1.0, 0.5, -2.25, 1e-3):
        r = oracle.gemm_ref(A, K, B, N, M, N, K, beta=beta, C0=C0, ldc0=N + 3)
        want = float(np.float32(beta)) * C0[:, :N].astype(np.float64)
        assert np.allclose(r - base, want, rtol=1e-14, atol=1e-15)
    poison = np.full((M, N), np.nan, np.float32)
    r0 = oracle.gemm_ref(A, K, B, N, M, N, K, beta=0.0, C0=poison)
    assert np.array_equal(r0, base)
    # bf16 old C is widened exactly (Section 4.3)
    Cb = bf16_bits(C0[:, :N].copy())
    r = oracle.gemm_ref(A, K, B, N, M, N, K, beta=1.0, C0=Cb, ldc0=N)
    assert np.allclose(r - base, oracle.bf16_to_f64(Cb), rtol=1e-14, atol=1e-15)


def test_bias_relu_epilogue(oracle):
    # Section 6: the measured kernel adds a bias row and applies ReLU before the store.
    A = np.array([[1, -2], [-3, 1]], dtype=np.float32)
    B = np.array([[1, 1], [1, 2]], dtype=np.float32)       # A B = [[-1,-3],[-2,-1]]
    bias = np.array([2.0, 2.0], dtype=np.float32)          # + bias = [[1,-1],[0,1]]
    r = oracle.gemm_ref(A, 2, B, 2, 2, 2, 2, bias=bias, relu=True)
    assert r.tolist() == [[1.0, 0.0], [0.0, 1.0]]
    r = oracle.gemm_ref(A, 2, B, 2, 2, 2, 2, bias=bias, relu=False)
    assert r.tolist() == [[1.0, -1.0], [0.0, 1.0]]


# ---------------------------------------------------------------- p9: shapes used in the paper's listings

@pytest.mark.parametrize("name,dtype,batch,M,K,N", [
    ("listing1_vnni_example", "bf16", 4, 32, 32, 192),     # Section 2.2 listing: 4 x [32x(16*2)] . [(16*2)x192]
    ("appendix_fp32", "f32", 2, 4, 32, 96),                # appendix, fp32 input kernel
    ("appendix_bf16", "bf16", 2, 64, 64, 64),              # appendix, bf16 input kernels
    ("section3_12x24", "f32", 1, 12, 8, 24),               # Section 3.1's 12 x 24 register-tiling case
])
def test_paper_listing_shapes_exact(oracle, name, dtype, batch, M, K, N):
    As = [W.small_int_matrix(300 + i, (M, K)) for i in range(batch)]
    Bs = [W.small_int_matrix(400 + i, (K, N)) for i in range(batch)]
    expect = sum(a.astype(np.int64) @ b.astype(np.int64) for a, b in zip(As, Bs))
    C0 = W.small_int_matrix(500, (M, N))
    expect = expect + C0.astype(np.int64)                  # the listings accumulate into C (beta = 1)
    A = np.stack(As)
    B = np.stack(Bs)
    if dtype == "bf16":
        A, B = bf16_bits(A), bf16_bits(B)
    a_off = [i * M * K for i in range(batch)]
    b_off = [i * K * N for i in range(batch)]
    r = oracle.brgemm_ref(A, a_off, K, B, b_off, N, M, N, K, beta=1.0, C0=C0)
    assert np.array_equal(r, expect.astype(np.float64))


# ---------------------------------------------------------------- p10: bf16 rounding helper

def test_bf16_rounding_bit_patterns(oracle):
    f = oracle.f64_to_bf16
    assert f(0.0) == 0x0000 and f(-0.0) == 0x8000
    assert f(1.0) == 0x3F80 and f(-2.0) == 0xC000
    assert f(1.0 + 2 ** -8) == 0x3F80            # tie, lower neighbour even -> down
    assert f(1.0 + 3 * 2 ** -8) == 0x3F82        # tie, upper neighbour even -> up
    assert f(1.0 + 2 ** -8 + 2 ** -30) == 0x3F81  # just above the tie -> up
    assert f(1.0 + 2 ** -8 - 2 ** -30) == 0x3F80  # just below the tie -> down
    assert f(2.0 - 2 ** -9) == 0x4000            # carry into the exponent
    assert f(float("inf")) == 0x7F80 and f(float("-inf")) == 0xFF80
    assert f(float("nan")) & 0x7FC0 == 0x7FC0
    big = (2.0 - 2.0 ** -7) * 2.0 ** 127          # largest finite bf16
    assert f(big) == 0x7F7F
    assert f((2.0 - 2.0 ** -8) * 2.0 ** 127) == 0x7F80       # the tie at the top goes to infinity
    assert f(np.nextafter((2.0 - 2.0 ** -8) * 2.0 ** 127, 0.0)) == 0x7F7F
    assert f(2.0 ** -133) == 0x0001                          # smallest subnormal
    assert f(2.0 ** -134) == 0x0000                          # tie to even (zero)
    assert f(3 * 2.0 ** -134) == 0x0002                      # tie to even (up)
    assert f(2.0 ** -126) == 0x0080                          # smallest normal


def test_bf16_rounding_matches_library_on_fp32(oracle):
    import torch
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 2 ** 32, size=1 << 18, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.round_to_out(x.astype(np.float64), BF16)
    assert np.array_equal(got, want)
    # and exact widening
    assert np.array_equal(oracle.bf16_to_f64(want),
                          torch.from_numpy(want.view(np.int16).copy()).view(torch.bfloat16).double().numpy())


def test_round_to_out_single_rounding(oracle):
    # A value that double rounding (fp64 -> fp32 -> bf16) gets wrong: just above a bf16 tie
    # by less than half an fp32 ulp.  One-step rounding must go up.
    v = 1.0 + 2 ** -8 + 2 ** -40
    assert oracle.f64_to_bf16(v) == 0x3F81
    assert oracle.round_to_out(np.array([v]), BF16)[0] == 0x3F81
    assert oracle.round_to_out(np.array([0.1]), F32)[0] == np.float32(0.1)


# ---------------------------------------------------------------- p11: full-size sanity against a library matmul

def test_statistical_against_library_matmul(oracle):
    case = W.config1_f32_256()
    ref = oracle.gemm_ref(case.A, case.lda, case.B, case.ldb, case.M, case.N, case.K)
    lib = case.A @ case.B                               # fp32 library routine
    err = np.linalg.norm(lib.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err < 5e-6
    lib64 = case.A.astype(np.float64) @ case.B.astype(np.float64)
    assert np.linalg.norm(lib64 - ref) / np.linalg.norm(ref) < 1e-14


def test_row_sampling_matches_full(oracle):
    M, N, K = 50, 30, 40
    A = W.normal_bf16(96, 0, (M, K))
    B = W.normal_bf16(96, 1, (N, K))
    full = oracle.gemm_ref(A, K, B, K, M, N, K, transB=1)
    rows = [49, 0, 17, 17, 3]
    part = oracle.gemm_ref(A, K, B, K, M, N, K, transB=1, rows=rows)
    assert np.array_equal(part, full[rows])
    with pytest.raises(ValueError):
        oracle.gemm_ref(A, K, B, K, M, N, K, transB=1, rows=[50])


def test_nan_row_propagates_only_to_its_row(oracle):
    M, N, K = 9, 11, 13
    A = W.uniform_f32(97, 0, (M, K))
    B = W.uniform_f32(97, 1, (K, N))
    A[4, 6] = np.nan
    r = oracle.gemm_ref(A, K, B, N, M, N, K)
    assert np.isnan(r[4]).all() and np.isfinite(np.delete(r, 4, axis=0)).all()


def test_empty_shapes(oracle):
    A = np.zeros((4, 0), np.float32)
    B = np.zeros((0, 5), np.float32)
    C0 = np.ones((4, 5), np.float32)
    assert np.array_equal(oracle.gemm_ref(A, 1, B, 5, 4, 5, 0, beta=3.0, C0=C0), 3.0 * np.ones((4, 5)))
    assert np.array_equal(oracle.gemm_ref(A, 1, B, 5, 4, 5, 0), np.zeros((4, 5)))
    assert oracle.gemm_ref(A, 1, B, 5, 0, 5, 0).shape == (0, 5)


# ---------------------------------------------------------------- VNNI packer (Section 2.2, Figure 1)

def _read_fig1():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fig1_vnni2_pack.txt")
    lines = [l.strip() for l in open(path) if l.strip() and not l.startswith("#")]
    assert lines[0].split()[0] == "flat"
    r, c = map(int, lines[0].split()[1:])
    flat = np.array([[int(x) for x in lines[1 + i].split()] for i in range(r)], dtype=np.uint16)
    assert flat.shape == (r, c)
    g, cc, v = map(int, lines[1 + r].split()[1:])
    packed = np.array([[[int(x) for x in pair.split(",")] for pair in lines[2 + r + i].split()] for i in range(g)],
                      dtype=np.uint16)
    assert packed.shape == (g, cc, v)
    return flat, packed


def test_pack_vnni_reproduces_figure_1(oracle):
    """The paper's worked example: a flat 4x4 matrix and its VNNI:2 packed form."""
    flat, packed = _read_fig1()
    got = oracle.pack_vnni(flat, 4, 4, 4, 2)
    assert got.shape == (2, 4, 2)
    assert (got == packed).all()
    # the same matrix handed over transposed (stored N x K) packs to the same image
    assert (oracle.pack_vnni(np.ascontiguousarray(flat.T), 4, 4, 4, 2, transB=1) == packed).all()


@pytest.mark.parametrize("v", [2, 4, 8])
@pytest.mark.parametrize("K,N", [(8, 5), (13, 7), (64, 33), (1, 1)])
def test_pack_vnni_against_reshape_and_inverse(oracle, v, K, N):
    """Where K is a multiple of v the packing is the textbook reshape/transposition
    (K/v, v, N) -> (K/v, N, v); in general unpacking gives B back and the rest is zero."""
    rng = np.random.default_rng(7 * v + K + N)
    Bm = rng.integers(1, 65535, size=(K, N + 3)).astype(np.uint16)      # padded leading dimension
    got = oracle.pack_vnni(Bm, N + 3, K, N, v)
    Kp = K + (-K) % v
    assert got.shape == (Kp // v, N, v)
    full = np.zeros((Kp, N), dtype=np.uint16)
    full[:K] = Bm[:, :N]
    assert (got == full.reshape(Kp // v, v, N).transpose(0, 2, 1)).all()
    # inverse: element (k, n) sits at [k // v, n, k % v]
    for k in range(K):
        for n in range(N):
            assert got[k // v, n, k % v] == Bm[k, n]
    # padded image: more k rows and a wider column pitch, all extra entries zero
    big = oracle.pack_vnni(Bm, N + 3, K, N, v, k_rows=Kp + 2 * v, n_pitch=N + 5)
    assert (big[:Kp // v, :N] == got).all()
    assert big[Kp // v:].sum() == 0 and big[:, N:].sum() == 0
    # transposed storage gives the same image
    BT = np.ascontiguousarray(Bm[:, :N].T)
    assert (oracle.pack_vnni(BT, K, K, N, v, transB=1) == got).all()


def test_packed_gemm_identity(oracle):
    """Contracting A against the unpacked image equals the plain product: the packed
    layout is a pure re-indexing (sum over g, j of A[m, 8g + j] * P[g, n, j])."""
    M, N, K, v = 5, 6, 24, 8
    A = W.small_int_matrix(50, (M, K))
    Bm = W.small_int_matrix(51, (K, N))
    P = oracle.pack_vnni(bf16_bits(Bm), N, K, N, v)
    Pv = oracle.bf16_to_f64(P)
    want = np.einsum("mgj,gnj->mn", A.astype(np.float64).reshape(M, K // v, v), Pv)
    ref = oracle.gemm_ref(bf16_bits(A), K, bf16_bits(Bm), N, M, N, K)
    assert (ref == want).all()
    assert (ref == (A.astype(np.int64) @ Bm.astype(np.int64))).all()


# ---------------------------------------------------------------- binary16 (Section 2.2 names FP16 next to BF16)

def test_f16_decoder_all_patterns_against_library(oracle):
    """Every one of the 65536 binary16 patterns decodes to what numpy's float16 says."""
    bits = np.arange(65536, dtype=np.uint16)
    lib = bits.view(np.float16).astype(np.float64)
    for b in list(range(0, 65536, 7)) + [0, 1, 0x03FF, 0x0400, 0x7BFF, 0x7C00, 0x8000, 0x8001, 0xFBFF, 0xFC00]:
        got = oracle.f16_to_f64(b)
        assert (np.isnan(got) and np.isnan(lib[b])) or got == lib[b], hex(b)
    # hand-picked values: smallest subnormal, largest subnormal, smallest normal, one, largest finite
    assert oracle.f16_to_f64(0x0001) == 2.0 ** -24
    assert oracle.f16_to_f64(0x03FF) == 1023 * 2.0 ** -24
    assert oracle.f16_to_f64(0x0400) == 2.0 ** -14
    assert oracle.f16_to_f64(0x3C00) == 1.0
    assert oracle.f16_to_f64(0x7BFF) == 65504.0
    assert oracle.f16_to_f64(0xC000) == -2.0


def test_f16_rounding_hand_picked_and_against_library(oracle):
    f = oracle.f64_to_f16
    assert f(0.0) == 0x0000 and f(-0.0) == 0x8000
    assert f(1.0) == 0x3C00
    assert f(1.0 + 2.0 ** -11) == 0x3C00            # tie: 1 is even
    assert f(1.0 + 3 * 2.0 ** -11) == 0x3C02        # tie: goes to the even neighbour above
    assert f(1.0 + 2.0 ** -11 + 2.0 ** -30) == 0x3C01
    assert f(2.0 - 2.0 ** -12) == 0x4000            # carry into the exponent
    assert f(65504.0) == 0x7BFF and f(65519.99) == 0x7BFF
    assert f(65520.0) == 0x7C00 and f(1e9) == 0x7C00 and f(-1e9) == 0xFC00
    assert f(2.0 ** -24) == 0x0001 and f(2.0 ** -25) == 0x0000      # tie to even (zero)
    assert f(3 * 2.0 ** -25) == 0x0002 and f(2.0 ** -14 - 2.0 ** -25) == 0x0400
    assert f(float("inf")) == 0x7C00 and (f(float("nan")) & 0x7FFF) > 0x7C00
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 5, 200000),
                        (rng.integers(0, 65536, 50000).astype(np.uint16).view(np.float16).astype(np.float64)
                         * (1 + rng.integers(-1, 2, 50000) * 2.0 ** -11))])
    with np.errstate(over="ignore", invalid="ignore"):
        lib = x.astype(np.float16).view(np.uint16)
    got = oracle.round_to_out(x, 2).view(np.uint16)
    nan = np.isnan(x)
    assert (got[~nan] == lib[~nan]).all()


def test_f16_gemm_small_integers_and_statistics(oracle):
    """binary16 operands: integer-valued matrices are exact against int64 arithmetic in every
    transpose; N(0,1) operands agree with a float64 library product of the widened inputs."""
    M, N, K = 17, 23, 40
    A = W.small_int_matrix(60, (M, K)).astype(np.float16)
    Bm = W.small_int_matrix(61, (K, N)).astype(np.float16)
    want = A.astype(np.int64) @ Bm.astype(np.int64)
    for tA in (0, 1):
        for tB in (0, 1):
            As = np.ascontiguousarray(A.T if tA else A)
            Bs = np.ascontiguousarray(Bm.T if tB else Bm)
            ref = oracle.gemm_ref(As, As.shape[1], Bs, Bs.shape[1], M, N, K, transA=tA, transB=tB)
            assert (ref == want).all(), (tA, tB)
    rng = np.random.default_rng(12)
    A = rng.standard_normal((64, 300)).astype(np.float16)
    Bm = rng.standard_normal((300, 48)).astype(np.float16)
    C0 = rng.standard_normal((64, 48)).astype(np.float16)
    ref = oracle.gemm_ref(A, 300, Bm, 48, 64, 48, 300, beta=0.5, C0=C0, ldc0=48)
    lib = 0.5 * C0.astype(np.float64) + A.astype(np.float64) @ Bm.astype(np.float64)
    assert np.abs(ref - lib).max() <= 1e-12 * np.abs(lib).max()


# ---------------------------------------------------------------- int8 (Section 2.2 names INT8)

def test_s8_literal_extremes_and_library(oracle):
    # [[1,-2],[3,4]] x [[-5,6],[7,-8]] = [[-19,22],[13,-14]]  (worked by hand)
    A = np.array([[1, -2], [3, 4]], dtype=np.int8)
    Bm = np.array([[-5, 6], [7, -8]], dtype=np.int8)
    assert oracle.gemm_s8_ref(A, 2, Bm, 2, 2, 2, 2).tolist() == [[-19, 22], [13, -14]]
    # extremes: (-128)^2 * K and -128 * 127 * K, closed form
    K = 1000
    A = np.full((3, K), -128, np.int8)
    Bm = np.full((K, 2), -128, np.int8)
    Bm[:, 1] = 127
    assert oracle.gemm_s8_ref(A, K, Bm, 2, 3, 2, K).tolist() == [[16384 * K, -128 * 127 * K]] * 3
    # random, all transposes, padded leading dimensions, accumulate: against numpy's int64 matmul
    rng = np.random.default_rng(21)
    M, N, K = 13, 9, 70
    Al = rng.integers(-128, 128, (M, K)).astype(np.int8)
    Bl = rng.integers(-128, 128, (K, N)).astype(np.int8)
    C0 = rng.integers(-2 ** 31, 2 ** 31, (M, N + 2)).astype(np.int32)
    want = Al.astype(np.int64) @ Bl.astype(np.int64)
    for tA in (0, 1):
        for tB in (0, 1):
            As = np.full((K, M + 3) if tA else (M, K + 3), 55, np.int8)
            Bs = np.full((N, K + 5) if tB else (K, N + 5), -77, np.int8)
            As[:, :(M if tA else K)] = Al.T if tA else Al
            Bs[:, :(K if tB else N)] = Bl.T if tB else Bl
            got = oracle.gemm_s8_ref(As, As.shape[1], Bs, Bs.shape[1], M, N, K, transA=tA, transB=tB)
            assert (got == want).all(), (tA, tB)
            got = oracle.gemm_s8_ref(As, As.shape[1], Bs, Bs.shape[1], M, N, K, transA=tA, transB=tB,
                                     C0=C0, ldc0=N + 2)
            assert (got == want + C0[:, :N].astype(np.int64)).all(), (tA, tB)
    # identity
    I = np.eye(K, dtype=np.int8)
    assert (oracle.gemm_s8_ref(Al, K, I, K, M, K, K) == Al).all()


# ---------------------------------------------------------------- FP8 E4M3 decoder

def test_f8e4m3_decoder_hand_values_and_structure(oracle):
    d = oracle.f8e4m3_to_f64
    assert d(0x00) == 0.0 and d(0x80) == 0.0 and np.signbit(d(0x80))
    assert d(0x01) == 2.0 ** -9 and d(0x07) == 7 * 2.0 ** -9          # subnormals
    assert d(0x08) == 2.0 ** -6                                      # smallest normal
    assert d(0x38) == 1.0 and d(0x3C) == 1.5 and d(0xB8) == -1.0
    assert d(0x40) == 2.0 and d(0x44) == 3.0 and d(0x48) == 4.0
    assert d(0x7E) == 448.0 and d(0xFE) == -448.0                    # largest finite: no infinities
    assert d(0x78) == 256.0                                          # exponent 15 is an ordinary binade
    assert np.isnan(d(0x7F)) and np.isnan(d(0xFF))
    vals = [d(b) for b in range(0x7F)]
    assert all(x < y for x, y in zip(vals, vals[1:]))               # strictly increasing over the positive codes
    for b in range(0x7F):
        assert d(b | 0x80) == -d(b)
    # every value is an integer multiple of 2^-9 and exactly representable in fp32
    w = oracle.f8e4m3_widen(np.arange(256, dtype=np.uint8))
    for b in range(256):
        v = d(b)
        if not np.isnan(v):
            assert w[b] == v and (v * 512) == int(v * 512)
    # second opinion where the library has the type
    try:
        import torch
        t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        ok = ~np.isnan(t)
        assert (t[ok] == w[ok]).all() and (np.isnan(t) == np.isnan(w)).all()
    except (ImportError, AttributeError, RuntimeError):
        pass


# ---------------------------------------------------------------- FP8 E5M2 decoder

def test_f8e5m2_decoder_hand_values_and_structure(oracle):
    d = oracle.f8e5m2_to_f64
    assert d(0x00) == 0.0 and d(0x80) == 0.0 and np.signbit(d(0x80))
    assert d(0x01) == 2.0 ** -16 and d(0x03) == 3 * 2.0 ** -16        # subnormals
    assert d(0x04) == 2.0 ** -14                                      # smallest normal
    assert d(0x3C) == 1.0 and d(0x3D) == 1.25 and d(0x3E) == 1.5 and d(0xBC) == -1.0
    assert d(0x40) == 2.0 and d(0x42) == 3.0 and d(0x44) == 4.0
    assert d(0x7B) == 57344.0 and d(0xFB) == -57344.0                 # largest finite
    assert d(0x7C) == np.inf and d(0xFC) == -np.inf
    assert all(np.isnan(d(b)) for b in (0x7D, 0x7E, 0x7F, 0xFD, 0xFE, 0xFF))
    vals = [d(b) for b in range(0x7D)]
    assert all(x < y for x, y in zip(vals, vals[1:]))                # strictly increasing up to +inf
    for b in range(0x7D):
        assert d(b | 0x80) == -d(b)
    # an E5M2 pattern is the top byte of the binary16 pattern of the same value: the
    # textbook definition, checked against numpy's binary16 decoding of byte << 8
    w = oracle.f8e5m2_widen(np.arange(256, dtype=np.uint8))
    half = (np.arange(256, dtype=np.uint16) << 8).view(np.float16).astype(np.float64)
    ok = ~np.isnan(half)
    assert (w[ok].astype(np.float64) == half[ok]).all() and (np.isnan(w) == np.isnan(half)).all()
    for b in range(256):
        v = d(b)
        if np.isfinite(v):
            assert w[b] == v and (v * 65536) == int(v * 65536)        # integer multiple of 2^-16
    try:
        import torch
        t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).to(torch.float32).numpy()
        okt = ~np.isnan(t)
        assert (t[okt] == w[okt]).all() and (np.isnan(t) == np.isnan(w)).all()
    except (ImportError, AttributeError, RuntimeError):
        pass


def test_f8e5m2_product_through_the_oracle(oracle):
    """Widened E5M2 operands through the GEMM oracle: integer-valued codes against int64."""
    codes = np.array([0x00, 0x3C, 0xBC, 0x40, 0xC0, 0x42, 0xC2, 0x44, 0xC4], np.uint8)      # 0, +-1, +-2, +-3, +-4
    ints = np.array([0, 1, -1, 2, -2, 3, -3, 4, -4], np.int64)
    rng = np.random.default_rng(17)
    ia, ib = rng.integers(0, 9, (13, 40)), rng.integers(0, 9, (40, 7))
    Aw, Bw = oracle.f8e5m2_widen(codes[ia]), oracle.f8e5m2_widen(codes[ib])
    ref = oracle.gemm_ref(Aw, 40, Bw, 7, 13, 7, 40)
    assert (ref == (ints[ia] @ ints[ib])).all()
