"""Helpers of the GPU parity tests: upload a workload case, call the C ABI through
the binding, fetch the result, and compute the oracle's answer for the same bits."""
import numpy as np
import torch

from paper_2511_13764_amd import binding as B
from paper_2511_13764_amd import workloads as W

TOL_F32 = 1e-5        # relative Frobenius error, fp32 in / fp32 out
TOL_BF16 = 2e-3       # bf16 in / fp32 accumulate / bf16 out
TOL_BF16_F32OUT = 1e-5  # bf16 in / fp32 out: only fp32 summation error remains

SENTINEL_F32 = np.float32(-7777.25)
SENTINEL_BF16 = np.uint16(0xC5F3)     # some finite bf16 value


def dev(x):
    """numpy -> device tensor (uint16 carried as int16; only the pointer matters)."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def host(t, as_uint16=False):
    a = t.cpu().numpy()
    return a.view(np.uint16) if as_uint16 else a


def widen(out):
    """GPU output (fp32 array or bf16 bits) -> fp64 values."""
    if out.dtype == np.uint16:
        return (out.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return out.astype(np.float64)


def rel_fro(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    d = np.linalg.norm(np.asarray(got, dtype=np.float64) - ref)
    n = np.linalg.norm(ref)
    return d / n if n > 0 else d


def make_c(M, N, ldc, c_is_f32, C0, beta):
    """Device C buffer of M rows with leading dimension ldc.  Padding columns hold
    a sentinel; the live part holds C0 (beta != 0) or NaN (beta == 0, must not be read)."""
    if c_is_f32:
        buf = np.full((M, ldc), SENTINEL_F32, dtype=np.float32)
        buf[:, :N] = C0 if (beta != 0.0 and C0 is not None) else np.float32(np.nan)
    else:
        buf = np.full((M, ldc), SENTINEL_BF16, dtype=np.uint16)
        buf[:, :N] = C0 if (beta != 0.0 and C0 is not None) else W.BF16_NAN
    return buf


def check_padding(out_full, N, c_is_f32):
    pad = out_full[:, N:]
    if pad.size:
        want = SENTINEL_F32 if c_is_f32 else SENTINEL_BF16
        assert (pad == want).all(), "kernel wrote outside the N live columns of C"


def run_gemm_case(case, *, ldc=None, workspace_bytes=0, bias=None, relu=False, force=None, via_fused=False,
                  bias_shift=0):
    """Run one GemmCase through the C ABI.  Returns (live output array, full buffer).
    bias_shift > 0 places the bias that many elements into a NaN-filled allocation, so
    that its pointer is 4-byte but not 16-byte aligned."""
    M, N, K = case.M, case.N, case.K
    ldc = ldc or N
    c_is_f32 = case.c_is_f32
    dA, dB = dev(case.A), dev(case.B)
    cbuf = make_c(M, N, ldc, c_is_f32, case.C0, case.beta)
    dC = dev(cbuf)
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    dbias = None
    if bias is not None:
        holder = np.full(bias_shift + bias.size + 4, np.nan, np.float32)
        holder[bias_shift:bias_shift + bias.size] = bias
        dbias = dev(holder)[bias_shift:]
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        if bias is not None or relu or via_fused:
            epi = (B.EPI_BIAS if bias is not None else 0) | (B.EPI_RELU if relu else 0)
            B.brgemm_fused(B.DTYPE_BF16 if case.dtype == "bf16" else B.DTYPE_F32, case.transA, case.transB,
                           M, N, K, 1, dA, None, case.lda, dB, None, case.ldb, case.beta, dC, ldc,
                           c_is_f32, dbias, epi, workspace=ws)
        elif case.dtype == "f32":
            B.gemm_f32(case.transA, case.transB, M, N, K, dA, case.lda, dB, case.ldb, case.beta, dC, ldc,
                       workspace=ws)
        else:
            B.gemm_bf16(case.transA, case.transB, M, N, K, dA, case.lda, dB, case.ldb, case.beta, dC, ldc,
                        c_is_f32, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = host(dC, as_uint16=not c_is_f32)
    check_padding(full, N, c_is_f32)
    return full[:, :N], full


def oracle_gemm_case(oracle, case, rows=None, bias=None, relu=False):
    return oracle.gemm_ref(case.A, case.lda, case.B, case.ldb, case.M, case.N, case.K,
                           transA=case.transA, transB=case.transB, beta=case.beta, C0=case.C0,
                           ldc0=(case.C0.shape[1] if case.C0 is not None else None),
                           bias=bias, relu=relu, rows=rows)


def run_brgemm_case(case, *, workspace_bytes=0, force=None):
    dpool = dev(case.pool)
    dAo = torch.from_numpy(case.A_off.astype(np.int64)).cuda()
    dBo = torch.from_numpy(case.B_off.astype(np.int64)).cuda()
    cbuf = make_c(case.M, case.N, case.ldc, True, case.C0, case.beta)
    dC = dev(cbuf)
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        B.brgemm_bf16(case.transA, case.transB, case.M, case.N, case.K, case.batch, dpool, dAo, case.lda,
                      dpool, dBo, case.ldb, case.beta, dC, case.ldc, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = host(dC)
    check_padding(full, case.N, True)
    return full[:, :case.N]


def oracle_brgemm_case(oracle, case, rows=None):
    return oracle.brgemm_ref(case.pool, case.A_off, case.lda, case.pool, case.B_off, case.ldb,
                             case.M, case.N, case.K, transA=case.transA, transB=case.transB,
                             beta=case.beta, C0=case.C0, ldc0=case.ldc, rows=rows)


def sample_rows(M, count, tile=256, seed=5):
    """Rows hitting the first, last and interior tiles and both halves of each wave tile."""
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 255, M - 256, M - 129, M - 128, M - 1, M // 2, M // 2 - 1]
    fixed = [r for r in fixed if 0 <= r < M]
    extra = rng.integers(0, M, size=max(0, count - len(fixed))).tolist()
    return sorted(set(fixed + extra))


def check_bf16_out_elementwise(oracle, out_bits, ref, abs_ref, K, *, what=""):
    """Every element of a bf16 C against the fp64 oracle.

    got = RNE_bf16(s), s an fp32 sum of the K exact products in some order.  abs_ref is
    the oracle's product of the absolute values, i.e. S = sum_k |a_k b_k| per element.
      (1) worst case: |s - ref| <= gamma_K * S  (gamma_K = K u / (1 - K u), u = 2^-24: the
          textbook bound for any order of K - 1 fp32 additions), and the rounding to 8
          significant bits moves s by at most half a spacing, 2^(floor(log2 |s|) - 8);
          must hold for every element.
      (2) the same with the rounding-error bound for errors that do not all pile up the
          same way, 4 sqrt(K) u S (Higham & Mary's probabilistic gamma with lambda = 4),
          about sqrt(K)/4 times tighter; also asserted for every element.  An element
          whose sum lost or gained one term of typical size fails it.
      (3) the stored bits equal the oracle's own rounding of ref except where the sum sits
          within the fp32 error of a rounding boundary: at most 1 % of the elements.
    Returns the largest |got - ref| / bound (2) and the fraction counted in (3)."""
    u = 2.0 ** -24
    got = widen(out_bits)
    err = np.abs(got - ref)
    tiny = 2.0 ** -133                                   # half the smallest bf16 subnormal
    for name, delta in (("worst-case", (K * u / (1.0 - K * u)) * abs_ref),
                        ("probabilistic", 4.0 * np.sqrt(K) * u * abs_ref)):
        big = np.maximum(np.abs(ref) + delta, 2.0 ** -126)
        bound = 2.0 ** (np.floor(np.log2(big)) - 8) + delta + tiny      # half a bf16 spacing at |s|
        excess = err - bound
        worst = np.unravel_index(np.argmax(excess), excess.shape)
        assert excess[worst] <= 0.0, (f"{what}: element {worst} got {got[worst]} ref {ref[worst]} "
                                      f"{name} bound {bound[worst]}")
    ratio = float((err / bound).max())
    want = oracle.round_to_out(ref, 1)
    frac = float((out_bits != want).mean())
    assert frac <= 0.01, f"{what}: {frac:.4f} of the elements differ from the oracle's rounding"
    return ratio, frac


def check_bf16_case_elementwise(oracle, case, out_bits, ref, bias=None):
    """Per-element bound for a bf16-out GemmCase of any size, beta and bias included: the
    stored value is RNE_bf16 of an fp32 evaluation of beta*C0 + sum_k a_k b_k (+ bias), so
    |got - ref| <= half a bf16 spacing at the fp32 value + gamma_{K+2} * S, where
    S = |beta||C0| + sum_k |a_k||b_k| (+ |bias|) comes from the oracle run on the absolute
    values.  Unlike a Frobenius tolerance this needs no allowance for results of only a few
    elements."""
    absA = case.A & np.uint16(0x7FFF) if case.A.dtype == np.uint16 else np.abs(case.A)
    absB = case.B & np.uint16(0x7FFF) if case.B.dtype == np.uint16 else np.abs(case.B)
    absC = None
    if case.C0 is not None and case.beta != 0.0:
        absC = case.C0 & np.uint16(0x7FFF) if case.C0.dtype == np.uint16 else np.abs(case.C0)
    S = oracle.gemm_ref(absA, case.lda, absB, case.ldb, case.M, case.N, case.K, transA=case.transA,
                        transB=case.transB, beta=abs(case.beta), C0=absC,
                        ldc0=(absC.shape[1] if absC is not None else None),
                        bias=(np.abs(bias) if bias is not None else None))
    u = 2.0 ** -24
    n = case.K + 2
    delta = (n * u / (1.0 - n * u)) * S
    got = widen(out_bits)
    big = np.maximum(np.abs(ref) + delta, 2.0 ** -126)
    bound = 2.0 ** (np.floor(np.log2(big)) - 8) + delta + 2.0 ** -133
    excess = np.abs(got - ref) - bound
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0.0, f"{case.name}: element {worst} got {got[worst]} ref {ref[worst]} bound {bound[worst]}"


def check_f32_case_elementwise(oracle, case, out, ref, rows=None):
    """Per-element bound for an fp32-in / fp32-out GemmCase: K rounded products, K - 1
    additions and the beta*C0 term, each with a relative error of at most u = 2^-24, in any
    order: |got - ref| <= gamma_{K+3} * S with S = |beta||C0| + sum_k |a_k||b_k| from the
    oracle run on the absolute values.  An element that lost one term of typical size fails."""
    absC = np.abs(case.C0) if (case.C0 is not None and case.beta != 0.0) else None
    S = oracle.gemm_ref(np.abs(case.A), case.lda, np.abs(case.B), case.ldb, case.M, case.N, case.K,
                        transA=case.transA, transB=case.transB, beta=abs(case.beta), C0=absC,
                        ldc0=(absC.shape[1] if absC is not None else None), rows=rows)
    u = 2.0 ** -24
    n = case.K + 3
    bound = (n * u / (1.0 - n * u)) * S + 2.0 ** -149
    excess = np.abs(widen(out) - ref) - bound
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0.0, f"{case.name}: element {worst} off by {np.abs(widen(out) - ref)[worst]}, bound {bound[worst]}"
    return float((np.abs(widen(out) - ref) / bound).max())
