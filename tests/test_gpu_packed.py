"""GPU parity of the pre-packed-B path (Section 2.2, Figure 1): the device packer
against the oracle's packer bit for bit, and the GEMM on the packed image against
the oracle's plain product of the unpacked operands."""
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


def gpu_pack_vnni(Bm, ldb, K, N, v, transB, k_rows, n_pitch):
    dB = H.dev(Bm)
    out = torch.full((k_rows // v, n_pitch, v), 0x7FC0, dtype=torch.int16, device="cuda")   # NaN canary
    B.gemm_pack_vnni_bf16(v, transB, K, N, dB, ldb, k_rows, n_pitch, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def test_device_packer_reproduces_figure_1(oracle):
    from test_oracle_pins import _read_fig1
    flat, packed = _read_fig1()
    got = gpu_pack_vnni(flat, 4, 4, 4, 2, 0, 4, 4)
    assert (got == packed).all()
    got_t = gpu_pack_vnni(np.ascontiguousarray(flat.T), 4, 4, 4, 2, 1, 4, 4)
    assert (got_t == packed).all()


@pytest.mark.parametrize("v", [2, 4, 8])
@pytest.mark.parametrize("transB", [0, 1])
@pytest.mark.parametrize("K,N,pad", [(64, 256, 0), (100, 37, 5), (1, 1, 0), (520, 1000, 8), (67, 300, 3)])
def test_device_packer_bit_exact(oracle, v, transB, K, N, pad):
    rng = np.random.default_rng(100 * v + K + N + transB)
    rows, cols = (N, K) if transB else (K, N)
    Bm = rng.integers(0, 65536, size=(rows, cols + pad)).astype(np.uint16)
    k_rows = (K + 63) // 64 * 64
    n_pitch = (N + 255) // 256 * 256
    say(f"pack v={v} transB={transB} {K}x{N} ld={cols + pad}")
    want = oracle.pack_vnni(Bm, cols + pad, K, N, v, transB=transB, k_rows=k_rows, n_pitch=n_pitch)
    got = gpu_pack_vnni(Bm, cols + pad, K, N, v, transB, k_rows, n_pitch)
    assert got.shape == want.shape and (got == want).all()


def run_packed(case, *, workspace_bytes=0, bias=None, relu=False, force=None, ldc=None):
    """Pack case.B on the device with the library's layout, then run the packed GEMM."""
    M, N, K = case.M, case.N, case.K
    ldc = ldc or N
    dA, dB = H.dev(case.A), H.dev(case.B)
    nbytes = B.gemm_packed_b_bytes(K, N)
    packed = torch.full((max(nbytes // 2, 8),), 0x7FC0, dtype=torch.int16, device="cuda")
    B.gemm_pack_b_bf16(case.transB, K, N, dB, case.ldb, packed)
    cbuf = H.make_c(M, N, ldc, case.c_is_f32, case.C0, case.beta)
    dC = H.dev(cbuf)
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    dbias = H.dev(bias) if bias is not None else None
    epi = (B.EPI_BIAS if bias is not None else 0) | (B.EPI_RELU if relu else 0)
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        B.gemm_bf16_packed(case.transA, M, N, K, dA, case.lda, packed, case.beta, dC, ldc, case.c_is_f32,
                           dbias, epi, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = H.host(dC, as_uint16=not case.c_is_f32)
    H.check_padding(full, N, case.c_is_f32)
    return full[:, :N], B.gemm_variant_name(B.gemm_last_variant()), B.gemm_last_split()


def make_case(name, M, N, K, tA, tB, beta=0.0, c_f32=True, seed=80, pad=0):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((ra, ca + pad), np.nan, np.float32)
    Bm = np.full((rb, cb + pad), np.nan, np.float32)
    A[:, :ca] = W.normal_f32(seed, 0, (ra, ca))
    Bm[:, :cb] = W.normal_f32(seed, 1, (rb, cb))
    C0 = None
    if beta != 0.0:
        C0 = W.normal_f32(seed, 2, (M, N))
        if not c_f32:
            C0 = W.to_bf16_bits(C0)
    return W.GemmCase(name, "bf16", M, N, K, tA, tB, beta, W.to_bf16_bits(A), W.to_bf16_bits(Bm), C0, c_f32)


def test_packed_gemm_every_variant(oracle):
    """Every kernel variant that takes bf16 operands, forced in turn, reads the packed image."""
    M, N, K = 512, 768, 512
    ws = B.gemm_workspace_bytes(1, M, N, K)
    for tA in (0, 1):
        case = make_case(f"packed_variants_t{tA}", M, N, K, tA, 0)
        ref = H.oracle_gemm_case(oracle, case)
        ran = []
        for v, name in enumerate(B.variants()):
            for split in (1, 2):
                say(f"{case.name} variant={name} split={split}")
                try:
                    out, used, _ = run_packed(case, workspace_bytes=ws, force=(v, split))
                except B.BrgemmError as e:
                    assert e.code == B.INVALID_ARG
                    continue
                assert used == name
                ran.append(name)
                assert H.rel_fro(H.widen(out), ref) <= 1e-5, (name, split)
        want = {"generic_64x64x16_f32mfma", "bf16_128x128x64", "bf16_pingpong_256x256x64"}
        if tA == 0:
            want |= {"bf16_stream_32x128x64", "bf16_stream_64x128x64", "bf16_stream_128x128x64"}
        assert want <= set(ran)


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(257, 131, 64), (16, 200, 1024), (300, 1000, 192), (33, 520, 100), (1, 1, 1),
                                   (128, 264, 2048)])
def test_packed_gemm_ragged(oracle, M, N, K, tA, tB):
    """Ragged M, N (the image is zero-padded to 256 columns), K that is not a multiple
    of 64 (general kernel), padded leading dimensions of the sources, beta and a bf16 C."""
    if tA == 1 and M % 8:
        M += 8 - M % 8          # keeps the tuned kernels in play for transposed A
    case = make_case(f"packed_ragged_{M}x{N}x{K}_t{tA}{tB}", M, N, K, tA, tB, beta=-0.75, c_f32=False, pad=8)
    say(case.name)
    ref = H.oracle_gemm_case(oracle, case)
    ws = B.gemm_workspace_bytes(1, M, N, K)
    out, used, split = run_packed(case, workspace_bytes=ws, ldc=N + 8)
    assert np.isfinite(H.widen(out)).all(), "padding (NaN) leaked into the result"
    # every element within one bf16 rounding of an fp32 evaluation; the Frobenius limit (an RMS
    # figure) only where there are enough elements for it to mean something
    H.check_bf16_case_elementwise(oracle, case, out, ref)
    if M * N >= 4096:
        err = H.rel_fro(H.widen(out), ref)
        assert err <= H.TOL_BF16, (used, split, err)


def test_packed_gemm_fused_bias_relu_matches_flat(oracle):
    M, N, K = 192, 520, 256
    case = make_case("packed_fused", M, N, K, 0, 1, beta=0.5, c_f32=True)
    bias = W.normal_f32(81, 3, (N,))
    ref = H.oracle_gemm_case(oracle, case, bias=bias, relu=True)
    out, used, _ = run_packed(case, bias=bias, relu=True, workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
    assert H.rel_fro(H.widen(out), ref) <= 1e-5, used
    assert (H.widen(out) >= 0).all()


@pytest.mark.parametrize("which,M", [("up", 16), ("up", 128), ("down", 16), ("up", 4096)])
def test_packed_mlp_shapes(oracle, which, M):
    """The MLP shapes with their weights packed once: skinny M takes the streaming
    kernels, M = 4096 the 256x256 kernel; checked on sampled complete rows."""
    case = W.config4_mlp(M, which)
    rows = H.sample_rows(M, 24) if M > 128 else None
    ref = H.oracle_gemm_case(oracle, case, rows=rows)
    out, used, split = run_packed(case, workspace_bytes=B.gemm_workspace_bytes(1, M, case.N, case.K))
    say(f"{case.name} packed -> {used} split={split}")
    got = H.widen(out if rows is None else out[rows])
    assert H.rel_fro(got, ref) <= H.TOL_BF16
    assert used.startswith("bf16_stream") if M <= 128 else used == "bf16_pingpong_256x256x64"
