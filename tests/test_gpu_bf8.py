"""GPU parity of the FP8 E5M2 operand path (gemm_bf8): the oracle widens the same bytes
exactly with its own decoder and multiplies them in fp64.  The limits come from the same
stated model of the 128-deep matrix instruction as for E4M3 (tests/test_gpu_f8.py), which
is checked on the device for this format too."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from paper_2511_13764_amd import binding as B
from paper_2511_13764_amd import workloads as W

import gpu_helpers as H
import test_gpu_f8 as F

pytestmark = pytest.mark.gpu

NAN_BYTE = 0x7F          # an E5M2 NaN pattern (exponent 31, fraction != 0)


def say(msg):
    print(f"[case] {msg}", flush=True)


def bf8_bytes(seed, tensor, shape, scale=1.0):
    """N(0, scale) values rounded to E5M2 by the library conversion (input generation only)."""
    x = torch.from_numpy(W.normal_f32(seed, tensor, shape) * np.float32(scale))
    return x.to(torch.float8_e5m2).view(torch.uint8).numpy().copy()


def run_bf8(A, Bm, M, N, K, tA, tB, *, beta=0.0, C0=None, c_f32=True, ldc=None, workspace_bytes=0, force=None):
    ldc = ldc or N
    cbuf = H.make_c(M, N, ldc, c_f32, C0, beta)
    dA, dB, dC = torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), H.dev(cbuf)
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda") if workspace_bytes else None
    if force is not None:
        B.gemm_force_variant(*force)
    try:
        B.gemm_bf8(tA, tB, M, N, K, dA, A.shape[1], dB, Bm.shape[1], beta, dC, ldc, c_f32, workspace=ws)
        torch.cuda.synchronize()
    finally:
        if force is not None:
            B.gemm_force_variant(-1, 0)
    full = H.host(dC, as_uint16=not c_f32)
    H.check_padding(full, N, c_f32)
    return H.widen(full[:, :N])


def ref_bf8(oracle, A, Bm, M, N, K, tA, tB, **kw):
    Aw, Bw = oracle.f8e5m2_widen(A), oracle.f8e5m2_widen(Bm)
    return oracle.gemm_ref(Aw, Aw.shape[1], Bw, Bw.shape[1], M, N, K, transA=tA, transB=tB, **kw)


def test_bf8_every_variant_nt(oracle):
    M, N, K = 512, 768, 512
    A, Bm = bf8_bytes(310, 0, (M, K)), bf8_bytes(310, 1, (N, K))
    ref = ref_bf8(oracle, A, Bm, M, N, K, 0, 1)
    Aw, Bw = oracle.f8e5m2_widen(A).astype(np.float64), oracle.f8e5m2_widen(Bm).astype(np.float64)
    ws = B.gemm_workspace_bytes(1, M, N, K)
    ran = set()
    for v, name in enumerate(B.variants()):
        for split in (1, 2):
            say(f"bf8 variant={name} split={split}")
            try:
                out = run_bf8(A, Bm, M, N, K, 0, 1, workspace_bytes=ws, force=(v, split))
            except B.BrgemmError as e:
                assert e.code == B.INVALID_ARG
                continue
            ran.add(name)
            if name.startswith("generic"):
                assert H.rel_fro(out, ref) <= 1e-6, (name, split)
            else:
                F.check_f8_against_model(out[::4], ref[::4], Aw[::4], Bw, f"bf8 {name} split={split}")
    assert {"generic_64x64x16_f32mfma", "bf16_pingpong_256x256x64", "bf16_stream_32x128x64",
            "bf16_stream_64x128x64", "bf16_stream_128x128x64"} <= ran


@pytest.mark.parametrize("tA,tB", [(0, 0), (1, 0), (1, 1)])
def test_bf8_every_variant_other_layouts(oracle, tA, tB):
    F.every_variant_other_layout(run_bf8, oracle.f8e5m2_widen, lambda *a: ref_bf8(oracle, *a), bf8_bytes, 312, tA, tB, "bf8")


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K,pad", [(257, 131, 67, 3), (360, 520, 1024, 16), (16, 384, 2048, 0), (368, 528, 1024, 16)])
def test_bf8_all_layouts_ragged_beta_bf16_out(oracle, M, N, K, pad, tA, tB):
    ra, ca = (K, M) if tA else (M, K)
    rb, cb = (N, K) if tB else (K, N)
    A = np.full((ra, ca + pad), NAN_BYTE, np.uint8)          # NaN in the padding
    Bm = np.full((rb, cb + pad), NAN_BYTE, np.uint8)
    A[:, :ca] = bf8_bytes(311, 0, (ra, ca))
    Bm[:, :cb] = bf8_bytes(311, 1, (rb, cb))
    C0 = W.to_bf16_bits(W.normal_f32(311, 2, (M, N)))
    say(f"bf8 {M}x{N}x{K} t{tA}{tB} pad={pad}")
    ref = ref_bf8(oracle, A, Bm, M, N, K, tA, tB, beta=-0.5, C0=C0, ldc0=N)
    out = run_bf8(A, Bm, M, N, K, tA, tB, beta=-0.5, C0=C0, c_f32=False, ldc=N + pad,
                  workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
    assert np.isfinite(out).all()
    assert H.rel_fro(out, ref) <= H.TOL_BF16, B.gemm_variant_name(B.gemm_last_variant())


def test_bf8_small_integers_extremes_and_infinity(oracle):
    M, N, K = 256, 384, 1024
    codes = np.array([0x00, 0x3C, 0xBC, 0x40, 0xC0, 0x42, 0xC2, 0x44, 0xC4], np.uint8)    # 0, +-1, +-2, +-3, +-4
    rng = np.random.default_rng(9)
    A, Bm = rng.choice(codes, (M, K)), rng.choice(codes, (N, K))
    ref = ref_bf8(oracle, A, Bm, M, N, K, 0, 1)
    out = run_bf8(A, Bm, M, N, K, 0, 1)
    assert (out == ref).all()
    A[:] = 0x7B                                                     # 57344, the largest finite value
    Bm[:] = 0xFB                                                    # -57344
    Bm[::2] = 0x01                                                  # 2^-16, the smallest subnormal
    ref = ref_bf8(oracle, A, Bm, M, N, K, 0, 1)
    out = run_bf8(A, Bm, M, N, K, 0, 1)
    assert (out == ref).all() and out[0, 1] == -57344.0 * 57344.0 * K and out[0, 0] == 57344.0 * 2.0 ** -16 * K
    # an infinity in row 3 of A reaches exactly row 3 of C (times a positive B: +inf)
    A[:] = 0x3C
    Bm[:] = 0x3C
    A[3, 5] = 0x7C
    out = run_bf8(A, Bm, M, N, K, 0, 1)
    assert np.isposinf(out[3]).all() and np.isfinite(np.delete(out, 3, axis=0)).all()


def test_bf8_full_size_sampled_rows(oracle):
    M = N = K = 4096
    A, Bm = bf8_bytes(312, 0, (M, K)), bf8_bytes(312, 1, (N, K), scale=0.05)
    rows = H.sample_rows(M, 16)
    ref = ref_bf8(oracle, A, Bm, M, N, K, 0, 1, rows=rows)
    out = run_bf8(A, Bm, M, N, K, 0, 1, workspace_bytes=B.gemm_workspace_bytes(1, M, N, K))
    say(f"bf8 4096^3 -> {B.gemm_variant_name(B.gemm_last_variant())}")
    sub = rows[::2][:8]
    idx = [rows.index(r) for r in sub]
    Aw = oracle.f8e5m2_widen(A[sub]).astype(np.float64)
    Bw = oracle.f8e5m2_widen(Bm[::4]).astype(np.float64)
    F.check_f8_against_model(out[sub][:, ::4], ref[idx][:, ::4], Aw, Bw, "bf8 4096^3")
    assert H.rel_fro(out[rows], ref) <= 2e-4        # E5M2 products lose bits sooner: 6-bit products, wider spread


def _one_element(prods, K=128):
    def code(v):
        t = torch.tensor([v], dtype=torch.float32).to(torch.float8_e5m2)
        assert float(t.float()[0]) == v, f"{v} is not an E5M2 value"
        return int(t.view(torch.uint8)[0])
    A = np.zeros((16, K), np.uint8)
    Bm = np.zeros((16, K), np.uint8)
    for k, (a, b) in enumerate(prods):
        A[0, k], Bm[0, k] = code(a), code(b)
    return run_bf8(A, Bm, 16, 16, K, 0, 1)[0, 0]


def test_bf8_instruction_keeps_13_bits_below_the_largest_product():
    """The model's behaviour observed for E5M2 operands (see the E4M3 test of the same name)."""
    big = (16.0, 16.0)                                                    # 2^8
    assert _one_element([big, (2.0 ** -5, 1.0)]) == 256.0 + 2.0 ** -5      # 13 bits below: kept
    assert _one_element([big, (2.0 ** -6, 1.0)]) == 256.0                  # 14 bits below: dropped
    assert _one_element([big, (1.75 * 2.0 ** -6, 1.0)]) == 256.0           # cut off, not rounded
    assert _one_element([big, (-1.75 * 2.0 ** -6, 1.0)]) == 256.0
    top = 57344.0 * 57344.0                                               # 1.53 * 2^31
    assert _one_element([(57344.0, 57344.0), (512.0, 512.0)]) == top + 2.0 ** 18   # 2^(31-13) kept
    assert _one_element([(57344.0, 57344.0), (256.0, 256.0)]) == top               # 2^16 dropped
    assert _one_element([big] + [(2.0 ** -6, 1.0)] * 7) == 256.0
    assert _one_element([big] + [(0.0, 0.0)] * 127 + [(2.0 ** -6, 1.0)], K=256) == 256.0 + 2.0 ** -6
    assert B.gemm_variant_name(B.gemm_last_variant()).startswith("bf16_stream")
