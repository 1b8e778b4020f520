"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before any GPU work (no compute calls here)."""
import os
import re

import pytest

from paper_2511_13764_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "brgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2511_13764_amd import build
        build.build()
    return B.load()


def test_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert {"gemm_f32", "gemm_bf16", "brgemm_bf16", "brgemm_fused", "gemm_workspace_bytes",
            "gemm_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in brgemm.h but not exported"
    assert set(B.EXPORTS) == set(names)


def test_strerror_and_variants(lib):
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(B.strerror(code), str) and B.strerror(code)
    v = B.variants()
    assert v and v[0].startswith("generic")
    assert B.gemm_variant_name(len(v)) == ""


P = 0x1000  # fake, never dereferenced: every call below is rejected or a no-op before launch


@pytest.mark.parametrize("kw", [
    dict(M=-1), dict(N=-1), dict(K=-1), dict(transA=2), dict(transB=-1),
    dict(lda=7), dict(ldb=7), dict(ldc=7), dict(A=0), dict(B=0), dict(C=0),
])
def test_gemm_rejects_bad_arguments(lib, kw):
    a = dict(transA=0, transB=0, M=8, N=8, K=8, A=P, lda=8, B=P, ldb=8, beta=0.0, C=P, ldc=8)
    a.update(kw)
    rc = B.gemm_f32(a["transA"], a["transB"], a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"],
                    a["beta"], a["C"], a["ldc"], stream=0, check=False)
    assert rc == B.INVALID_ARG
    rc = B.gemm_bf16(a["transA"], a["transB"], a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"],
                     a["beta"], a["C"], a["ldc"], 0, stream=0, check=False)
    assert rc == B.INVALID_ARG


def test_leading_dimension_follows_transpose_flag(lib):
    # transA: stored K x M, so lda >= M (not K); transB: stored N x K, so ldb >= K.
    assert B.gemm_f32(1, 0, 16, 8, 4, P, 8, P, 8, 0.0, P, 8, stream=0, check=False) == B.INVALID_ARG
    assert B.gemm_f32(0, 1, 4, 8, 16, P, 16, P, 8, 0.0, P, 8, stream=0, check=False) == B.INVALID_ARG


def test_empty_problems_are_no_ops(lib):
    assert B.gemm_f32(0, 0, 0, 8, 8, 0, 8, 0, 8, 0.0, 0, 8, stream=0, check=False) == B.OK
    assert B.gemm_f32(0, 0, 8, 0, 8, 0, 8, 0, 8, 0.0, 0, 8, stream=0, check=False) == B.OK
    assert B.gemm_bf16(0, 0, 0, 0, 0, 0, 1, 0, 1, 1.0, 0, 1, 1, stream=0, check=False) == B.OK
    # K == 0 with beta == 1: C = C, nothing to launch
    assert B.gemm_f32(0, 0, 8, 8, 0, 0, 1, 0, 8, 1.0, P, 8, stream=0, check=False) == B.OK


def test_brgemm_argument_rules(lib):
    ok = dict(transA=0, transB=0, M=8, N=8, K=8, batch=2, A=P, Ao=P, lda=8, B=P, Bo=P, ldb=8, C=P, ldc=8)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return B.brgemm_bf16(a["transA"], a["transB"], a["M"], a["N"], a["K"], a["batch"], a["A"], a["Ao"],
                             a["lda"], a["B"], a["Bo"], a["ldb"], 1.0, a["C"], a["ldc"], stream=0, check=False)
    assert call(batch=-1) == B.INVALID_ARG
    assert call(Ao=0) == B.INVALID_ARG
    assert call(Bo=0) == B.INVALID_ARG
    assert call(batch=0) == B.OK            # C = 1*C
    # fused entry: unknown dtype / flags, bias flag without bias, bf16 C with fp32 operands
    f = lambda **kw: B.brgemm_fused(kw.get("dt", 1), 0, 0, 8, 8, 8, 1, P, 0, 8, P, 0, 8, 0.0, P, 8,
                                    kw.get("cf32", 1), kw.get("bias", 0), kw.get("epi", 0), stream=0,
                                    check=False)
    assert f(dt=7) == B.INVALID_ARG
    assert f(epi=8) == B.INVALID_ARG
    assert f(epi=B.EPI_BIAS, bias=0) == B.INVALID_ARG
    assert f(dt=0, cf32=0) == B.INVALID_ARG


def test_workspace_rules(lib):
    assert B.gemm_workspace_bytes(B.DTYPE_BF16, 0, 8, 8, 1) == 0
    need = B.gemm_workspace_bytes(B.DTYPE_BF16, 128, 256, 64, 1)
    assert need >= 2 * 128 * 256 * 4
    lib = B.load()
    import ctypes
    # workspace_bytes > 0 with NULL pointer; misaligned workspace
    rc = lib.gemm_f32(0, 0, 8, 8, 8, P, 8, P, 8, 0.0, P, 8, None, 1024, None)
    assert rc == B.INVALID_ARG
    rc = lib.gemm_f32(0, 0, 8, 8, 8, P, 8, P, 8, 0.0, P, 8, ctypes.c_void_p(0x1010), 1024, None)
    assert rc == B.MISALIGNED_WORKSPACE
    # forced split without enough workspace
    B.gemm_force_variant(0, 4)
    try:
        rc = lib.gemm_f32(0, 0, 8, 8, 8, P, 8, P, 8, 0.0, P, 8, ctypes.c_void_p(0x1000), 256, None)
        assert rc == B.WORKSPACE_TOO_SMALL
    finally:
        B.gemm_force_variant(-1, 0)
    with pytest.raises(B.BrgemmError):
        B.gemm_force_variant(10_000, 0)


def test_mfma_probe_rejects_bad_arguments(lib):
    for kw in (dict(dtype=7), dict(operands=0), dict(sink=0), dict(iters=-1), dict(blocks=0)):
        a = dict(dtype=B.DTYPE_BF16, operands=P, iters=1, blocks=1, sink=P)
        a.update(kw)
        rc = B.gemm_mfma_probe(a["dtype"], a["operands"], a["iters"], a["blocks"], a["sink"], stream=0, check=False)
        assert rc == 0.0        # rejected before launch: no operation count is reported
        assert lib.gemm_mfma_probe(a["dtype"], a["operands"], a["iters"], a["blocks"], a["sink"], None, 0) == \
            B.INVALID_ARG


def test_packed_b_size_and_argument_rules(lib):
    assert B.gemm_packed_b_bytes(0, 5) == 0 and B.gemm_packed_b_bytes(5, -1) == 0
    assert B.gemm_packed_b_bytes(1, 1) == 64 * 256 * 2
    assert B.gemm_packed_b_bytes(4096, 11008) == 4096 * 11008 * 2
    assert B.gemm_packed_b_bytes(65, 257) == 128 * 512 * 2
    ok = dict(vnni=8, transB=0, K=16, N=8, B=P, ldb=8, k_rows=16, n_pitch=8, out=P)
    for kw in (dict(vnni=3), dict(vnni=16), dict(transB=2), dict(K=-1), dict(N=-1), dict(ldb=7), dict(k_rows=8),
               dict(k_rows=20), dict(n_pitch=7), dict(out=0), dict(out=P + 2), dict(B=0)):
        a = dict(ok)
        a.update(kw)
        rc = B.gemm_pack_vnni_bf16(a["vnni"], a["transB"], a["K"], a["N"], a["B"], a["ldb"], a["k_rows"],
                                   a["n_pitch"], a["out"], stream=0, check=False)
        assert rc == B.INVALID_ARG, kw
    # too small a destination for the library's own layout
    assert B.gemm_pack_b_bf16(0, 16, 8, P, 8, P, packed_bytes=64 * 256 * 2 - 1, stream=0, check=False) == B.INVALID_ARG
    # empty problems are no-ops
    assert B.gemm_pack_b_bf16(0, 0, 8, 0, 8, 0, packed_bytes=0, stream=0, check=False) == B.OK
    assert B.gemm_bf16_packed(0, 0, 8, 16, 0, 16, 0, 0.0, 0, 8, 0, stream=0, check=False) == B.OK
    # misaligned image, bad epilogue flags, missing bias
    assert B.gemm_bf16_packed(0, 4, 8, 16, P, 16, P + 2, 0.0, P, 8, 0, stream=0, check=False) == B.INVALID_ARG
    assert B.gemm_bf16_packed(0, 4, 8, 16, P, 16, P, 0.0, P, 8, 0, epilogue=4, stream=0, check=False) == B.INVALID_ARG
    assert B.gemm_bf16_packed(0, 4, 8, 16, P, 16, P, 0.0, P, 8, 0, epilogue=B.EPI_BIAS, stream=0,
                              check=False) == B.INVALID_ARG
    assert B.gemm_bf16_packed(0, 4, 8, 16, P, 15, P, 0.0, P, 8, 0, stream=0, check=False) == B.INVALID_ARG


def test_batched_argument_rules(lib):
    def call(**kw):
        a = dict(tA=0, tB=0, M=4, N=8, K=16, nmat=3, A=P, lda=16, sA=64, B=P, ldb=8, sB=128, beta=0.0, C=P, ldc=8,
                 sC=32, f32=0)
        a.update(kw)
        return B.gemm_bf16_batched(a["tA"], a["tB"], a["M"], a["N"], a["K"], a["nmat"], a["A"], a["lda"], a["sA"],
                                   a["B"], a["ldb"], a["sB"], a["beta"], a["C"], a["ldc"], a["sC"], a["f32"],
                                   stream=0, check=False)
    assert call(nmat=0) == B.OK                       # nothing to do
    assert call(M=0) == B.OK
    for kw in (dict(nmat=-1), dict(nmat=65536), dict(sA=-1), dict(sB=-8), dict(sC=31), dict(lda=15), dict(A=0),
               dict(tA=3)):
        assert call(**kw) == B.INVALID_ARG, kw
    assert B.gemm_f32_batched(0, 0, 4, 8, 16, 2, P, 16, 64, P, 8, 128, 0.0, P, 8, 3, stream=0, check=False) == \
        B.INVALID_ARG                                  # C matrices would overlap


def test_s8_argument_rules(lib):
    def call(**kw):
        a = dict(tA=0, tB=1, M=4, N=8, K=128, A=P, lda=128, B=P, ldb=128, acc=0, C=P, ldc=8)
        a.update(kw)
        return B.gemm_s8(a["tA"], a["tB"], a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"], a["acc"],
                         a["C"], a["ldc"], stream=0, check=False)
    assert call(M=0) == B.OK and call(N=0) == B.OK
    for kw in (dict(M=-1), dict(K=-1), dict(tA=2), dict(lda=127), dict(ldb=127), dict(ldc=7), dict(A=0), dict(C=0)):
        assert call(**kw) == B.INVALID_ARG, kw


def test_shape_to_tile_table(lib):
    """The automatic plan for the named configurations and around its crossovers (host logic)."""
    q = B.gemm_query_plan
    BF, F32, F16 = B.DTYPE_BF16, B.DTYPE_F32, B.DTYPE_F16
    assert q(BF, 0, 0, 4096, 4096, 4096) == ("bf16_pingpong_256x256x64", 1)
    assert q(BF, 0, 0, 8192, 8192, 8192) == ("bf16_pingpong_256x256x64", 1)
    assert q(F16, 0, 0, 4096, 4096, 4096) == ("bf16_pingpong_256x256x64", 1)
    assert q(BF, 0, 1, 4096, 11008, 4096) == ("bf16_pingpong_256x256x64", 1)
    assert q(BF, 0, 1, 4096, 4096, 11008) == ("bf16_pingpong_256x256x64", 1)
    # skinny M: streaming kernels, split from rounds x k-blocks
    assert q(BF, 0, 1, 16, 11008, 4096) == ("bf16_stream_32x128x64", 5)
    assert q(BF, 0, 1, 16, 4096, 11008) == ("bf16_stream_32x128x64", 8)
    assert q(BF, 0, 1, 128, 11008, 4096) == ("bf16_stream_128x128x64", 2)
    assert q(BF, 0, 1, 64, 11008, 4096)[0] == "bf16_stream_64x128x64"
    assert q(BF, 0, 1, 16, 11008, 4096, workspace_bytes=0) == ("bf16_stream_32x128x64", 1)   # no workspace, no split
    # squares: up to 256 tiles of 128x128 a streaming kernel, its tile height by how many
    # workgroups that puts on the chip; 257..512 tiles the two-stage kernel; beyond that 256x256
    assert q(BF, 0, 0, 512, 512, 512) == ("bf16_stream_32x128x64", 1)
    assert q(BF, 0, 0, 1024, 1024, 1024) == ("bf16_stream_32x128x64", 1)
    assert q(BF, 1, 0, 1024, 1024, 1024) == ("bf16_stream_128x128x64", 1)      # m-contiguous A: 128 rows only
    assert q(BF, 0, 0, 1280, 1280, 1280) == ("bf16_stream_64x128x64", 1)
    assert q(BF, 0, 0, 1536, 1536, 1536) == ("bf16_stream_128x128x64", 1)
    assert q(BF, 0, 0, 2048, 2048, 2048) == ("bf16_stream_128x128x64", 1)
    assert q(BF, 0, 0, 2304, 2304, 2304) == ("bf16_128x128x64", 1)
    assert q(BF, 0, 0, 2816, 2816, 2816) == ("bf16_128x128x64", 1)
    assert q(BF, 0, 0, 3072, 3072, 3072) == ("bf16_pingpong_256x256x64", 1)
    # 257..512 tiles with a long reduction: 256x256 tiles with the reduction split to fill the chip
    assert q(BF, 0, 1, 2048, 4096, 11008) == ("bf16_pingpong_256x256x64", 2)
    assert q(BF, 0, 1, 1024, 8192, 8192) == ("bf16_pingpong_256x256x64", 2)
    assert q(BF, 0, 1, 2048, 4096, 4096) == ("bf16_128x128x64", 1)              # short reduction: level, stays
    assert q(BF, 0, 1, 2048, 4096, 11008, workspace_bytes=0) == ("bf16_128x128x64", 1)
    # a B operand that streams (far larger than the L2s): only 128-row tiles
    assert q(BF, 0, 1, 256, 4096, 4096)[0] == "bf16_stream_128x128x64"
    assert q(BF, 0, 1, 1024, 2048, 8192) == ("bf16_stream_128x128x64", 2)
    # batch-reduce into a small C: split over the flattened (batch, k) range
    assert q(BF, 0, 0, 512, 512, 64, batch=64, lda=64, ldb=512) == ("bf16_stream_32x128x64", 8)
    # fp32: one kernel, split by the time model
    assert q(F32, 0, 0, 2048, 2048, 2048) == ("f32_128x128x32", 1)
    assert q(F32, 0, 0, 1024, 1024, 1024) == ("f32_128x128x32", 4)
    assert q(F32, 0, 0, 256, 256, 256) == ("f32_128x128x32", 8)
    # shapes the tuned kernels do not take run on the general kernel
    assert q(BF, 0, 0, 257, 131, 67)[0].startswith("generic")
    assert q(F32, 0, 0, 257, 131, 67)[0].startswith("generic")
    assert q(BF, 0, 0, 256, 256, 256, lda=260)[0].startswith("generic")        # ld % 8 != 0
    # bad queries
    import ctypes
    v, s = ctypes.c_int(), ctypes.c_int()
    assert lib.gemm_query_plan(7, 0, 0, 4, 4, 4, 1, 4, 4, 0, ctypes.byref(v), ctypes.byref(s)) == B.INVALID_ARG
    assert lib.gemm_query_plan(1, 0, 0, 4, 4, 64, 1, 8, 4, 0, ctypes.byref(v), ctypes.byref(s)) == B.INVALID_ARG


def test_f8_argument_rules(lib):
    def call(**kw):
        a = dict(tA=0, tB=1, M=4, N=8, K=128, A=P, lda=128, B=P, ldb=128, beta=0.0, C=P, ldc=8, f32=1)
        a.update(kw)
        return B.gemm_f8(a["tA"], a["tB"], a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"], a["beta"],
                         a["C"], a["ldc"], a["f32"], stream=0, check=False)
    assert call(M=0) == B.OK and call(N=0) == B.OK
    for kw in (dict(M=-1), dict(K=-1), dict(tB=2), dict(lda=127), dict(ldb=127), dict(ldc=7), dict(B=0), dict(C=0)):
        assert call(**kw) == B.INVALID_ARG, kw


def test_tune_rejects_bad_arguments_before_any_device_work(lib):
    import ctypes
    v, sp = ctypes.c_int(0), ctypes.c_int(0)
    ok = [B.DTYPE_BF16, 0, 0, 64, 64, 64, P, 64, P, 64, P, 64, 0, None, 0, None, ctypes.byref(v), ctypes.byref(sp), None]
    for pos, bad in ((0, 9), (1, 2), (3, 0), (4, -1), (5, 0), (7, 8), (9, 8), (11, 8), (6, None), (10, None)):
        a = list(ok)
        a[pos] = bad
        assert lib.gemm_tune(*a) == B.INVALID_ARG, pos
    a = list(ok)
    a[16] = None                                         # nowhere to put the answer
    assert lib.gemm_tune(*a) == B.INVALID_ARG
    a = list(ok)
    a[0], a[12] = B.DTYPE_F32, 0                         # fp32 operands need an fp32 C
    assert lib.gemm_tune(*a) == B.INVALID_ARG
    lib.gemm_tune_reset()
