"""Thin ctypes binding of libbrgemm_gfx950.so (include/brgemm.h).

Argument marshalling only: every step of the computation runs in the HIP
kernels behind the C ABI.  torch is used for device memory and streams.  The
library is loaded on first use; if it has not been built the call raises -
there is no CPU fallback.

Functions mirror the C entry points by name: gemm_f32, gemm_bf16, brgemm_bf16,
brgemm_fused, gemm_workspace_bytes, gemm_strerror, gemm_force_variant, ...
Tensor arguments are torch CUDA tensors (bf16 data may be torch.bfloat16,
torch.int16 or torch.uint16 - only the pointer is used); sizes and leading
dimensions are explicit, exactly as in the C signatures.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbrgemm_gfx950.so")

OK = 0
INVALID_ARG = -1
UNSUPPORTED = -2
WORKSPACE_TOO_SMALL = -3
HIP_ERROR = -4
MISALIGNED_WORKSPACE = -5
SCRATCH_TOO_SMALL = -6
NOALLOC_SCRATCH_BYTES = 32 << 20
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
PROBE_S8, PROBE_F8, PROBE_BF16_16X16X32 = 3, 4, 5
EPI_NONE, EPI_BIAS, EPI_RELU = 0, 1, 2

EXPORTS = ["gemm_f32", "gemm_bf16", "brgemm_bf16", "brgemm_fused", "gemm_workspace_bytes",
           "gemm_strerror", "gemm_last_hip_error", "gemm_force_variant", "gemm_variant_name",
           "gemm_last_variant", "gemm_last_split", "gemm_mfma_probe", "gemm_pack_vnni_bf16",
           "gemm_packed_b_bytes", "gemm_pack_b_bf16", "gemm_bf16_packed", "gemm_bf16_batched",
           "gemm_f32_batched", "gemm_f16", "gemm_s8", "gemm_query_plan", "gemm_f8", "gemm_bf16_noalloc", "gemm_bf8", "gemm_tune", "gemm_tune_reset"]

_lib = None


class BrgemmError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where} failed: {strerror(code)} (code {code})")


def load():
    """Load the shared library (once).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2511_13764_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci, cf, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.gemm_f32.restype = ci
    lib.gemm_f32.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, vp, sz, vp]
    lib.gemm_bf16.restype = ci
    lib.gemm_bf16.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, ci, vp, sz, vp]
    lib.gemm_bf16_noalloc.restype = ci
    lib.gemm_bf16_noalloc.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, ci, vp]
    lib.gemm_f16.restype = ci
    lib.gemm_f16.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, ci, vp, sz, vp]
    lib.gemm_f8.restype = ci
    lib.gemm_f8.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, ci, vp, sz, vp]
    lib.gemm_bf8.restype = ci
    lib.gemm_bf8.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, cf, vp, i64, ci, vp, sz, vp]
    lib.gemm_s8.restype = ci
    lib.gemm_s8.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, ci, vp, i64, vp]
    lib.brgemm_bf16.restype = ci
    lib.brgemm_bf16.argtypes = [ci, ci, i64, i64, i64, i64, vp, vp, i64, vp, vp, i64, cf, vp, i64, vp, sz, vp]
    lib.brgemm_fused.restype = ci
    lib.brgemm_fused.argtypes = [ci, ci, ci, i64, i64, i64, i64, vp, vp, i64, vp, vp, i64, cf, vp, i64, ci,
                                 vp, ci, vp, sz, vp]
    lib.gemm_workspace_bytes.restype = sz
    lib.gemm_workspace_bytes.argtypes = [ci, i64, i64, i64, i64]
    lib.gemm_strerror.restype = ctypes.c_char_p
    lib.gemm_strerror.argtypes = [ci]
    lib.gemm_last_hip_error.restype = ci
    lib.gemm_last_hip_error.argtypes = []
    lib.gemm_force_variant.restype = ci
    lib.gemm_force_variant.argtypes = [ci, ci]
    lib.gemm_variant_name.restype = ctypes.c_char_p
    lib.gemm_variant_name.argtypes = [ci]
    lib.gemm_last_variant.restype = ci
    lib.gemm_last_variant.argtypes = []
    lib.gemm_last_split.restype = ci
    lib.gemm_last_split.argtypes = []
    lib.gemm_pack_vnni_bf16.restype = ci
    lib.gemm_pack_vnni_bf16.argtypes = [ci, ci, i64, i64, vp, i64, i64, i64, vp, vp]
    lib.gemm_packed_b_bytes.restype = sz
    lib.gemm_packed_b_bytes.argtypes = [i64, i64]
    lib.gemm_pack_b_bf16.restype = ci
    lib.gemm_pack_b_bf16.argtypes = [ci, i64, i64, vp, i64, vp, sz, vp]
    lib.gemm_bf16_packed.restype = ci
    lib.gemm_bf16_packed.argtypes = [ci, i64, i64, i64, vp, i64, vp, cf, vp, i64, ci, vp, ci, vp, sz, vp]
    lib.gemm_bf16_batched.restype = ci
    lib.gemm_bf16_batched.argtypes = [ci, ci, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, cf, vp, i64, i64, ci, vp]
    lib.gemm_f32_batched.restype = ci
    lib.gemm_f32_batched.argtypes = [ci, ci, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, cf, vp, i64, i64, vp]
    lib.gemm_query_plan.restype = ci
    lib.gemm_query_plan.argtypes = [ci, ci, ci, i64, i64, i64, i64, i64, i64, sz, ctypes.POINTER(ci),
                                    ctypes.POINTER(ci)]
    lib.gemm_tune.restype = ci
    lib.gemm_tune.argtypes = [ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp, sz, vp,
                              ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_float)]
    lib.gemm_tune_reset.restype = None
    lib.gemm_tune_reset.argtypes = []
    lib.gemm_mfma_probe.restype = ci
    lib.gemm_mfma_probe.argtypes = [ci, vp, i64, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    _lib = lib
    return lib


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _ws(workspace):
    if workspace is None:
        return ctypes.c_void_p(0), 0
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _check(rc, where, check):
    if check and rc != OK:
        raise BrgemmError(rc, where)
    return rc


def gemm_f32(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_f32(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                         ws, nb, _stream(stream))
    return _check(rc, "gemm_f32", check)


def gemm_bf16(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, c_is_f32, workspace=None, stream=None,
              check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_bf16(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                          int(bool(c_is_f32)), ws, nb, _stream(stream))
    return _check(rc, "gemm_bf16", check)


def gemm_bf16_noalloc(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, c_is_f32, stream=None, check=True):
    rc = load().gemm_bf16_noalloc(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                                  int(bool(c_is_f32)), _stream(stream))
    return _check(rc, "gemm_bf16_noalloc", check)


def gemm_f16(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, c_is_f32, workspace=None, stream=None,
             check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_f16(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                         int(bool(c_is_f32)), ws, nb, _stream(stream))
    return _check(rc, "gemm_f16", check)


def gemm_f8(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, c_is_f32, workspace=None, stream=None,
            check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_f8(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                        int(bool(c_is_f32)), ws, nb, _stream(stream))
    return _check(rc, "gemm_f8", check)


def gemm_bf8(transA, transB, M, N, K, A, lda, B, ldb, beta, C, ldc, c_is_f32, workspace=None, stream=None,
             check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_bf8(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                         int(bool(c_is_f32)), ws, nb, _stream(stream))
    return _check(rc, "gemm_bf8", check)


def gemm_s8(transA, transB, M, N, K, A, lda, B, ldb, accumulate, C, ldc, stream=None, check=True):
    rc = load().gemm_s8(transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, int(bool(accumulate)), _ptr(C), ldc,
                        _stream(stream))
    return _check(rc, "gemm_s8", check)


def brgemm_bf16(transA, transB, M, N, K, batch, A_base, A_off, lda, B_base, B_off, ldb, beta, C, ldc,
                workspace=None, stream=None, check=True):
    ws, nb = _ws(workspace)
    rc = load().brgemm_bf16(transA, transB, M, N, K, batch, _ptr(A_base), _ptr(A_off), lda,
                            _ptr(B_base), _ptr(B_off), ldb, beta, _ptr(C), ldc, ws, nb, _stream(stream))
    return _check(rc, "brgemm_bf16", check)


def brgemm_fused(in_dtype, transA, transB, M, N, K, batch, A_base, A_off, lda, B_base, B_off, ldb, beta,
                 C, ldc, c_is_f32, bias, epilogue, workspace=None, stream=None, check=True):
    ws, nb = _ws(workspace)
    rc = load().brgemm_fused(in_dtype, transA, transB, M, N, K, batch, _ptr(A_base), _ptr(A_off), lda,
                             _ptr(B_base), _ptr(B_off), ldb, beta, _ptr(C), ldc, int(bool(c_is_f32)),
                             _ptr(bias), epilogue, ws, nb, _stream(stream))
    return _check(rc, "brgemm_fused", check)


def gemm_pack_vnni_bf16(vnni, transB, K, N, B, ldb, k_rows, n_pitch, out, stream=None, check=True):
    rc = load().gemm_pack_vnni_bf16(vnni, transB, K, N, _ptr(B), ldb, k_rows, n_pitch, _ptr(out), _stream(stream))
    return _check(rc, "gemm_pack_vnni_bf16", check)


def gemm_packed_b_bytes(K, N):
    return int(load().gemm_packed_b_bytes(K, N))


def gemm_pack_b_bf16(transB, K, N, B, ldb, packed, packed_bytes=None, stream=None, check=True):
    if packed_bytes is None:
        packed_bytes = packed.numel() * packed.element_size()
    rc = load().gemm_pack_b_bf16(transB, K, N, _ptr(B), ldb, _ptr(packed), packed_bytes, _stream(stream))
    return _check(rc, "gemm_pack_b_bf16", check)


def gemm_bf16_packed(transA, M, N, K, A, lda, packedB, beta, C, ldc, c_is_f32, bias=None, epilogue=0,
                     workspace=None, stream=None, check=True):
    ws, nb = _ws(workspace)
    rc = load().gemm_bf16_packed(transA, M, N, K, _ptr(A), lda, _ptr(packedB), beta, _ptr(C), ldc,
                                 int(bool(c_is_f32)), _ptr(bias), epilogue, ws, nb, _stream(stream))
    return _check(rc, "gemm_bf16_packed", check)


def gemm_bf16_batched(transA, transB, M, N, K, nmat, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC,
                      c_is_f32, stream=None, check=True):
    rc = load().gemm_bf16_batched(transA, transB, M, N, K, nmat, _ptr(A), lda, strideA, _ptr(B), ldb, strideB,
                                  beta, _ptr(C), ldc, strideC, int(bool(c_is_f32)), _stream(stream))
    return _check(rc, "gemm_bf16_batched", check)


def gemm_f32_batched(transA, transB, M, N, K, nmat, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC,
                     stream=None, check=True):
    rc = load().gemm_f32_batched(transA, transB, M, N, K, nmat, _ptr(A), lda, strideA, _ptr(B), ldb, strideB,
                                 beta, _ptr(C), ldc, strideC, _stream(stream))
    return _check(rc, "gemm_f32_batched", check)


def gemm_query_plan(dtype, transA, transB, M, N, K, batch=1, lda=None, ldb=None, workspace_bytes=1 << 40):
    """(variant name, split) the automatic plan picks; host logic only."""
    lda = (M if transA else K) if lda is None else lda
    ldb = (K if transB else N) if ldb is None else ldb
    v, s = ctypes.c_int(-1), ctypes.c_int(0)
    rc = load().gemm_query_plan(dtype, transA, transB, M, N, K, batch, lda, ldb, workspace_bytes,
                                ctypes.byref(v), ctypes.byref(s))
    if rc != OK:
        raise BrgemmError(rc, "gemm_query_plan")
    return gemm_variant_name(v.value), s.value


def gemm_tune(dtype, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, c_is_f32, workspace=None, stream=None,
              check=True):
    """Returns (variant name, split, microseconds per launch) of the fastest plan, which later calls
    of the same shape then take.  Waits for the device.  With check=False: the return code."""
    ws, nb = _ws(workspace)
    v, sp, us = ctypes.c_int(-1), ctypes.c_int(0), ctypes.c_float(0.0)
    rc = load().gemm_tune(dtype, transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                          int(bool(c_is_f32)), ws, nb, _stream(stream), ctypes.byref(v), ctypes.byref(sp),
                          ctypes.byref(us))
    if not check:
        return rc
    _check(rc, "gemm_tune", True)
    return gemm_variant_name(v.value), sp.value, us.value


def gemm_tune_reset():
    load().gemm_tune_reset()


def gemm_mfma_probe(dtype, operands, iters, blocks, sink, stream=None, check=True):
    """Returns the number of floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    rc = load().gemm_mfma_probe(dtype, _ptr(operands), iters, blocks, _ptr(sink), ctypes.byref(flops),
                                _stream(stream))
    _check(rc, "gemm_mfma_probe", check)
    return flops.value


def gemm_workspace_bytes(dtype, M, N, K, batch=1):
    return int(load().gemm_workspace_bytes(dtype, M, N, K, batch))


def strerror(code):
    return load().gemm_strerror(code).decode()


gemm_strerror = strerror


def gemm_last_hip_error():
    return int(load().gemm_last_hip_error())


def gemm_force_variant(variant, split=0):
    rc = load().gemm_force_variant(variant, split)
    if rc != OK:
        raise BrgemmError(rc, "gemm_force_variant")


def gemm_variant_name(v):
    return load().gemm_variant_name(v).decode()


def variants():
    """All variant names, indexed by variant number."""
    out, v = [], 0
    while True:
        n = gemm_variant_name(v)
        if not n:
            return out
        out.append(n)
        v += 1


def gemm_last_variant():
    return int(load().gemm_last_variant())


def gemm_last_split():
    return int(load().gemm_last_split())
