"""ctypes front end of the CPU oracle (oracle/brgemm_oracle.c).

TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this module.  It imports nothing from the GPU
package and the GPU package imports nothing from here.

The arithmetic lives in the C file; this module only marshals numpy arrays.
Element types: numpy float32 = fp32, numpy uint16 = bf16 bit patterns.

Defines (Algorithm 1's input/output statement; Section 2.1 for scattered
tiles; Section 5(d) for GEMM as the batch-1 case):

    ref = beta * C0 + sum_i A_i x B_i      (fp64, every input widened exactly)
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_brgemm.so")
_lib = None

F32, BF16, F16 = 0, 1, 2


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _b  # building the checker is not using it
        _b.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    i64, vp, cint = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.oracle_brgemm.restype = cint
    lib.oracle_brgemm.argtypes = [cint, cint, cint, i64, i64, i64, i64,
                                  vp, vp, i64, vp, vp, i64,
                                  ctypes.c_float, vp, cint, i64,
                                  vp, cint, vp, i64, vp]
    lib.oracle_round_to_out.restype = None
    lib.oracle_round_to_out.argtypes = [vp, i64, cint, vp]
    lib.oracle_f64_to_bf16.restype = ctypes.c_uint16
    lib.oracle_f64_to_bf16.argtypes = [ctypes.c_double]
    lib.oracle_bf16_to_f64.restype = ctypes.c_double
    lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_f64_to_f16.restype = ctypes.c_uint16
    lib.oracle_f64_to_f16.argtypes = [ctypes.c_double]
    lib.oracle_f16_to_f64.restype = ctypes.c_double
    lib.oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_num_threads.restype = cint
    lib.oracle_num_threads.argtypes = []
    lib.oracle_f8e4m3_to_f64.restype = ctypes.c_double
    lib.oracle_f8e4m3_to_f64.argtypes = [ctypes.c_uint8]
    lib.oracle_f8e4m3_widen.restype = None
    lib.oracle_f8e4m3_widen.argtypes = [vp, i64, vp]
    lib.oracle_f8e5m2_to_f64.restype = ctypes.c_double
    lib.oracle_f8e5m2_to_f64.argtypes = [ctypes.c_uint8]
    lib.oracle_f8e5m2_widen.restype = None
    lib.oracle_f8e5m2_widen.argtypes = [vp, i64, vp]
    lib.oracle_gemm_s8.restype = cint
    lib.oracle_gemm_s8.argtypes = [cint, cint, i64, i64, i64, vp, i64, vp, i64, cint, vp, i64, vp]
    lib.oracle_pack_vnni.restype = cint
    lib.oracle_pack_vnni.argtypes = [cint, cint, i64, i64, vp, i64, i64, i64, vp]
    _lib = lib
    return lib


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"oracle takes float32, uint16 (bf16 bits) or float16, got {a.dtype}")


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def num_threads():
    return int(_load().oracle_num_threads())


def brgemm_ref(A_base, A_off, lda, B_base, B_off, ldb, M, N, K, *,
               transA=0, transB=0, beta=0.0, C0=None, ldc0=None,
               bias=None, relu=False, rows=None):
    """fp64 reference of C = beta*C0 + sum_i A_i x B_i (optionally + bias, ReLU).

    A_base/B_base: flat (or any-shape, C-contiguous) arrays; tile i starts at
    element A_off[i] / B_off[i].  rows: optional list of row indices of C to
    compute (result is len(rows) x N); default all M rows.
    """
    lib = _load()
    A_base = np.ascontiguousarray(A_base)
    B_base = np.ascontiguousarray(B_base)
    dt = _dtype_code(A_base)
    if _dtype_code(B_base) != dt:
        raise TypeError("A and B must have the same element type")
    A_off = np.ascontiguousarray(np.asarray(A_off, dtype=np.int64))
    B_off = np.ascontiguousarray(np.asarray(B_off, dtype=np.int64))
    batch = int(A_off.shape[0])
    if B_off.shape[0] != batch:
        raise ValueError("A_off and B_off differ in length")
    # Host-side bounds check so a wrong offset fails here, not in C.
    if batch and M and N and K:
        a_span = ((K - 1) * lda + M) if transA else ((M - 1) * lda + K)
        b_span = ((N - 1) * ldb + K) if transB else ((K - 1) * ldb + N)
        if A_off.min() < 0 or A_off.max() + a_span > A_base.size:
            raise ValueError("A tile out of bounds")
        if B_off.min() < 0 or B_off.max() + b_span > B_base.size:
            raise ValueError("B tile out of bounds")
    c0_dt = F32
    if beta != 0.0:
        if C0 is None:
            raise ValueError("beta != 0 needs C0")
        C0 = np.ascontiguousarray(C0)
        c0_dt = _dtype_code(C0)
        if ldc0 is None:
            ldc0 = N
        if M and N and (M - 1) * ldc0 + N > C0.size:
            raise ValueError("C0 out of bounds")
    else:
        C0, ldc0 = None, 0
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.size != N:
            raise ValueError("bias must have N entries")
    rows_arr = None
    R = M
    if rows is not None:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        R = int(rows_arr.shape[0])
    ref = np.empty((R, N), dtype=np.float64)
    rc = lib.oracle_brgemm(dt, int(transA), int(transB), M, N, K, batch,
                           _ptr(A_base), _ptr(A_off), lda,
                           _ptr(B_base), _ptr(B_off), ldb,
                           ctypes.c_float(beta), _ptr(C0), c0_dt, int(ldc0),
                           _ptr(bias), int(bool(relu)),
                           _ptr(rows_arr), R, _ptr(ref))
    if rc != 0:
        raise ValueError("oracle_brgemm rejected its arguments")
    return ref


def gemm_ref(A, lda, B, ldb, M, N, K, **kw):
    """fp64 reference of C = beta*C0 + A x B: the batch == 1 case (Section 5(d))."""
    return brgemm_ref(A, [0], lda, B, [0], ldb, M, N, K, **kw)


def round_to_out(ref, out_dtype):
    """Round an fp64 result once to the library's output type (F32 or BF16 bits)."""
    lib = _load()
    ref = np.ascontiguousarray(ref, dtype=np.float64)
    out = np.empty(ref.shape, dtype={BF16: np.uint16, F16: np.float16}.get(out_dtype, np.float32))
    lib.oracle_round_to_out(_ptr(ref), ref.size, out_dtype, _ptr(out))
    return out


def f64_to_bf16(x):
    return int(_load().oracle_f64_to_bf16(float(x)))


def f64_to_f16(x):
    """fp64 -> binary16 bit pattern, round-to-nearest-even (the oracle's own rounding)."""
    return int(_load().oracle_f64_to_f16(float(x)))


def f16_to_f64(bits):
    """Exact widening of one binary16 bit pattern to fp64 (the oracle's own decoder)."""
    return float(_load().oracle_f16_to_f64(int(bits)))


def bf16_to_f64(bits):
    """Exact widening of bf16 bit patterns (scalar or array) to fp64."""
    if np.isscalar(bits):
        return float(_load().oracle_bf16_to_f64(int(bits)))
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def pack_vnni(B, ldb, K, N, v, *, transB=0, k_rows=None, n_pitch=None):
    """VNNI packing (Section 2.2, Figure 1) of a K x N matrix of 16-bit patterns:
    returns an array of shape (k_rows / v, n_pitch, v), zero outside B."""
    B = np.ascontiguousarray(B, dtype=np.uint16)
    k_rows = K + (-K) % v if k_rows is None else k_rows
    n_pitch = N if n_pitch is None else n_pitch
    out = np.empty((k_rows // v, n_pitch, v), dtype=np.uint16)
    rc = _load().oracle_pack_vnni(v, int(transB), K, N, _ptr(B), ldb, k_rows, n_pitch, _ptr(out))
    if rc != 0:
        raise ValueError("oracle_pack_vnni rejected its arguments")
    return out


def gemm_s8_ref(A, lda, B, ldb, M, N, K, *, transA=0, transB=0, C0=None, ldc0=None):
    """Exact int64 reference of the int8 product (plus an int32 C0 when given)."""
    A = np.ascontiguousarray(A, dtype=np.int8)
    B = np.ascontiguousarray(B, dtype=np.int8)
    if M and K and ((K - 1) * lda + M if transA else (M - 1) * lda + K) > A.size:
        raise ValueError("A out of bounds")
    if N and K and ((N - 1) * ldb + K if transB else (K - 1) * ldb + N) > B.size:
        raise ValueError("B out of bounds")
    acc = C0 is not None
    if acc:
        C0 = np.ascontiguousarray(C0, dtype=np.int32)
        ldc0 = N if ldc0 is None else ldc0
        if M and N and (M - 1) * ldc0 + N > C0.size:
            raise ValueError("C0 out of bounds")
    out = np.empty((M, N), dtype=np.int64)
    rc = _load().oracle_gemm_s8(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, int(acc),
                                _ptr(C0) if acc else ctypes.c_void_p(0), int(ldc0 or 0), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_gemm_s8 rejected its arguments")
    return out


def f8e4m3_to_f64(byte):
    """Exact value of one FP8 E4M3 pattern."""
    return float(_load().oracle_f8e4m3_to_f64(int(byte)))


def f8e4m3_widen(a):
    """uint8 array of E4M3 patterns -> float32 array of the same shape (exact)."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    out = np.empty(a.shape, dtype=np.float32)
    _load().oracle_f8e4m3_widen(_ptr(a), a.size, _ptr(out))
    return out


def f8e5m2_to_f64(byte):
    """Exact value of one FP8 E5M2 pattern."""
    return float(_load().oracle_f8e5m2_to_f64(int(byte)))


def f8e5m2_widen(a):
    """uint8 array of E5M2 patterns -> float32 array of the same shape (exact)."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    out = np.empty(a.shape, dtype=np.float32)
    _load().oracle_f8e5m2_widen(_ptr(a), a.size, _ptr(out))
    return out
