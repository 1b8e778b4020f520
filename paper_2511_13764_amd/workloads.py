"""Seeded synthetic inputs for the GEMM / BRGEMM workloads.

This module produces INPUTS only (host numpy arrays) and holds none of the
method's arithmetic; both the GPU tests and the CPU checker are fed from here
so that they see identical bits.  It imports neither of them.

The paper's evaluation (Section 6, "Output Verification") initialises A, B and C
from a fixed random seed; these generators stand in for that: uniform[-1,1]
for the fp32 cases, N(0,1) activations and N(0,0.02) weights rounded to bf16
for the bf16 cases, and a 64 MiB pool holding scattered tiles for the
batch-reduce case (Section 2.1: source tiles need not be contiguous).

bf16 values are carried as numpy uint16 bit patterns.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 20251113


def _rng(config_index: int, tensor_index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + config_index * 100 + tensor_index))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16) using the library conversion of torch."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def uniform_f32(config_index, tensor_index, shape):
    return _rng(config_index, tensor_index).uniform(-1.0, 1.0, size=shape).astype(np.float32)


def normal_f32(config_index, tensor_index, shape, sigma=1.0):
    g = _rng(config_index, tensor_index).standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        g = g * np.float32(sigma)
    return g


def normal_bf16(config_index, tensor_index, shape, sigma=1.0):
    return to_bf16_bits(normal_f32(config_index, tensor_index, shape, sigma))


@dataclass
class GemmCase:
    """One GEMM problem: logical C[M,N] = beta*C0 + A[M,K] x B[K,N]."""
    name: str
    dtype: str                  # "f32" or "bf16" (element type of A and B)
    M: int
    N: int
    K: int
    transA: int
    transB: int
    beta: float
    A: np.ndarray               # stored operand (2-D, row-major)
    B: np.ndarray
    C0: Optional[np.ndarray]    # old C (same type as the output) or None
    c_is_f32: bool = True
    lda: int = 0
    ldb: int = 0
    ldc: int = 0

    def __post_init__(self):
        self.lda = self.lda or self.A.shape[1]
        self.ldb = self.ldb or self.B.shape[1]
        self.ldc = self.ldc or self.N

    @property
    def flops(self):
        return 2.0 * self.M * self.N * self.K


def _stored(shape_logical, trans):
    r, c = shape_logical
    return (c, r) if trans else (r, c)


def config1_f32_256():
    """fp32 C = A x B, M=N=K=256, uniform[-1,1], beta = 0."""
    M = N = K = 256
    A = uniform_f32(1, 0, (M, K))
    B = uniform_f32(1, 1, (K, N))
    return GemmCase("f32_256", "f32", M, N, K, 0, 0, 0.0, A, B, None, True)


def config2_f32_2048(size=2048):
    """fp32 C = A x B + 0.5 C, M=N=K=2048, A, B and the old C uniform[-1,1]."""
    M = N = K = size
    A = uniform_f32(2, 0, (M, K))
    B = uniform_f32(2, 1, (K, N))
    C0 = uniform_f32(2, 2, (M, N))
    return GemmCase(f"f32_{size}_beta0.5", "f32", M, N, K, 0, 0, 0.5, A, B, C0, True)


def config3_bf16_square(size):
    """bf16 in / fp32 accumulate / bf16 out, M=N=K=size, N(0,1), beta = 0, row-major."""
    M = N = K = size
    idx = {1024: 0, 2048: 1, 4096: 2, 8192: 3}.get(size, 9)
    A = normal_bf16(3, 10 * idx + 0, (M, K))
    B = normal_bf16(3, 10 * idx + 1, (K, N))
    return GemmCase(f"bf16_{size}", "bf16", M, N, K, 0, 0, 0.0, A, B, None, False)


def config4_mlp(M, which):
    """Transformer-MLP layer, bf16, weights stored transposed (N x K, "NT").

    which = "up":   K=4096,  N=11008;   which = "down": K=11008, N=4096.
    Activations N(0,1), weights N(0,0.02), both rounded to bf16; bf16 output.
    """
    K, N = (4096, 11008) if which == "up" else (11008, 4096)
    t = {"up": 0, "down": 1}[which]
    A = normal_bf16(4, 10 * t + 0, (M, K))
    W = normal_bf16(4, 10 * t + 1, (N, K), sigma=0.02)
    return GemmCase(f"mlp_{which}_M{M}", "bf16", M, N, K, 0, 1, 0.0, A, W, None, False)


@dataclass
class BrgemmCase:
    """Batch-reduce problem: C[M,N] (fp32) = beta*C0 + sum_i A_i[M,K] x B_i[K,N]."""
    name: str
    M: int
    N: int
    K: int
    batch: int
    transA: int
    transB: int
    beta: float
    pool: np.ndarray            # uint16 bf16 bits; both A_base and B_base
    A_off: np.ndarray           # int64 element offsets into pool
    B_off: np.ndarray
    lda: int
    ldb: int
    C0: Optional[np.ndarray]
    ldc: int = 0
    canary: bool = True

    def __post_init__(self):
        self.ldc = self.ldc or self.N

    @property
    def flops(self):
        return 2.0 * self.M * self.N * self.K * self.batch


BF16_NAN = np.uint16(0x7FC0)


def config5_brgemm(M=512, N=512, K=64, batch=64, pool_elems=32 * 1024 * 1024, beta=1.0,
                   config_index=5):
    """C[512,512] fp32 += sum_{i<64} A_i[512,64] x B_i[64,512] over scattered tiles.

    One 64 MiB bf16 pool.  Every A_i (dense, lda = K) and B_i (dense, ldb = N)
    sits in its own slot; slots are picked by a seeded permutation, and inside
    its slot a tile starts at a seeded jitter that is a multiple of 64 elements
    (128 bytes), so tiles never overlap, never touch, and are not in batch
    order.  Everything between the tiles is bf16 NaN: a stray read poisons C.
    Initial C is zero and beta = 1 (accumulate form).
    """
    rng = _rng(config_index, 0)
    tile_a, tile_b = M * K, K * N
    tile = max(tile_a, tile_b)
    n_tiles = 2 * batch
    slot = pool_elems // (4 * n_tiles) if pool_elems // (4 * n_tiles) >= 2 * tile else 2 * tile
    n_slots = pool_elems // slot
    assert n_slots >= n_tiles, "pool too small for the requested tiles"
    pool = np.full(pool_elems, BF16_NAN, dtype=np.uint16)
    slots = rng.permutation(n_slots)[:n_tiles]
    max_jit = (slot - tile) // 64 - 1          # leave >= 64 elements before the next slot
    jitter = rng.integers(1, max(2, max_jit), size=n_tiles) * 64
    starts = slots.astype(np.int64) * slot + jitter
    A_off, B_off = starts[:batch].copy(), starts[batch:].copy()
    vals = _rng(config_index, 1)
    for i in range(batch):
        a = to_bf16_bits(vals.standard_normal(size=tile_a, dtype=np.float32))
        b = to_bf16_bits(vals.standard_normal(size=tile_b, dtype=np.float32))
        pool[A_off[i]:A_off[i] + tile_a] = a
        pool[B_off[i]:B_off[i] + tile_b] = b
    C0 = np.zeros((M, N), dtype=np.float32) if beta != 0.0 else None
    return BrgemmCase(f"brgemm_{M}x{N}x{K}x{batch}", M, N, K, batch, 0, 0, beta,
                      pool, A_off, B_off, K, N, C0)


def small_int_matrix(seed, shape, lo=-4, hi=4, dtype="f32"):
    """Integer-valued entries in [lo, hi]: exact in bf16 and fp32, so any order of
    summation gives the same fp32 result while K * hi^2 stays below 2^24."""
    g = np.random.Generator(np.random.PCG64(seed)).integers(lo, hi + 1, size=shape)
    x = g.astype(np.float32)
    return to_bf16_bits(x) if dtype == "bf16" else x
