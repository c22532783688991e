"""Seeded synthetic inputs for BCR (Block-based Column-Row) sparse products.

This module only *draws inputs*: per-block kept-row / kept-column index sets,
weight and activation values, and the one-time rounding of those values to the
storage type.  It holds none of the method's arithmetic (no masking, packing or
multiplication), so both the CPU oracle's tests and the GPU library's tests can
feed from it without sharing any code of the method itself.

The paper evaluates block sizes on layers whose weights are drawn at random to
satisfy a pruning rate and a block size (Section "Block size optimization",
Listing 1, ``synthesize``), arguing that latency depends on the rate and not on
where the survivors sit.  The generators here follow that recipe: every block
keeps a uniform random subset of its rows and of its columns, independently.

Block convention (Section 3.2, search-space example: 64x64 layer, 4x16 blocks,
column pruning only -> 1024 prunable block-columns): a block of size ``BR x BC``
has BR rows (outputs / filters) and BC columns (inputs).  Blocks are numbered
row-major, ``b = s * nbc + c`` for row strip ``s`` and column block ``c``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 20210811

F32, F16, BF16 = "f32", "f16", "bf16"
DTYPES = (F32, F16, BF16)


# --------------------------------------------------------------------------
# storage types: fp32 -> fp16 / bf16 rounding (round to nearest even), and the
# exact widening back to fp64.  bf16 has no NumPy dtype; it is carried as the
# uint16 bit pattern (upper half of the fp32 encoding).
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    lsb = (u >> 16) & 1
    r = ((u + (0x7FFF + lsb)) >> 16).astype(np.uint16)
    r[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_storage(a32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array -> array in the storage type (f32: float32, f16: float16,
    bf16: uint16 bit patterns)."""
    a32 = np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == F32:
        return a32.copy()
    if dtype == F16:
        return a32.astype(np.float16)
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored values to fp64."""
    if dtype == F32:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == F16:
        return np.asarray(a, dtype=np.float16).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_numpy_dtype(dtype: str):
    return {F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype]


def storage_itemsize(dtype: str) -> int:
    return 4 if dtype == F32 else 2


# --------------------------------------------------------------------------
# masks
# --------------------------------------------------------------------------
@dataclass
class BcrMask:
    """Per-block kept-row and kept-column index sets in CSR-like form.

    ``row_idx[row_ptr[b]:row_ptr[b+1]]`` are the kept rows of block ``b``
    (local to the block, strictly ascending, uint16); likewise for columns.
    """
    M: int
    K: int
    BR: int
    BC: int
    row_ptr: np.ndarray
    row_idx: np.ndarray
    col_ptr: np.ndarray
    col_idx: np.ndarray

    @property
    def nbr(self) -> int:
        return self.M // self.BR

    @property
    def nbc(self) -> int:
        return self.K // self.BC

    @property
    def nb(self) -> int:
        return self.nbr * self.nbc

    def kr(self) -> np.ndarray:
        return np.diff(self.row_ptr).astype(np.int64)

    def kc(self) -> np.ndarray:
        return np.diff(self.col_ptr).astype(np.int64)

    def nnz(self) -> int:
        """Structural survivor count, sum over blocks of kept rows x kept columns."""
        return int((self.kr() * self.kc()).sum())

    def rows_of(self, b: int) -> np.ndarray:
        return self.row_idx[self.row_ptr[b]:self.row_ptr[b + 1]]

    def cols_of(self, b: int) -> np.ndarray:
        return self.col_idx[self.col_ptr[b]:self.col_ptr[b + 1]]


def _subsets(rng: np.random.Generator, counts: np.ndarray, size: int) -> Tuple[np.ndarray, np.ndarray]:
    """For every block draw ``counts[b]`` of ``size`` local indices uniformly
    without replacement; return (ptr int32, idx uint16 ascending per block)."""
    nb = counts.shape[0]
    order = np.argsort(rng.random((nb, size)), axis=1, kind="stable")
    rank = np.empty_like(order)
    np.put_along_axis(rank, order, np.broadcast_to(np.arange(size), (nb, size)).copy(), axis=1)
    keep = rank < counts[:, None]                     # [nb, size], True at kept local indices
    ptr = np.zeros(nb + 1, dtype=np.int32)
    np.cumsum(counts, out=ptr[1:])
    idx = np.nonzero(keep)[1].astype(np.uint16)       # row-major nonzero -> ascending per block
    return ptr, idx


def random_mask(M: int, K: int, BR: int, BC: int,
                kr, kc, seed: int, stream: int = 0) -> BcrMask:
    """Uniform random BCR mask.  ``kr`` / ``kc`` are either an int (same count
    in every block), or a sequence of candidate counts from which each block
    draws independently and uniformly."""
    if M % BR or K % BC:
        raise ValueError("block size must divide the matrix")
    nb = (M // BR) * (K // BC)
    rng = np.random.default_rng(np.random.SeedSequence([SEED_BASE, seed, stream, 1]))

    def counts(k, size):
        if np.isscalar(k):
            if not 0 <= int(k) <= size:
                raise ValueError("kept count out of range")
            return np.full(nb, int(k), dtype=np.int64)
        choices = np.asarray(list(k), dtype=np.int64)
        return choices[rng.integers(0, len(choices), size=nb)]

    kr_b = counts(kr, BR)
    kc_b = counts(kc, BC)
    row_ptr, row_idx = _subsets(rng, kr_b, BR)
    col_ptr, col_idx = _subsets(rng, kc_b, BC)
    return BcrMask(M, K, BR, BC, row_ptr, row_idx, col_ptr, col_idx)


def full_mask(M: int, K: int, BR: int, BC: int) -> BcrMask:
    """Every row and column of every block kept (a dense layer)."""
    nb = (M // BR) * (K // BC)
    row_ptr = (np.arange(nb + 1) * BR).astype(np.int32)
    col_ptr = (np.arange(nb + 1) * BC).astype(np.int32)
    row_idx = np.tile(np.arange(BR, dtype=np.uint16), nb)
    col_idx = np.tile(np.arange(BC, dtype=np.uint16), nb)
    return BcrMask(M, K, BR, BC, row_ptr, row_idx, col_ptr, col_idx)


def mask_from_sets(M: int, K: int, BR: int, BC: int,
                   rows: Sequence[Sequence[int]], cols: Sequence[Sequence[int]]) -> BcrMask:
    """Build a mask from explicit per-block lists (used by hand-made test cases)."""
    nb = (M // BR) * (K // BC)
    assert len(rows) == nb and len(cols) == nb
    row_ptr = np.zeros(nb + 1, dtype=np.int32)
    col_ptr = np.zeros(nb + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(r) for r in rows])
    col_ptr[1:] = np.cumsum([len(c) for c in cols])
    row_idx = np.array([i for r in rows for i in r], dtype=np.uint16)
    col_idx = np.array([j for c in cols for j in c], dtype=np.uint16)
    return BcrMask(M, K, BR, BC, row_ptr, row_idx, col_ptr, col_idx)


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------
def normal_weights(M: int, K: int, dtype: str, seed: int, stream: int = 0,
                   sigma: float = 0.02) -> np.ndarray:
    """Dense M x K weights ~ N(0, sigma), drawn in fp32 and rounded once to the
    storage type.  Any value that rounds to +-0 is redrawn, so that the count
    of nonzero survivors equals the structural count."""
    rng = np.random.default_rng(np.random.SeedSequence([SEED_BASE, seed, stream, 2]))
    w = (rng.standard_normal((M, K), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    s = round_to_storage(w, dtype)
    for _ in range(64):
        z = storage_to_f64(s, dtype) == 0.0
        n = int(z.sum())
        if n == 0:
            break
        w[z] = rng.standard_normal(n, dtype=np.float32) * np.float32(sigma)
        s = round_to_storage(w, dtype)
    return s


def normal_activations(K: int, N: int, dtype: str, seed: int, stream: int = 0,
                       relu: bool = False) -> np.ndarray:
    """Dense K x N activations ~ N(0,1) (optionally passed through ReLU, as
    the input of a conv layer that follows a ReLU is), rounded once."""
    rng = np.random.default_rng(np.random.SeedSequence([SEED_BASE, seed, stream, 3]))
    x = rng.standard_normal((K, N), dtype=np.float32)
    if relu:
        np.maximum(x, 0.0, out=x)
    return round_to_storage(x, dtype)


def small_int_values(shape, dtype: str, seed: int, stream: int = 0, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Small integers (exactly representable in every storage type); sums of
    their products are exact in fp32 and fp64, so every correct implementation
    must agree bit for bit."""
    rng = np.random.default_rng(np.random.SeedSequence([SEED_BASE, seed, stream, 4]))
    v = rng.integers(lo, hi + 1, size=shape).astype(np.float32)
    return round_to_storage(v, dtype)


# --------------------------------------------------------------------------
# the named workloads
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    dtype: str
    mask: BcrMask
    W: np.ndarray            # dense M x K in the storage type (unmasked)
    X: np.ndarray            # K x N in the storage type
    N: int
    note: str = ""

    @property
    def M(self):
        return self.mask.M

    @property
    def K(self):
        return self.mask.K

    def useful_flops(self) -> int:
        return 2 * self.mask.nnz() * self.N


def _make(name, dtype, M, K, N, BR, BC, kr, kc, seed, relu, note="", dense=False) -> Workload:
    mask = full_mask(M, K, BR, BC) if dense else random_mask(M, K, BR, BC, kr, kc, seed)
    W = normal_weights(M, K, dtype, seed)
    X = normal_activations(K, N, dtype, seed, relu=relu)
    return Workload(name, dtype, mask, W, X, N, note)


def c1_single_fp32() -> Workload:
    """256x256 fp32, 16x16 blocks, keep 4/16 rows and 8/16 columns."""
    return _make("c1", F32, 256, 256, 64, 16, 16, 4, 8, seed=1, relu=False)


def c2_vgg_conv(N: int = 3136) -> Workload:
    """VGG-style 3x3 conv, Cin=Cout=256 at 56x56, as im2col GEMM:
    M=256, K=2304, N=3136; 16x32 blocks keeping 8/16 rows, 8/32 columns."""
    return _make("c2", F16, 256, 2304, N, 16, 32, 8, 8, seed=2, relu=True)


def c3_lstm_gates(batch: int = 1) -> Workload:
    """LSTM gate matrices [W_ih | W_hh], hidden = input = 1024: 4096 x 2048,
    32x32 blocks keeping 8 rows x 12 columns (about 10.7x compression)."""
    return _make(f"c3_b{batch}", F16, 4096, 2048, batch, 32, 32, 8, 12, seed=3, relu=False)


# (M, K, N) of the 13 VGG-16 conv layers at batch 1, 224x224 input.
VGG16_LAYERS = (
    (64, 27, 50176), (64, 576, 50176),
    (128, 576, 12544), (128, 1152, 12544),
    (256, 1152, 3136), (256, 2304, 3136), (256, 2304, 3136),
    (512, 2304, 784), (512, 4608, 784), (512, 4608, 784),
    (512, 4608, 196), (512, 4608, 196), (512, 4608, 196),
)


def c4_vgg16_layer(layer: int, N: Optional[int] = None) -> Workload:
    """Layer ``layer`` (0-based) of VGG-16 as im2col BCR SpMM, fp16.  The first
    layer (K = 27) is left dense as one 16x27 block per strip; the others use
    16x32 blocks keeping 8/16 rows and 8/32 columns."""
    M, K, N0 = VGG16_LAYERS[layer]
    N = N0 if N is None else N
    if layer == 0:
        return _make(f"c4_L{layer + 1}", F16, M, K, N, 16, 27, 16, 27, seed=40 + layer,
                     relu=False, dense=True)
    return _make(f"c4_L{layer + 1}", F16, M, K, N, 16, 32, 8, 8, seed=40 + layer, relu=True)


def c5_nonuniform(N: int = 25088) -> Workload:
    """512 x 4608 bf16, 32x32 blocks; each block's kept-row and kept-column
    fractions are drawn independently from {1/8, 1/4, 1/2}."""
    return _make("c5", BF16, 512, 4608, N, 32, 32, (4, 8, 16), (4, 8, 16), seed=5, relu=True)
