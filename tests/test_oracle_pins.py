"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- a hand-worked fixture, library routines on special cases
where BCR degenerates to a textbook product, an independent brute-force loop
nest, exactness on integer data, and the counting facts the paper states."""
import math

import numpy as np
import pytest
import scipy.sparse as sp

import bcr_inputs as gen
from oracle import bcr_oracle as orc
from oracle import pack_ref
from conftest import read_golden


def _ints(s):
    return [int(t) for t in s.split()]


def _sets(s):
    return [[int(t) for t in part.split()] for part in s.split("|")]


def _brute_force(W64, X64, mask):
    """Independent formulation: loop over blocks, kept rows, kept columns and
    accumulate into Y (a different loop nest from the oracle's mask-then-GEMM)."""
    M, K = W64.shape
    N = X64.shape[1]
    Y = np.zeros((M, N))
    nbc = K // mask.BC
    for b in range(mask.nb):
        s, c = divmod(b, nbc)
        for i in mask.rows_of(b):
            for j in mask.cols_of(b):
                r, k = s * mask.BR + int(i), c * mask.BC + int(j)
                for n in range(N):
                    Y[r, n] += W64[r, k] * X64[k, n]
    return Y


# ---------------------------------------------------------------- hand-worked
def test_hand_worked_fixture_mask_product_and_arrays():
    g = read_golden("tiny_bcr_case.txt")
    M, K, N, BR, BC = (int(g[k]) for k in ("M", "K", "N", "BR", "BC"))
    W = np.array(_ints(g["W"]), dtype=np.float64).reshape(M, K)
    X = np.array(_ints(g["X"]), dtype=np.float64).reshape(K, N)
    mask = gen.mask_from_sets(M, K, BR, BC, _sets(g["rows"]), _sets(g["cols"]))
    Wm = orc.masked_dense(W, BR, BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx)
    assert np.array_equal(Wm, np.array(_ints(g["W_bcr"]), dtype=np.float64).reshape(M, K))
    Y, S = orc.bcr_product(W, X, mask)
    assert np.array_equal(Y, np.array(_ints(g["Y"]), dtype=np.float64).reshape(M, N))
    assert np.array_equal(S, np.abs(Wm) @ np.abs(X))
    arrays = pack_ref.pack(W.astype(np.float32), mask)
    for key in ("strip_order", "row_ptr", "row_idx", "col_ptr", "col_idx", "blk_ptr"):
        assert arrays[key].tolist() == _ints(g[key]), key
    assert arrays["weights"].tolist() == [float(v) for v in _ints(g["weights"])]
    assert np.array_equal(pack_ref.unpack(arrays, M, K, BR, BC, np.float32), Wm.astype(np.float32))


# ------------------------------------------------------- library special cases
@pytest.mark.parametrize("M,K,N,BR,BC", [(12, 20, 7, 4, 5), (6, 8, 3, 6, 8), (9, 4, 5, 1, 1)])
def test_all_kept_is_dense_gemm(M, K, N, BR, BC):
    rng = np.random.default_rng(7)
    W, X = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    Y, _ = orc.bcr_product(W, X, gen.full_mask(M, K, BR, BC), skip_zero=False)
    np.testing.assert_allclose(Y, W @ X, rtol=0, atol=1e-13)


def test_single_block_is_row_column_pruned_gemm():
    # block = whole matrix: BCR degenerates to plain row/column pruning (Section 3.2)
    M, K, N = 10, 14, 6
    rng = np.random.default_rng(8)
    W, X = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    R, C = [1, 4, 5, 9], [0, 2, 3, 8, 13]
    mask = gen.mask_from_sets(M, K, M, K, [R], [C])
    Y, _ = orc.bcr_product(W, X, mask)
    expect = np.zeros((M, N))
    expect[R] = W[np.ix_(R, C)] @ X[C]
    np.testing.assert_allclose(Y, expect, rtol=0, atol=1e-13)


def test_unit_blocks_are_unstructured_sparsity_csr():
    # 1x1 blocks: BCR degenerates to non-structured pruning (Section 3.2)
    M, K, N = 17, 23, 5
    rng = np.random.default_rng(9)
    W, X = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    keep = rng.random((M, K)) < 0.3
    rows = [[0] if keep.flat[b] else [] for b in range(M * K)]
    cols = [[0] if keep.flat[b] else [] for b in range(M * K)]
    mask = gen.mask_from_sets(M, K, 1, 1, rows, cols)
    Y, _ = orc.bcr_product(W, X, mask)
    np.testing.assert_allclose(Y, sp.csr_matrix(W * keep) @ X, rtol=0, atol=1e-13)


def test_nothing_kept_gives_zero():
    M, K, N = 8, 12, 4
    W, X = np.ones((M, K)), np.ones((K, N))
    for kr, kc in ((0, 3), (2, 0), (0, 0)):
        Y, S = orc.bcr_product(W, X, gen.random_mask(M, K, 4, 6, kr, kc, seed=3))
        assert not Y.any() and not S.any()


# ------------------------------------------------------------------ brute force
@pytest.mark.parametrize("M,K,N,BR,BC,kr,kc", [
    (8, 12, 3, 4, 6, 2, 3), (12, 8, 5, 3, 4, (0, 1, 3), (1, 2, 4)), (16, 32, 2, 16, 16, 4, 8)])
def test_brute_force_per_block_loops(M, K, N, BR, BC, kr, kc):
    rng = np.random.default_rng(10)
    W, X = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=11)
    Y, _ = orc.bcr_product(W, X, mask)
    np.testing.assert_allclose(Y, _brute_force(W, X, mask), rtol=0, atol=1e-13)


def test_integer_data_exact_and_invariants():
    M, K, N, BR, BC = 32, 48, 9, 8, 16
    mask = gen.random_mask(M, K, BR, BC, (2, 4, 8), (4, 8), seed=12)
    W = gen.storage_to_f64(gen.small_int_values((M, K), gen.F32, 1), gen.F32)
    X1 = gen.storage_to_f64(gen.small_int_values((K, N), gen.F32, 2), gen.F32)
    X2 = gen.storage_to_f64(gen.small_int_values((K, N), gen.F32, 3), gen.F32)
    Y1, _ = orc.bcr_product(W, X1, mask)
    Y2, _ = orc.bcr_product(W, X2, mask)
    Y12, _ = orc.bcr_product(W, X1 + X2, mask)
    assert np.array_equal(Y1, _brute_force(W, X1, mask))          # exact, bit for bit
    assert np.array_equal(Y12, Y1 + Y2)                           # linear in X
    perm = np.random.default_rng(4).permutation(N)
    Yp, _ = orc.bcr_product(W, X1[:, perm], mask)
    assert np.array_equal(Yp, Y1[:, perm])                        # columns are independent
    # the sampled form returns the same entries
    rows, cols = np.array([3, 17, 30]), np.array([0, 8])
    Ys, _ = orc.bcr_product(W, X1, mask, rows=rows, cols=cols)
    assert np.array_equal(Ys, Y1[np.ix_(rows, cols)])
    # skipping stored zeros changes nothing
    Yn, _ = orc.bcr_product(W, X1, mask, skip_zero=False)
    assert np.array_equal(Yn, Y1)


def test_mask_orientation_rows_are_outputs():
    # A block "a x b" has a rows (outputs) and b columns (inputs): Section 3.2
    # counts 64 blocks and 1024 prunable block-columns for a 64x64 layer cut 4x16.
    mask = gen.full_mask(64, 64, 4, 16)
    assert mask.nb == 64 and int(mask.kc().sum()) == 1024 and int(mask.kr().sum()) == 256
    # pruning a column of one block zeroes a K index (input) for that strip only
    M, K = 8, 32
    rows = [[0, 1, 2, 3]] * 4
    cols = [list(range(16))] * 4
    cols[1] = [j for j in range(16) if j != 5]        # block (strip 0, column block 1)
    Wm = orc.masked_dense(np.ones((M, K)), 4, 16, *_arrs(gen.mask_from_sets(M, K, 4, 16, rows, cols)))
    expect = np.ones((M, K))
    expect[0:4, 16 + 5] = 0
    assert np.array_equal(Wm, expect)


def _arrs(mask):
    return mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx


# --------------------------------------------------------------- counting facts
def test_survivor_count_closed_form_section_3_2():
    # 1024 x 1024, 64 blocks, 8x pruning rate -> 2,048 survivors per block
    mask = gen.random_mask(1024, 1024, 128, 128, 64, 32, seed=13)
    assert mask.nb == 64
    per_block = mask.kr() * mask.kc()
    assert (per_block == 2048).all() and mask.nnz() == 1024 * 1024 // 8
    W = np.ones((1024, 1024))
    Wm = orc.masked_dense(W, 128, 128, *_arrs(mask))
    assert int(Wm.sum()) == mask.nnz()
    blocks = Wm.reshape(8, 128, 8, 128).sum(axis=(1, 3))
    assert (blocks == 2048).all()


@pytest.mark.parametrize("name,nnz", [("c1", 8192), ("c2", 73728), ("c3", 786432)])
def test_named_workloads_have_prescribed_rates(name, nnz):
    wl = {"c1": gen.c1_single_fp32, "c2": lambda: gen.c2_vgg_conv(N=8),
          "c3": gen.c3_lstm_gates}[name]()
    assert wl.mask.nnz() == nnz
    Wm = orc.masked_dense(gen.storage_to_f64(wl.W, wl.dtype), wl.mask.BR, wl.mask.BC, *_arrs(wl.mask))
    assert int(np.count_nonzero(Wm)) == nnz            # generator redraws values that round to 0
    for b in (0, wl.mask.nb // 2, wl.mask.nb - 1):
        r, c = wl.mask.rows_of(b), wl.mask.cols_of(b)
        assert (np.diff(r.astype(int)) > 0).all() and (np.diff(c.astype(int)) > 0).all()
        assert r.max() < wl.mask.BR and c.max() < wl.mask.BC


def test_c5_block_densities_span_1_64_to_1_4():
    mask = gen.random_mask(512, 4608, 32, 32, (4, 8, 16), (4, 8, 16), seed=5)
    d = (mask.kr() * mask.kc()) / 1024.0
    assert set(np.unique(mask.kr())) == {4, 8, 16} and set(np.unique(mask.kc())) == {4, 8, 16}
    assert math.isclose(d.min(), 1 / 64) and math.isclose(d.max(), 1 / 4)
    assert abs(d.mean() - (28 / 96) ** 2) < 0.01        # E[frac]^2 = (7/24)^2 = 0.0851


# ------------------------------------------------------- compact-format reference
@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
def test_pack_ref_roundtrip_and_order(dtype):
    M, K, BR, BC = 64, 96, 16, 32
    mask = gen.random_mask(M, K, BR, BC, (0, 4, 8, 16), (0, 8, 32), seed=14)
    W = gen.normal_weights(M, K, dtype, seed=15)
    a = pack_ref.pack(W, mask)
    assert a["weights"].shape[0] == mask.nnz() == int(a["blk_ptr"][-1])
    Wm64 = orc.masked_dense(gen.storage_to_f64(W, dtype), BR, BC, *_arrs(mask))
    back = pack_ref.unpack(a, M, K, BR, BC, W.dtype)
    assert np.array_equal(gen.storage_to_f64(back, dtype), Wm64)
    assert back.tobytes() == np.where(Wm64 != 0, W, np.zeros_like(W)).tobytes()
    work = pack_ref.strip_work(mask)
    order = a["strip_order"]
    assert sorted(order.tolist()) == list(range(M // BR))
    assert (np.diff(work[order]) <= 0).all()                 # regular work after reorder (Fig. 11)
    ties = np.diff(work[order]) == 0
    assert (np.diff(order)[ties] > 0).all()                  # stable
    # idempotence: packing the unpacked matrix gives the same arrays
    b = pack_ref.pack(back, mask)
    assert all(np.array_equal(a[k], b[k]) for k in a)


def test_storage_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-5, 65504.0, 1e-40], dtype=np.float32)
    bits = gen.f32_to_bf16_bits(x)
    back = gen.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie -> rounds to even (1.0); 1 + 3*2^-8 is a tie -> rounds up to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert back[3] == -2.5
    assert abs(back[4] - 3.0e-5) <= 3.0e-5 * 2.0 ** -8
    assert gen.storage_to_f64(x.astype(np.float16), gen.F16)[5] == 65504.0
