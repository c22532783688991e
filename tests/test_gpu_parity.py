"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Structures must match bit for bit; values within 1e-5 (fp32) or
2e-3 (fp16 / bf16 inputs, fp32 accumulation), measured against the sum of |terms| and
against max|Y|."""
import numpy as np
import pytest

import bcr_inputs as gen
from oracle import pack_ref
from helpers import (assert_close, oracle_product, pack_workload, run_spmm, run_spmv, to_device, torch_dev)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2108_11033_amd as lib
    lib.load_library()
    return lib


def _check_structure(A, wl):
    ref = pack_ref.pack(wl.W, wl.mask)
    got = A.arrays()
    for k in ref:
        assert got[k].tobytes() == ref[k].tobytes(), k
    assert A.unpack().tobytes() == pack_ref.unpack(ref, wl.M, wl.K, wl.mask.BR, wl.mask.BC, wl.W.dtype).tobytes()


def _spmm_case(g, wl, what, structure=True, **tune):
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    if structure:
        _check_structure(A, wl)
    Y = run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N, **tune)
    Yref, S = oracle_product(wl.W, wl.X, wl.dtype, wl.mask)
    return assert_close(Y, Yref, S, wl.dtype, what)


# ------------------------------------------------------------------ the named configurations
def test_c1_fp32_single_spmm(g):
    _spmm_case(g, gen.c1_single_fp32(), "c1")


@pytest.mark.parametrize("N", [200, 3136])
def test_c2_vgg_conv_fp16(g, N):
    _spmm_case(g, gen.c2_vgg_conv(N), f"c2 N={N}")


@pytest.mark.parametrize("batch", [1, 8])
def test_c3_lstm_gates_spmv(g, batch):
    wl = gen.c3_lstm_gates(batch)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    _check_structure(A, wl)
    y = run_spmv(g, A, wl.X, wl.dtype, wl.M, batch)
    yref, S = oracle_product(wl.W, wl.X, wl.dtype, wl.mask)
    assert_close(y, yref, S, wl.dtype, f"c3 batch={batch}")
    # spmm with N <= 8 reaches the same kernel and the same bits
    y2 = run_spmm(g, A, wl.X, wl.dtype, wl.M, batch)
    assert y2.tobytes() == y.tobytes()
    if batch == 8:
        # 8 columns of this matrix run as 8 sets of workgroups of the one-column kernel (32 workgroups each: all 256 at
        # once); every column then has the bits the one-column call gives, whatever the leading dimensions
        X = to_device(wl.X, wl.dtype)
        assert g.spmm_kernel_name(A, X, 8, 8) == "bcr_spmv"
        y3 = run_spmv(g, A, wl.X, wl.dtype, wl.M, batch, ldx=12, ldy=9)
        assert y3.tobytes() == y.tobytes()
        for b in (0, 5, 7):
            y1 = run_spmv(g, A, np.ascontiguousarray(wl.X[:, b:b + 1]), wl.dtype, wl.M, 1)
            assert y1[:, 0].tobytes() == np.ascontiguousarray(y[:, b]).tobytes(), f"column {b}"
        # the same product forced onto the matrix-core kernel (what larger or non-uniform matrices take at 8 columns)
        y4 = run_spmm(g, A, wl.X, wl.dtype, wl.M, batch, kernel=3)
        assert_close(y4, yref, S, wl.dtype, "c3 batch=8 on the row-gathering kernel")


@pytest.mark.parametrize("layer", range(13))
def test_c4_vgg16_layers_fp16(g, layer):
    # the large-N layers are cut to a few tiles plus a ragged tail; N = 784 and 196 run whole
    N0 = gen.VGG16_LAYERS[layer][2]
    N = N0 if N0 <= 784 else 328
    _spmm_case(g, gen.c4_vgg16_layer(layer, N), f"c4 L{layer + 1} N={N}", structure=layer < 3)


def test_c5_nonuniform_bf16_small_n(g):
    _spmm_case(g, gen.c5_nonuniform(N=300), "c5 N=300")


def _full_size_sampled(g, wl, what, rows_per_strip=3, seed=55, **tune):
    """A configuration at its full size, in the launch form grim_bcr_spmm picks for it (the one bench.py times): the
    oracle computes a sample of rows -- a few in EVERY row strip -- times a sample of columns: the first and last 70
    (first, last and ragged tiles), 40 on either side of every multiple of 4096 (where the launches that cut a product
    into whole rounds of workgroups plus a remainder put their cut, and where rounds of workgroups meet) and 200 drawn
    at random."""
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    Y = run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N, **tune)
    rng = np.random.default_rng(seed)
    BR = wl.mask.BR
    rows = np.sort(np.concatenate([s * BR + rng.choice(BR, min(BR, rows_per_strip), replace=False)
                                   for s in range(wl.M // BR)]))
    cuts = np.arange(4096, wl.N, 4096)
    near = np.concatenate([np.arange(c - 40, c + 40) for c in cuts]) if len(cuts) else np.zeros(0, dtype=np.int64)
    cols = np.unique(np.concatenate([np.arange(0, 70), np.arange(wl.N - 70, wl.N), near,
                                     rng.choice(wl.N, 200, replace=False)]).astype(np.int64))
    Yref, S = oracle_product(wl.W, wl.X, wl.dtype, wl.mask, rows=rows, cols=cols)
    assert_close(Y[np.ix_(rows, cols)], Yref, S, wl.dtype, what)
    assert np.isfinite(Y).all()
    return A, Y


def test_c5_full_size_sampled(g):
    _full_size_sampled(g, gen.c5_nonuniform(), "c5 full size, sampled")


@pytest.mark.parametrize("layer", range(7))
def test_c4_large_layers_full_size_sampled(g, layer):
    # layers 1-7 (N = 50176, 12544 and 3136) on the layers' own matrices, the dense 16 x 27 first layer included
    wl = gen.c4_vgg16_layer(layer)
    _full_size_sampled(g, wl, f"c4 L{layer + 1} full size N={wl.N}, sampled", seed=60 + layer)


def test_c2_at_224x224_full_size_sampled(g):
    # c2's layer at N = 50176, as bench.py times it
    wl = gen.c2_vgg_conv(50176)
    A, Y = _full_size_sampled(g, wl, "c2 at N=50176, sampled", seed=70)
    # and the whole result against one forced launch of the row-gathering kernel (another summation order:
    # closeness only)
    Yg = run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N, kernel=3)
    scale = np.abs(Yg).max()
    assert np.abs(Y - Yg).max() <= 2 * 2e-3 * scale


@pytest.mark.parametrize("ragged", [20, 21])
def test_staged_kernel_whole_rounds_and_a_remainder(g, ragged):
    """Free kernel choice at a size where the staged kernel's workgroups would leave a nearly empty last round: the
    leading columns that fill whole rounds run on the staged kernel, the rest as a product of their own (the
    row-gathering kernel when the remainder is a multiple of 4 columns, else the staged one again).  Sampled rows x the
    columns around the cut, both ends and a random sample."""
    torch, dev = torch_dev()
    wl0 = gen.c2_vgg_conv(64)
    A = pack_workload(g, wl0.W, wl0.dtype, wl0.mask)
    probe = torch.empty(16, dtype=torch.float16, device=dev)              # only the address is looked at
    tiles = next((t for t in (259, 515, 771) if g.spmm_kernel_name(A, probe, 64 * t - ragged, 64 * t - ragged) == "bcr_spmm_mma"), None)
    assert tiles is not None, "the staged kernel is never chosen for this matrix"
    N, cut = 64 * tiles - ragged, 64 * (tiles - 3)
    X = gen.normal_activations(wl0.K, N, wl0.dtype, seed=95, relu=True)
    Y = run_spmm(g, A, X, wl0.dtype, wl0.M, N)
    rng = np.random.default_rng(96)
    rows = np.sort(rng.choice(wl0.M, 40, replace=False))
    cols = np.unique(np.concatenate([np.arange(0, 70), np.arange(cut - 70, cut + 70), np.arange(N - 70, N),
                                     rng.choice(N, 200, replace=False)]))
    Yref, S = oracle_product(wl0.W, X, wl0.dtype, wl0.mask, rows=rows, cols=cols)
    assert_close(Y[np.ix_(rows, cols)], Yref, S, wl0.dtype, f"whole rounds + remainder, N={N}")
    assert np.isfinite(Y).all()


# ------------------------------------------------------------------ launch shapes and kernels
@pytest.mark.parametrize("dtype,BR", [(gen.F16, 16), (gen.BF16, 16), (gen.F16, 32), (gen.BF16, 32)])
@pytest.mark.parametrize("tile_n,strips", [(32, 4), (32, 16), (64, 4), (64, 8), (64, 16), (128, 4), (128, 8)])
def test_mma_kernel_all_tilings(g, dtype, BR, tile_n, strips):
    M, K, N = 6 * BR, 416, 333                     # 6 strips (ragged group), 13 column blocks, ragged N
    mask = gen.random_mask(M, K, BR, 32, (0, 4, 8, 16), (0, 4, 8, 12, 32), seed=70 + BR)
    W = gen.normal_weights(M, K, dtype, seed=71)
    X = gen.normal_activations(K, N, dtype, seed=72, relu=True)
    A = pack_workload(g, W, dtype, mask)
    Yref, S = oracle_product(W, X, dtype, mask)
    try:
        Y = run_spmm(g, A, X, dtype, M, N, tile_n=tile_n, strips_per_wg=strips, kernel=2)
    except g.GrimError as e:                # a shape that is not compiled, or whose staging does not fit LDS
        assert e.name == "GRIM_ERR_UNSUPPORTED"
        pytest.skip(f"launch shape tn={tile_n} strips={strips} refused for this matrix")
    assert_close(Y, Yref, S, dtype, f"mma {dtype} BR={BR} tn={tile_n} g={strips}")


@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("BR,BC", [(1, 1), (4, 16), (8, 8), (16, 16), (32, 32), (64, 48), (16, 27)])
def test_fma_kernel_block_shapes(g, dtype, BR, BC):
    M, K, N = BR * 3, BC * 5, 130
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, max(1, BR // 2), BR})),
                           tuple(sorted({0, 1, max(1, BC // 4), BC})), seed=80 + BR)
    W = gen.normal_weights(M, K, dtype, seed=81)
    X = gen.normal_activations(K, N, dtype, seed=82)
    A = pack_workload(g, W, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, kernel=1)
    Yref, S = oracle_product(W, X, dtype, mask)
    assert_close(Y, Yref, S, dtype, f"fma {dtype} {BR}x{BC}")


def test_unaligned_leading_dimensions_and_tails(g):
    for dtype, BR in ((gen.F16, 16), (gen.BF16, 32)):
        M, K = 4 * BR, 256
        mask = gen.random_mask(M, K, BR, 32, (4, 8), (8, 12), seed=90)
        W = gen.normal_weights(M, K, dtype, seed=91)
        for N, ldx, ldy in ((196, 196, 196), (67, 71, 69), (1, 1, 1), (9, 12, 9), (64, 64, 66), (130, 136, 132)):
            X = gen.normal_activations(K, N, dtype, seed=92)
            A = pack_workload(g, W, dtype, mask)
            Y = run_spmm(g, A, X, dtype, M, N, ldx=ldx, ldy=ldy, kernel=2)
            Yref, S = oracle_product(W, X, dtype, mask)
            assert_close(Y, Yref, S, dtype, f"{dtype} N={N} ldx={ldx} ldy={ldy}")


# ------------------------------------------------------------------ degenerate cases
@pytest.mark.parametrize("dtype", [gen.F32, gen.F16])
def test_degenerate_masks(g, dtype):
    M, K, N, BR, BC = 64, 128, 70, 16, 32
    W = gen.normal_weights(M, K, dtype, seed=100)
    X = gen.normal_activations(K, N, dtype, seed=101)
    cases = {
        "nothing kept": gen.random_mask(M, K, BR, BC, 0, 0, seed=1),
        "rows but no columns": gen.random_mask(M, K, BR, BC, 4, 0, seed=2),
        "columns but no rows": gen.random_mask(M, K, BR, BC, 0, 8, seed=3),
        "everything kept": gen.full_mask(M, K, BR, BC),
        "one row one column": gen.random_mask(M, K, BR, BC, 1, 1, seed=4),
        "whole-matrix block": gen.random_mask(M, K, M, K, 9, 40, seed=5),
    }
    for name, mask in cases.items():
        A = pack_workload(g, W, dtype, mask)
        Y = run_spmm(g, A, X, dtype, M, N)
        Yref, S = oracle_product(W, X, dtype, mask)
        assert_close(Y, Yref, S, dtype, name)
        for batch in (1, 3):
            if mask.BR <= 64:
                y = run_spmv(g, A, X[:, :batch].copy(), dtype, M, batch)
                assert_close(y, Yref[:, :batch], S[:, :batch], dtype, name + " spmv")


def test_integer_data_is_bit_exact_and_reproducible(g):
    # small integers: every partial sum is exact in fp32, so GPU == oracle bit for bit
    for dtype, BR, kern in ((gen.F32, 16, 0), (gen.F16, 16, 2), (gen.BF16, 32, 2), (gen.F16, 32, 1)):
        M, K, N = 4 * BR, 320, 150
        mask = gen.random_mask(M, K, BR, 32, (2, 4, 8), (4, 8, 16), seed=110)
        W = gen.small_int_values((M, K), dtype, seed=111)
        X = gen.small_int_values((K, N), dtype, seed=112)
        A = pack_workload(g, W, dtype, mask)
        Y1 = run_spmm(g, A, X, dtype, M, N, kernel=kern)
        Y2 = run_spmm(g, A, X, dtype, M, N, kernel=kern)
        Yref, _ = oracle_product(W, X, dtype, mask)
        assert np.array_equal(Y1.astype(np.float64), Yref)
        assert Y1.tobytes() == Y2.tobytes()
        y = run_spmv(g, A, X[:, :5].copy(), dtype, M, 5)
        assert np.array_equal(y.astype(np.float64), Yref[:, :5])


def test_run_to_run_bit_reproducible_random_data(g):
    wl = gen.c2_vgg_conv(N=640)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    Ys = [run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N) for _ in range(3)]
    assert Ys[0].tobytes() == Ys[1].tobytes() == Ys[2].tobytes()
    wl = gen.c3_lstm_gates(8)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    ys = [run_spmv(g, A, wl.X, wl.dtype, wl.M, 8) for _ in range(3)]
    assert ys[0].tobytes() == ys[1].tobytes() == ys[2].tobytes()


def test_fp16_subnormal_weights_are_not_flushed(g):
    # N(0, 0.02) puts ~0.24% of the weights below the smallest normal fp16; here all of them
    M, K, N, BR, BC = 32, 128, 64, 16, 32
    rng = np.random.default_rng(120)
    W = (rng.integers(1, 1000, size=(M, K)) * 2.0 ** -24 * rng.choice([-1, 1], size=(M, K))).astype(np.float16)
    X = (rng.integers(1, 64, size=(K, N)) * 16.0).astype(np.float16)
    mask = gen.random_mask(M, K, BR, BC, 8, 8, seed=121)
    A = pack_workload(g, W, gen.F16, mask)
    for kern in (1, 2):
        Y = run_spmm(g, A, X, gen.F16, M, N, kernel=kern)
        Yref, S = oracle_product(W, X, gen.F16, mask)
        assert np.abs(Yref).max() > 0
        assert_close(Y, Yref, S, gen.F16, f"subnormal kernel={kern}")
    y = run_spmv(g, A, X[:, :2].copy(), gen.F16, M, 2)
    assert_close(y, Yref[:, :2], S[:, :2], gen.F16, "subnormal spmv")


def test_no_reorder_option_gives_same_product(g):
    wl = gen.c5_nonuniform(N=96)
    A0 = pack_workload(g, wl.W, wl.dtype, wl.mask, no_reorder=True)
    A1 = pack_workload(g, wl.W, wl.dtype, wl.mask)
    assert A0.arrays()["strip_order"].tolist() == list(range(wl.M // 32))
    ref = pack_ref.pack(wl.W, wl.mask, reorder=False)
    assert all(A0.arrays()[k].tobytes() == ref[k].tobytes() for k in ref)
    Y0 = run_spmm(g, A0, wl.X, wl.dtype, wl.M, wl.N)
    Y1 = run_spmm(g, A1, wl.X, wl.dtype, wl.M, wl.N)
    assert Y0.tobytes() == Y1.tobytes()          # per-row arithmetic does not depend on strip order


# ------------------------------------------------------------------ SpMV
@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 6, 7, 8])
def test_spmv_nonuniform_all_batches(g, dtype, batch):
    M, K, BR, BC = 160, 1120, 32, 32                  # 35 column blocks: a full pass of 32 and a ragged one
    mask = gen.random_mask(M, K, BR, BC, (0, 1, 8, 13, 32), (0, 3, 12, 16, 32), seed=130)
    W = gen.normal_weights(M, K, dtype, seed=131)
    x = gen.normal_activations(K, batch, dtype, seed=132)
    A = pack_workload(g, W, dtype, mask)
    yref, S = oracle_product(W, x, dtype, mask)
    y = run_spmv(g, A, x, dtype, M, batch)
    assert_close(y, yref, S, dtype, f"spmv {dtype} b={batch}")
    y2 = run_spmv(g, A, x, dtype, M, batch, ldx=batch + 3, ldy=batch + 1)
    if batch == 8 and dtype != gen.F32:
        # 8 columns in 16-byte-aligned rows went to the matrix-core kernel, padded rows go to the SpMV kernel:
        # two orders of addition; the SpMV kernel's own bits must not depend on the padding
        assert_close(y2, yref, S, dtype, f"spmv {dtype} b={batch}, padded rows")
        assert run_spmv(g, A, x, dtype, M, batch, ldx=batch + 4, ldy=batch).tobytes() == y2.tobytes()
    else:
        assert y2.tobytes() == y.tobytes()


@pytest.mark.parametrize("BR,BC", [(8, 16), (16, 8), (32, 24), (4, 32)])
def test_spmv_small_blocks(g, BR, BC):
    dtype = gen.F16
    M, K = BR * 10, BC * 20
    mask = gen.random_mask(M, K, BR, BC, (1, BR // 2, BR), (1, BC // 2, BC), seed=140)
    W = gen.normal_weights(M, K, dtype, seed=141)
    x = gen.normal_activations(K, 4, dtype, seed=142)
    A = pack_workload(g, W, dtype, mask)
    yref, S = oracle_product(W, x, dtype, mask)
    assert_close(run_spmv(g, A, x, dtype, M, 4), yref, S, dtype, f"spmv {BR}x{BC}")


def test_spmv_falls_back_when_blocks_exceed_masks(g):
    dtype = gen.F16
    M, K = 128, 256
    mask = gen.random_mask(M, K, 64, 64, (8, 16), (8, 32), seed=150)
    W = gen.normal_weights(M, K, dtype, seed=151)
    x = gen.normal_activations(K, 2, dtype, seed=152)
    A = pack_workload(g, W, dtype, mask)
    yref, S = oracle_product(W, x, dtype, mask)
    assert_close(run_spmv(g, A, x, dtype, M, 2), yref, S, dtype, "spmv 64x64 blocks")
    # batches the row-gathering kernel takes (multiples of 4) go there, the rest to the vector-ALU kernel
    for batch in (4, 8, 5):
        xb = gen.normal_activations(K, batch, dtype, seed=153 + batch)
        yref, S = oracle_product(W, xb, dtype, mask)
        assert_close(run_spmv(g, A, xb, dtype, M, batch), yref, S, dtype, f"spmv 64x64 blocks, batch {batch}")
        assert g.spmm_kernel_name(A, to_device(xb, dtype), batch, batch) == ("bcr_spmm_gather" if batch % 4 == 0 else "bcr_spmm_fma")


# ------------------------------------------------------------------ staged kernel: more tiles than compute units
@pytest.mark.parametrize("dtype,BR", [(gen.F16, 16), (gen.BF16, 32)])
@pytest.mark.parametrize("N,tile_n,strips", [(9004, 32, 4), (17000, 64, 4), (17001, 64, 8), (9004, 32, 8)])
def test_staged_kernel_more_tiles_than_compute_units(g, dtype, BR, N, tile_n, strips):
    """More workgroups than the GPU holds at once (256 compute units), so that workgroups start while others are
    still running: odd chunk counts, one and two strip groups per tile, rows of X at every alignment, ragged ends,
    every entry checked."""
    M, K, BC = BR * (strips if strips == 4 else 2 * strips), 96 * 3, 32      # chunk of 96 rows -> 3 chunks per tile
    mask = gen.random_mask(M, K, BR, BC, (0, BR // 4, BR // 2, BR), (0, 8, 11, 32), seed=320 + BR)
    W = gen.normal_weights(M, K, dtype, seed=321)
    X = gen.normal_activations(K, N, dtype, seed=322, relu=True)
    A = pack_workload(g, W, dtype, mask, chunk_rows=96)
    Yref, S = oracle_product(W, X, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, kernel=2, tile_n=tile_n, strips_per_wg=strips)
    assert_close(Y, Yref, S, dtype, f"staged {dtype} N={N} tile {tile_n} strips {strips}")
    Y2 = run_spmm(g, A, X, dtype, M, N, kernel=2, tile_n=tile_n, strips_per_wg=strips)
    assert Y2.tobytes() == Y.tobytes()


# ------------------------------------------------------------------ wide-tile staged matrix-core kernel
@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("BR,tile_n", [(16, 128), (16, 192), (32, 96)])
@pytest.mark.parametrize("strips,K,N,ldx_pad,ldy_pad,chunk_rows", [
    (16, 416, 1000, 0, 0, 0),       # one group, K tail (416 = 3 chunks of 128 + 32), ragged last tile
    (24, 288, 776, 8, 4, 96),       # a second, half-filled strip group; 96-row chunks; padded leading dimensions
    (8, 128, 200, 0, 0, 0),         # waves without a second strip; one chunk; one full tile + a shifted one (or one)
    (5, 640, 384, 16, 8, 64),       # fewer strips than waves; 64-row chunks; N a multiple of both widths
])
def test_wide_kernel_shapes(g, dtype, BR, tile_n, strips, K, N, ldx_pad, ldy_pad, chunk_rows):
    """kernel = 4 forced: every compiled tile width per block height, strip groups that are full, ragged and nearly
    empty, chunk counts 1..10 (odd and even: both register sets end the pipeline), K tails, shifted last tiles, empty
    blocks and empty strips; every entry against the oracle, and twice for bit reproducibility."""
    M = strips * BR
    mask = gen.random_mask(M, K, BR, 32, (0, BR // 4, BR // 2), (0, 4, 8, 13), seed=800 + BR + strips)
    W = gen.normal_weights(M, K, dtype, seed=801)
    X = gen.normal_activations(K, N, dtype, seed=802, relu=True)
    A = pack_workload(g, W, dtype, mask, chunk_rows=chunk_rows)
    Yref, S = oracle_product(W, X, dtype, mask)
    if N < tile_n:
        with pytest.raises(g.GrimError):
            run_spmm(g, A, X, dtype, M, N, kernel=4, tile_n=tile_n)
        return
    Y = run_spmm(g, A, X, dtype, M, N, ldx=N + ldx_pad, ldy=N + ldy_pad, kernel=4, tile_n=tile_n)
    assert_close(Y, Yref, S, dtype, f"wide {dtype} BR={BR} tn={tile_n} strips={strips} K={K} N={N}")
    Y2 = run_spmm(g, A, X, dtype, M, N, ldx=N + ldx_pad, ldy=N + ldy_pad, kernel=4, tile_n=tile_n)
    assert Y2.tobytes() == Y.tobytes()
    assert A.unpack_layout(4).tobytes() == A.unpack().tobytes()


def test_wide_kernel_integer_data_is_exact(g):
    M, K, N, BR = 512, 1024, 2048, 32
    mask = gen.random_mask(M, K, BR, 32, (4, 8, 16), (4, 8, 16), seed=810)
    W = gen.small_int_values((M, K), gen.BF16, seed=811)
    X = gen.small_int_values((K, N), gen.BF16, seed=812)
    A = pack_workload(g, W, gen.BF16, mask)
    Yref, _ = oracle_product(W, X, gen.BF16, mask)
    for tn in (96, 0):
        Y = run_spmm(g, A, X, gen.BF16, M, N, kernel=4, tile_n=tn)
        assert np.array_equal(Y.astype(np.float64), Yref)


def test_wide_kernel_more_tiles_than_compute_units_and_refusals(g):
    """Two rounds of workgroups on the GPU (600 tiles), two strip groups; and the operands the kernel refuses."""
    torch, dev = torch_dev()
    M, K, N, BR = 32 * 16, 256, 600 * 96, 16
    mask = gen.random_mask(M, K, BR, 32, (0, 4, 8), (0, 8, 16), seed=820)
    W = gen.normal_weights(M, K, gen.F16, seed=821)
    X = gen.normal_activations(K, N, gen.F16, seed=822, relu=True)
    A = pack_workload(g, W, gen.F16, mask)
    Y = run_spmm(g, A, X, gen.F16, M, N, kernel=4, tile_n=128)
    rows = np.arange(0, M, 5)
    cols = np.unique(np.concatenate([np.arange(0, 200), np.arange(N - 200, N), np.arange(256 * 128 - 64, 256 * 128 + 64),
                                     np.random.default_rng(3).choice(N, 300, replace=False)]))
    Yref, S = oracle_product(W, X, gen.F16, mask, rows=rows, cols=cols)
    assert_close(Y[np.ix_(rows, cols)], Yref, S, gen.F16, "wide, 2 rounds of workgroups")
    Xd = to_device(X[:, :1024].copy(), gen.F16)
    Yd = torch.empty((M, 1024), dtype=torch.float32, device=dev)
    s = torch.cuda.current_stream()
    for kw in (dict(tile_n=96), dict(tile_n=64), dict(tile_n=128, strips_per_wg=4)):      # widths of the other block height
        with pytest.raises(g.GrimError):
            g.spmm(A, Xd, 1024, 1024, Yd, 1024, s, kernel=4, **kw)
    with pytest.raises(g.GrimError):
        g.spmm(A, Xd, 1020, 1024, Yd, 1024, s, kernel=4)                                   # N not a multiple of 8
    with pytest.raises(g.GrimError):
        g.spmm(A, Xd, 1000, 1020, Yd, 1024, s, kernel=4)                                   # rows of X not 16-byte aligned
    w1 = gen.c1_single_fp32()
    A1 = pack_workload(g, w1.W, w1.dtype, w1.mask)
    with pytest.raises(g.GrimError):
        run_spmm(g, A1, w1.X, w1.dtype, w1.M, w1.N, kernel=4)                              # fp32


# ------------------------------------------------------------------ row-gathering matrix-core kernel
@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("N,ldx_pad,ldy_pad", [(64, 0, 0), (200, 0, 0), (196, 0, 0), (328, 8, 4), (132, 4, 3),
                                               (4, 0, 0), (8, 0, 1), (12, 0, 0), (32, 0, 0), (36, 4, 0), (60, 0, 2)])
def test_gather_kernel_shapes(g, dtype, N, ldx_pad, ldy_pad):
    """kernel = 3 forced: tiles that overlap at the ragged end, fewer than 64 columns (one tile, the pieces past N
    never fetched past the end of X nor stored), rows of X aligned to 16 and to 8 bytes,
    padded leading dimensions (Y with a stride that rules out 16-byte stores), non-uniform blocks with
    empty ones, strips with fewer steps than waves, an all-empty strip."""
    M, K, BR, BC = 16 * 9, 32 * 23, 16, 32
    mask = gen.random_mask(M, K, BR, BC, (0, 1, 5, 8, 16), (0, 3, 8, 17, 32), seed=300)
    # strip 2 keeps nothing at all, strip 4 a single block
    keep_r, keep_c = [], []
    nbc = K // BC
    for b in range((M // BR) * nbc):
        r = mask.row_idx[mask.row_ptr[b]:mask.row_ptr[b + 1]]
        c = mask.col_idx[mask.col_ptr[b]:mask.col_ptr[b + 1]]
        s_, c_ = divmod(b, nbc)
        if s_ == 2 or (s_ == 4 and c_ != 7):
            r, c = r[:0], c[:0]
        keep_r.append(r); keep_c.append(c)
    mask = gen.mask_from_sets(M, K, BR, BC, keep_r, keep_c)
    W = gen.normal_weights(M, K, dtype, seed=301)
    X = gen.normal_activations(K, N, dtype, seed=302)
    A = pack_workload(g, W, dtype, mask)
    Yref, S = oracle_product(W, X, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, ldx=N + ldx_pad, ldy=N + ldy_pad, kernel=3)
    assert_close(Y, Yref, S, dtype, f"gather {dtype} N={N}")
    Y2 = run_spmm(g, A, X, dtype, M, N, ldx=N + ldx_pad, ldy=N + ldy_pad, kernel=3)
    assert Y2.tobytes() == Y.tobytes()


def test_gather_kernel_every_tile_count_around_the_xcd_count(g):
    """1 to 17 tiles: the tiles past the last multiple of 8 are cut into 2, 4 or 8 sets of strips (here 5 strips, so the
    sets are uneven and some are empty) and dealt to the XCDs; every (tile, strip) must be computed exactly once."""
    dtype = gen.F16
    M, K, BR, BC = 80, 256, 16, 32
    mask = gen.random_mask(M, K, BR, BC, (4, 8, 16), (4, 8, 12), seed=340)
    W = gen.normal_weights(M, K, dtype, seed=341)
    A = pack_workload(g, W, dtype, mask)
    Xall = gen.normal_activations(K, 64 * 17, dtype, seed=342)
    Yall, Sall = oracle_product(W, Xall, dtype, mask)
    for tiles in range(1, 18):
        N = 64 * tiles - (4 if tiles % 3 == 0 else 0)
        Y = run_spmm(g, A, Xall[:, :N].copy(), dtype, M, N, kernel=3)
        assert_close(Y, Yall[:, :N], Sall[:, :N], dtype, f"gather, {tiles} tiles")


@pytest.mark.parametrize("dtype,N", [(gen.F16, 44820), (gen.BF16, 44808)])
def test_gather_kernel_wave_per_strip(g, dtype, N):
    """Strips of a few steps and thousands of (tile, strip) pairs (the first layers of a CNN at full resolution): every
    wave then takes a pair of its own.  Six strips, so the second workgroup of a tile has two idle waves; one strip keeps
    nothing; rows of X 8- and 16-byte aligned; a ragged last tile; every entry checked."""
    M, K, BR, BC = 96, 96, 16, 32
    mask = gen.random_mask(M, K, BR, BC, (0, 3, 8, 16), (0, 5, 8, 32), seed=330)
    nbc = K // BC
    keep_r, keep_c = [], []
    for b in range((M // BR) * nbc):
        r = mask.row_idx[mask.row_ptr[b]:mask.row_ptr[b + 1]]
        c = mask.col_idx[mask.col_ptr[b]:mask.col_ptr[b + 1]]
        if b // nbc == 4:
            r, c = r[:0], c[:0]
        keep_r.append(r); keep_c.append(c)
    mask = gen.mask_from_sets(M, K, BR, BC, keep_r, keep_c)
    W = gen.normal_weights(M, K, dtype, seed=331)
    X = gen.normal_activations(K, N, dtype, seed=332, relu=True)
    A = pack_workload(g, W, dtype, mask)
    Yref, S = oracle_product(W, X, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, kernel=3)
    assert_close(Y, Yref, S, dtype, f"gather, wave per strip, {dtype} N={N}")
    assert run_spmm(g, A, X, dtype, M, N, kernel=3).tobytes() == Y.tobytes()


def test_gather_kernel_wave_per_strip_long_strips(g):
    """Strips of more than 8 steps take the wave-per-pair form from 1536 (tile, strip) pairs on: a wave then runs
    several batches of steps on its own.  Non-uniform blocks (4 to 22 steps per strip), 3 strips (one idle wave per
    workgroup), 520 tiles with a ragged last one; every entry checked."""
    dtype, N = gen.F16, 64 * 520 - 12
    M, K, BR, BC = 48, 32 * 22, 16, 32
    mask = gen.random_mask(M, K, BR, BC, (3, 8, 16), (4, 16, 32), seed=350)
    # strip 1 keeps every column of every block: 22 steps
    nbc = K // BC
    keep_r, keep_c = [], []
    for b in range((M // BR) * nbc):
        r = mask.row_idx[mask.row_ptr[b]:mask.row_ptr[b + 1]]
        c = mask.col_idx[mask.col_ptr[b]:mask.col_ptr[b + 1]]
        if b // nbc == 1:
            c = np.arange(BC, dtype=c.dtype)
        keep_r.append(r); keep_c.append(c)
    mask = gen.mask_from_sets(M, K, BR, BC, keep_r, keep_c)
    W = gen.normal_weights(M, K, dtype, seed=351)
    X = gen.normal_activations(K, N, dtype, seed=352, relu=True)
    A = pack_workload(g, W, dtype, mask)
    Yref, S = oracle_product(W, X, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, kernel=3)
    assert_close(Y, Yref, S, dtype, "gather, wave per strip, long strips")


def test_gather_kernel_c2_and_refusals(g):
    wl = gen.c2_vgg_conv(3136)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    Yref, S = oracle_product(wl.W, wl.X, wl.dtype, wl.mask)
    Y = run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N, kernel=3)
    assert_close(Y, Yref, S, wl.dtype, "gather c2")
    from paper_2108_11033_amd.binding import GrimError
    for N in (2, 63, 66, 201):                                   # rows not 8-byte aligned
        X = gen.normal_activations(wl.K, N, wl.dtype, seed=303)
        with pytest.raises(GrimError) as e:
            run_spmm(g, A, X, wl.dtype, wl.M, N, kernel=3)
        assert e.value.status == 7
    with pytest.raises(GrimError):                                # tile knobs belong to the staged kernel
        run_spmm(g, A, wl.X, wl.dtype, wl.M, wl.N, kernel=3, tile_n=64)
    w1 = gen.c1_single_fp32()                                     # fp32: no matrix-core kernel
    A1 = pack_workload(g, w1.W, w1.dtype, w1.mask)
    with pytest.raises(GrimError) as e:
        run_spmm(g, A1, w1.X, w1.dtype, w1.M, w1.N, kernel=3)
    assert e.value.status == 7
    M, K = 96, 128                                                # 24-row blocks neither divide 16 nor are a multiple
    m24 = gen.random_mask(M, K, 24, 32, 12, 8, seed=304)
    A24 = pack_workload(g, gen.normal_weights(M, K, gen.F16, seed=305), gen.F16, m24)
    with pytest.raises(GrimError) as e:
        run_spmm(g, A24, gen.normal_activations(K, 64, gen.F16, seed=306), gen.F16, M, 64, kernel=3)
    assert e.value.status == 7


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("BR,BC", [(4, 16), (1, 32), (2, 8), (8, 24), (32, 32), (48, 16), (64, 64)])
def test_gather_kernel_block_heights(g, dtype, BR, BC):
    """Block heights that divide 16 (several strips share a 16-row tile; 4 x 16 is the block size of the
    paper's CNN evaluation) or are multiples of 16 (a strip spans several tiles), mixed kept counts with
    empty blocks, a row count that is not a multiple of 16 where the block height allows it; forced and
    chosen by the library."""
    M = 192 if BR in (48, 64) else 72 if 72 % BR == 0 else 96
    K, N = BC * 13, 136
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, (BR + 1) // 2, BR})), tuple(sorted({0, 1, BC // 3 + 1, BC})), seed=310 + BR)
    W = gen.normal_weights(M, K, dtype, seed=311)
    X = gen.normal_activations(K, N, dtype, seed=312)
    A = pack_workload(g, W, dtype, mask)
    Yref, S = oracle_product(W, X, dtype, mask)
    Y = run_spmm(g, A, X, dtype, M, N, kernel=3)
    assert_close(Y, Yref, S, dtype, f"gather {dtype} {BR}x{BC}")
    Xd = to_device(X, dtype)
    if BR not in (16, 32):
        assert g.spmm_kernel_name(A, Xd, N, N) == "bcr_spmm_gather"      # the only matrix-core route
    Y0 = run_spmm(g, A, X, dtype, M, N)
    assert_close(Y0, Yref, S, dtype, f"auto {dtype} {BR}x{BC}")


def test_kernel_choice_follows_the_cost_model(g):
    """grim_bcr_spmm_kernel_name reports the route; few tiles per strip group -> row-gathering kernel, very
    many tiles of a many-strip matrix -> wide-tile staged kernel; fp32 -> FMA kernel; N <= 8 -> SpMV."""
    torch, dev = torch_dev()
    wl = gen.c2_vgg_conv(200)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    X = to_device(wl.X, wl.dtype)
    assert g.spmm_kernel_name(A, X, 200, 200) == "bcr_spmm_gather"
    assert g.spmm_kernel_name(A, X, 200, 200, kernel=2) == "bcr_spmm_mma"
    assert g.spmm_kernel_name(A, X, 200, 200, tile_n=64) == "bcr_spmm_mma"
    assert g.spmm_kernel_name(A, X, 4, 200) == "bcr_spmv"
    assert g.spmm_kernel_name(A, X, 8, 200) == "bcr_spmv"             # uniform blocks: a set of workgroups per column
    assert g.spmm_kernel_name(A, X, 8, 204) == "bcr_spmv"             # rows 8-byte aligned only
    assert g.spmm_kernel_name(A, X, 199, 200) == "bcr_spmm_mma"       # rows not 8-byte aligned
    assert g.spmm_kernel_name(A, X, 200, 200, kernel=1) == "bcr_spmm_fma"
    assert g.spmm_kernel_name(A, X, 200, 100) == "none"               # ldx < N
    big = torch.empty(16, dtype=torch.float16, device=dev)            # only the address is looked at
    assert g.spmm_kernel_name(A, big, 50176, 50176) == "bcr_spmm_wide"     # a round of 192-column tiles (+ a remainder)
    assert g.spmm_kernel_name(A, big, 50176, 50176, kernel=2) == "bcr_spmm_mma"
    assert g.spmm_kernel_name(A, big, 50176, 50176, kernel=4, tile_n=128) == "bcr_spmm_wide"
    assert g.spmm_kernel_name(A, big, 50176, 50176, kernel=4, tile_n=96) == "none"      # 96 columns: 32-row blocks only
    assert g.spmm_kernel_name(A, big, 50180, 50180) != "bcr_spmm_wide"     # N not a multiple of 8
    w1 = gen.c1_single_fp32()
    A1 = pack_workload(g, w1.W, w1.dtype, w1.mask)
    assert g.spmm_kernel_name(A1, to_device(w1.X, w1.dtype), w1.N, w1.N) == "bcr_spmm_fma"
    assert g.spmm_kernel_name(A1, to_device(w1.X, w1.dtype), w1.N, w1.N, kernel=3) == "none"


# Every (kept rows, kept columns) pair the uniform one-right-hand-side kernel is compiled for, in each
# element type, with: 16- and 32-row blocks (4 and 2 output lane groups), a strip of more than 64 column
# blocks (two passes of lanes, the second ragged), a strip count that is not a multiple of the 4 strips
# of a workgroup, unit and non-unit strides of x and y.
UNIFORM_PAIRS = [(4, 4), (4, 8), (4, 12), (4, 16), (8, 4), (8, 8), (8, 12), (8, 16), (16, 4), (16, 8), (16, 12)]


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16, gen.F32])
@pytest.mark.parametrize("kr,kc", UNIFORM_PAIRS)
def test_spmv_uniform_pairs(g, dtype, kr, kc):
    for BR, nbr, nbc in ((16, 7, 70), (32, 5, 9)):
        BC = 32
        M, K = BR * nbr, BC * nbc
        mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=200 + kr * 17 + kc)
        W = gen.normal_weights(M, K, dtype, seed=201 + kr)
        x = gen.normal_activations(K, 1, dtype, seed=202 + kc)
        A = pack_workload(g, W, dtype, mask)
        yref, S = oracle_product(W, x, dtype, mask)
        y = run_spmv(g, A, x, dtype, M, 1)
        assert_close(y, yref, S, dtype, f"uniform spmv {dtype} {BR}x{BC} keep {kr}x{kc}")
        y2 = run_spmv(g, A, x, dtype, M, 1, ldx=3, ldy=2)
        assert y2.tobytes() == y.tobytes()
        A.free()


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("batch", [2, 5, 8])
@pytest.mark.parametrize("kr,kc", UNIFORM_PAIRS)
def test_spmv_uniform_pairs_several_rhs(g, dtype, batch, kr, kc):
    """2..8 right-hand sides on uniformly pruned matrices: launches of at least 1024 strips of at most 64
    column blocks take the wave-per-strip kernel with a loop over the right-hand sides (smaller ones the
    workgroup-per-strip kernel, covered by the single calls below); contiguous and strided x / y."""
    torch, dev = torch_dev()
    from paper_2108_11033_amd import binding
    for BR, nbr, nbc, count in ((16, 11, 64, 96), (32, 5, 9, 208)):
        BC = 32
        M, K = BR * nbr, BC * nbc
        mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=220 + kr * 17 + kc)
        W = gen.normal_weights(M, K, dtype, seed=221 + kr)
        A = pack_workload(g, W, dtype, mask)
        xs = [gen.normal_activations(K, batch, dtype, seed=222 + kc + i) for i in range(2)]
        refs = [oracle_product(W, x, dtype, mask) for x in xs]
        G = binding.group([A] * count)
        stream = torch.cuda.current_stream()
        xd = to_device(np.stack([xs[i % 2] for i in range(count)]), dtype)               # [count, K, batch]
        yd = torch.full((count, M, batch), float("nan"), dtype=torch.float32, device=dev)
        g.spmv_batched(G, xd, K * batch, batch, batch, yd, M * batch, batch, stream)
        torch.cuda.synchronize()
        y = yd.cpu().numpy()
        for i in (0, 1, count // 2, count - 2, count - 1):
            assert_close(y[i], refs[i % 2][0], refs[i % 2][1], dtype,
                         f"uniform {dtype} {BR}x{BC} keep {kr}x{kc} b={batch} product {i}")
        assert all(y[i].tobytes() == y[i % 2].tobytes() for i in range(count))
        # strided x and y
        ldx, ldy = batch + 3, batch + 1
        xp = np.zeros((count, K, ldx), dtype=xs[0].dtype)
        for i in range(count):
            xp[i, :, :batch] = xs[i % 2]
        xd2 = to_device(xp, dtype)
        yd2 = torch.full((count, M, ldy), float("nan"), dtype=torch.float32, device=dev)
        g.spmv_batched(G, xd2, K * ldx, batch, ldx, yd2, M * ldy, ldy, stream)
        torch.cuda.synchronize()
        y2 = yd2.cpu().numpy()
        assert np.isnan(y2[:, :, batch:]).all()
        assert y2[:, :, :batch].tobytes() == y.tobytes()
        # one product at a time gives the same values to within the tolerance
        y1 = run_spmv(g, A, xs[0], dtype, M, batch)
        assert_close(y1, refs[0][0], refs[0][1], dtype, "single call")
        G.free()
        A.free()


@pytest.mark.parametrize("dtype", [gen.F16, gen.F32])
def test_spmv_uniform_many_products_per_launch(g, dtype):
    """Enough products in one launch that every wave walks several strips (next strip's loads in flight,
    finished strips stored in groups), with a strip count that leaves the last waves short."""
    torch, dev = torch_dev()
    M, K, BR, BC, count = 16 * 37, 32 * 20, 16, 32, 256
    mask = gen.random_mask(M, K, BR, BC, 8, 12, seed=210)
    W = gen.normal_weights(M, K, dtype, seed=211)
    A = pack_workload(g, W, dtype, mask)
    xs = [gen.normal_activations(K, 1, dtype, seed=212 + i) for i in range(3)]
    refs = [oracle_product(W, x, dtype, mask) for x in xs]
    from paper_2108_11033_amd import binding
    G = binding.group([A] * count)
    xd = to_device(np.stack([xs[i % 3] for i in range(count)]), dtype)
    yd = torch.full((count, M, 1), float("nan"), dtype=torch.float32, device=dev)
    g.spmv_batched(G, xd, K, 1, 1, yd, M, 1, torch.cuda.current_stream())
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    for i in range(count):
        assert_close(y[i], refs[i % 3][0], refs[i % 3][1], dtype, f"product {i} of {count}")
    for i in range(3):
        assert y[i].tobytes() == run_spmv(g, A, xs[i], dtype, M, 1).tobytes()


@pytest.mark.parametrize("batch", [1, 8])
def test_spmv_batched_matches_single_calls(g, batch):
    torch, dev = torch_dev()
    dtype = gen.F16
    M, K, BR, BC, count = 256, 512, 32, 32, 5
    mats, xs, refs = [], [], []
    for i in range(count):
        mask = gen.random_mask(M, K, BR, BC, 8, 12, seed=160 + i)
        W = gen.normal_weights(M, K, dtype, seed=170 + i)
        x = gen.normal_activations(K, batch, dtype, seed=180 + i)
        mats.append(pack_workload(g, W, dtype, mask))
        xs.append(x)
        refs.append(oracle_product(W, x, dtype, mask))
    from paper_2108_11033_amd import binding
    G = binding.group(mats)
    xd = to_device(np.stack(xs), dtype)                       # [count, K, batch]
    yd = torch.full((count, M, batch), float("nan"), dtype=torch.float32, device=dev)
    g.spmv_batched(G, xd, K * batch, batch, batch, yd, M * batch, batch, torch.cuda.current_stream())
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    for i in range(count):
        assert_close(y[i], refs[i][0], refs[i][1], dtype, f"batched {i}")
        # (a leading dimension that is no multiple of 8 keeps the single call on the SpMV kernels at batch 8)
        yi = run_spmv(g, mats[i], xs[i], dtype, M, batch, ldx=batch + 4)
        assert yi.tobytes() == y[i].tobytes()


# ------------------------------------------------------------------ errors leave Y untouched
def test_device_call_errors(g):
    torch, dev = torch_dev()
    wl = gen.c2_vgg_conv(N=64)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)
    Xd = to_device(wl.X, wl.dtype)
    Yd = torch.full((wl.M, 64), 7.0, dtype=torch.float32, device=dev)
    from paper_2108_11033_amd import GrimError
    for kwargs, name in (
        (dict(N=0, ldx=64, ldy=64), "GRIM_ERR_SHAPE"),
        (dict(N=64, ldx=63, ldy=64), "GRIM_ERR_SHAPE"),
        (dict(N=64, ldx=64, ldy=10), "GRIM_ERR_SHAPE"),
    ):
        with pytest.raises(GrimError) as e:
            g.spmm(A, Xd, kwargs["N"], kwargs["ldx"], Yd, kwargs["ldy"])
        assert e.value.name == name
    with pytest.raises(GrimError) as e:
        g.spmm(A, None, 64, 64, Yd, 64)
    assert e.value.name == "GRIM_ERR_NULL"
    with pytest.raises(GrimError) as e:
        g.spmv(A, Xd, 9, 64, Yd, 64)
    assert e.value.name == "GRIM_ERR_SHAPE"
    with pytest.raises(GrimError) as e:
        g.spmm(A, Xd, 64, 64, Yd, 64, tile_n=48)
    assert e.value.name == "GRIM_ERR_UNSUPPORTED"
    H = pack_workload(g, wl.W, wl.dtype, wl.mask, host_only=True)
    with pytest.raises(GrimError) as e:
        g.spmm(H, Xd, 64, 64, Yd, 64)
    assert e.value.name == "GRIM_ERR_DEVICE"
    big = gen.random_mask(144, 256, 72, 32, 8, 8, seed=1)        # 72-row blocks: too tall for the FMA kernel, no 16-row tiling
    B = pack_workload(g, gen.normal_weights(144, 256, gen.F16, 1), gen.F16, big)
    with pytest.raises(GrimError) as e:
        g.spmm(B, Xd, 64, 64, Yd, 64)
    assert e.value.name == "GRIM_ERR_UNSUPPORTED"
    torch.cuda.synchronize()
    assert (Yd == 7.0).all()
