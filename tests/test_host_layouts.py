"""Host-side checks of the layouts the kernels read (no GPU): every derived layout -- the staged matrix-core
SpMM's step records, the row-gathering SpMM's steps per 16-row run, the SpMV's bit masks -- decodes back to
exactly the masked dense matrix, over a seeded sweep of odd shapes: block heights and widths from 1 to 64,
empty blocks, empty strips, a K = 27 dense first layer, matrices of one block."""
import numpy as np
import pytest

import bcr_inputs as gen
import paper_2108_11033_amd as g
from paper_2108_11033_amd.binding import GrimError
from oracle import bcr_oracle as orc

LAYOUTS = {1: "staged SpMM", 2: "row-gathering SpMM", 3: "SpMV", 4: "wide-tile staged SpMM"}


def _expected_layouts(dtype, BR, BC):
    want = set()
    if dtype != gen.F32 and BR in (16, 32) and BC <= 256:
        want.add(1)
    if dtype != gen.F32 and BR in (16, 32) and BC <= 128:
        want.add(4)
    if dtype != gen.F32 and (16 % BR == 0 or BR % 16 == 0):
        want.add(2)
    if BR <= 32 and BC <= 32:
        want.add(3)
    return want


def _check(M, K, BR, BC, kr, kc, dtype, seed, dense=False):
    mask = gen.full_mask(M, K, BR, BC) if dense else gen.random_mask(M, K, BR, BC, kr, kc, seed=seed)
    W = gen.normal_weights(M, K, dtype, seed=seed + 1)
    for reorder in (True, False):
        A = g.pack(W, dtype, BR, BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, host_only=2,
                   no_reorder=not reorder)
        ref = A.unpack()
        Wm = orc.masked_dense(gen.storage_to_f64(W, dtype), BR, BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx)
        assert ref.tobytes() == np.where(Wm != 0, W, np.zeros_like(W)).tobytes()
        have = set()
        for lay in LAYOUTS:
            try:
                got = A.unpack_layout(lay)
            except GrimError as e:
                assert e.name == "GRIM_ERR_UNSUPPORTED", (lay, e)
                continue
            have.add(lay)
            assert got.tobytes() == ref.tobytes(), f"{LAYOUTS[lay]} layout of {M}x{K} {BR}x{BC} {dtype} decodes wrongly"
        assert have == _expected_layouts(dtype, BR, BC), (have, dtype, BR, BC)


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16, gen.F32])
@pytest.mark.parametrize("M,K,BR,BC,kr,kc", [
    (64, 96, 16, 32, (0, 4, 8, 16), (0, 8, 32)),       # empty and full blocks
    (96, 128, 32, 32, (4, 8, 16), (4, 8, 16)),         # the non-uniform workload's law
    (48, 64, 4, 16, (0, 2, 4), (0, 4, 16)),            # the paper's CNN block size
    (128, 128, 64, 64, (8, 32), (8, 24)),
    (30, 28, 5, 7, (0, 1, 5), (0, 2, 7)),              # heights that fit no matrix-core tile
    (12, 10, 1, 1, (0, 1), (0, 1)),                    # non-structured limit
    (16, 24, 16, 24, 5, 9),                            # one block = the whole matrix
    (96, 40, 48, 8, (0, 7, 48), (1, 3, 8)),
    (32, 576, 16, 32, 8, 8),                           # c2's pattern, several chunks of the staged layout
    (64, 512, 32, 32, (0, 32), (0, 1, 32)),
    (40, 66, 8, 33, (1, 8), (1, 17, 33)),              # odd block width
    (34, 64, 2, 64, (0, 1, 2), (3, 9, 64)),
])
def test_every_layout_decodes_to_the_masked_matrix(dtype, M, K, BR, BC, kr, kc):
    _check(M, K, BR, BC, kr, kc, dtype, seed=500 + M + K)


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
def test_dense_first_layer_layouts(dtype):
    # VGG-16 layer 1: K = 27, one dense 16 x 27 block per strip
    _check(64, 27, 16, 27, 16, 27, dtype, seed=700, dense=True)


def test_seeded_sweep_of_block_shapes():
    rng = np.random.default_rng(20210811)
    for it in range(60):
        BR = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]))
        BC = int(rng.choice([1, 2, 5, 8, 9, 16, 27, 32, 40, 64]))
        nbr, nbc = int(rng.integers(1, 5)), int(rng.integers(1, 7))
        kr = tuple(sorted({0, int(rng.integers(0, BR + 1)), int(rng.integers(0, BR + 1)), BR}))
        kc = tuple(sorted({0, int(rng.integers(0, BC + 1)), int(rng.integers(0, BC + 1)), BC}))
        dtype = [gen.F16, gen.BF16, gen.F32][it % 3]
        _check(nbr * BR, nbc * BC, BR, BC, kr, kc, dtype, seed=1000 + it)


def test_unpack_layout_argument_errors():
    mask = gen.random_mask(32, 32, 16, 16, 4, 8, seed=1)
    W = gen.normal_weights(32, 32, gen.F16, seed=2)
    A = g.pack(W, gen.F16, 16, 16, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, host_only=2)
    lib = g.load_library()
    out = np.empty((32, 32), dtype=np.float16)
    p = out.ctypes.data
    assert lib.grim_bcr_unpack_layout(None, 1, p, 32) == 1                 # NULL
    assert lib.grim_bcr_unpack_layout(A.handle, 1, None, 32) == 1
    assert lib.grim_bcr_unpack_layout(A.handle, 1, p, 31) == 2             # ldw < K
    assert lib.grim_bcr_unpack_layout(A.handle, 0, p, 32) == 2             # unknown layout
    assert lib.grim_bcr_unpack_layout(A.handle, 5, p, 32) == 2
    B = g.pack(W, gen.F16, 16, 16, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, host_only=True)
    assert lib.grim_bcr_unpack_layout(B.handle, 2, p, 32) == 7             # canonical arrays only: no layouts
