"""BCRC export (the paper's six-array compact storage, Section 4.3): library vs the dense-picture reference,
the values the paper's text quotes, round trip, and the index-overhead comparison with CSR.  CPU only."""
import numpy as np
import pytest

import bcr_inputs as gen
import paper_2108_11033_amd as g
from oracle import bcrc_ref
from conftest import read_golden


def _pack_host(W, dtype, mask):
    return g.pack(W, dtype, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, host_only=True)


def _same(lib: dict, ref: dict, W):
    for k in ("reorder", "row_offset", "occurrence", "column_stride", "compact_column"):
        assert lib[k].dtype == ref[k].dtype and np.array_equal(lib[k], ref[k]), k
    assert lib["weights"].tobytes() == np.ascontiguousarray(ref["weights"]).tobytes()


def test_paper_quoted_values():
    gold = read_golden("bcrc_paper_example.txt")

    def ints(key):
        return [int(v) for v in gold[key].split()]
    M, K, BR, BC = (ints(k)[0] for k in ("M", "K", "BR", "BC"))
    kept = ints("kept_col_of_row")
    nbc = K // BC
    mask = gen.mask_from_sets(M, K, BR, BC, [[0]] * (M * nbc), [[kept[b // nbc]] for b in range(M * nbc)])
    W = np.array(ints("W"), dtype=np.float32).reshape(M, K)
    ref = bcrc_ref.bcrc(W, bcrc_ref.keep_matrix(mask))
    lib = g.export_bcrc(_pack_host(W, gen.F32, mask))
    for out in (ref, lib):
        for name in ("reorder", "row_offset", "column_stride", "compact_column", "occurrence"):
            pre = ints(name + "_prefix")
            assert out[name][:len(pre)].tolist() == pre, name       # what the paper prints
            assert out[name].tolist() == ints(name), name           # the full arrays under our reading
        assert out["weights"].tolist() == [float(v) for v in ints("weights")]
    _same(lib, ref, W)


@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("shape", [(64, 96, 16, 32), (48, 60, 4, 5), (40, 64, 1, 1), (32, 64, 32, 64)])
def test_library_matches_reference_and_round_trips(dtype, shape):
    M, K, BR, BC = shape
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, BR // 2, BR})), tuple(sorted({0, 1, BC // 2, BC})), seed=500 + M)
    W = gen.normal_weights(M, K, dtype, seed=501)
    keep = bcrc_ref.keep_matrix(mask)
    ref = bcrc_ref.bcrc(W, keep)
    A = _pack_host(W, dtype, mask)
    lib = g.export_bcrc(A)
    _same(lib, ref, W)
    # invariants: reorder is a permutation; groups have distinct column lists; rows of a group share theirs
    assert sorted(lib["reorder"].tolist()) == list(range(M))
    lists = [tuple(lib["compact_column"][lib["column_stride"][i]:lib["column_stride"][i + 1]]) for i in range(lib["ngroups"])]
    assert len(set(lists)) == len(lists)
    for i in range(lib["ngroups"]):
        for p in range(lib["occurrence"][i], lib["occurrence"][i + 1]):
            assert tuple(np.nonzero(keep[lib["reorder"][p]])[0]) == lists[i]
            assert lib["row_offset"][p + 1] - lib["row_offset"][p] == len(lists[i])
    assert lib["nnz"] == int(keep.sum()) == A.view().nnz
    # round trip to the masked dense matrix, bit for bit (compare with the library's own unpack)
    dense = bcrc_ref.to_dense(lib, M, K)
    assert dense.tobytes() == A.unpack().tobytes()


def test_empty_and_full():
    M, K, BR, BC = 32, 64, 16, 32
    W = gen.normal_weights(M, K, gen.F16, seed=510)
    empty = gen.random_mask(M, K, BR, BC, 0, 0, seed=511)
    e = g.export_bcrc(_pack_host(W, gen.F16, empty))
    assert e["ngroups"] == 1 and e["nnz"] == 0 and e["reorder"].tolist() == list(range(M)) and len(e["compact_column"]) == 0
    full = gen.full_mask(M, K, BR, BC)
    f = g.export_bcrc(_pack_host(W, gen.F16, full))
    assert f["ngroups"] == 1 and f["nnz"] == M * K and f["compact_column"].tolist() == list(range(K))
    assert f["weights"].tobytes() == W.tobytes()


def test_index_overhead_against_csr():
    """The paper's comparison (Section 6.4, BCRC versus CSR): bytes that are not weights.  The saving comes from
    rows that share one column list.  With one column block per strip (the paper's figure: few blocks) all kept
    rows of a strip share theirs; with many independently pruned column blocks per strip (c2: 72) almost no two
    rows agree on every block, and BCRC's extra arrays make it no smaller than CSR."""
    M, K = 256, 1152
    W = gen.normal_weights(M, K, gen.F16, seed=520)
    wide = gen.random_mask(M, K, 16, K, 8, K // 4, seed=521)          # one block per strip
    b = g.export_bcrc(_pack_host(W, gen.F16, wide))
    o = bcrc_ref.index_bytes(b, M)
    assert b["ngroups"] == M // 16 + 1                                 # one list per strip + the rows that keep nothing
    assert o["saving"] > 0.8
    wl = gen.c2_vgg_conv(64)
    b2 = g.export_bcrc(_pack_host(wl.W, wl.dtype, wl.mask))
    o2 = bcrc_ref.index_bytes(b2, wl.M)
    assert b2["ngroups"] > wl.M // 2 and abs(o2["saving"]) < 0.05
