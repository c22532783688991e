"""Host-side checks that need no GPU: the C ABI library loads and exports every symbol the
header declares, the C++ packer matches the NumPy reference byte for byte, pack -> unpack is
the masked matrix, and malformed arguments come back as status codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import bcr_inputs as gen
import paper_2108_11033_amd as g
from paper_2108_11033_amd import binding
from oracle import bcr_oracle as orc
from oracle import pack_ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _pack(W, dtype, mask, **kw):
    return g.pack(W, dtype, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx,
                  host_only=True, **kw)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "grim_bcr.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(grim_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(g.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert g.load_library().grim_status_str(2).startswith(b"GRIM_ERR_SHAPE")


@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("M,K,BR,BC,kr,kc", [
    (64, 96, 16, 32, (0, 4, 8, 16), (0, 8, 32)),
    (96, 64, 32, 32, (4, 8, 16), (4, 8, 16)),
    (30, 28, 5, 7, (0, 1, 5), (0, 2, 7)),
    (12, 10, 1, 1, (0, 1), (0, 1)),
    (16, 24, 16, 24, 5, 9),
])
def test_pack_matches_numpy_reference_bytes(dtype, M, K, BR, BC, kr, kc):
    mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=21)
    W = gen.normal_weights(M, K, dtype, seed=22)
    for reorder in (True, False):
        A = _pack(W, dtype, mask, no_reorder=not reorder)
        got, ref = A.arrays(), pack_ref.pack(W, mask, reorder=reorder)
        for k in ref:
            assert got[k].dtype == ref[k].dtype and got[k].tobytes() == ref[k].tobytes(), k
        v = A.view()
        assert (v.M, v.K, v.BR, v.BC, v.nnz, v.reordered) == (M, K, BR, BC, mask.nnz(), int(reorder))
        # pack -> unpack is the masked dense matrix, bit for bit (pruned entries +0)
        Wm = orc.masked_dense(gen.storage_to_f64(W, dtype), BR, BC, mask.row_ptr, mask.row_idx,
                              mask.col_ptr, mask.col_idx)
        back = A.unpack()
        assert back.tobytes() == np.where(Wm != 0, W, np.zeros_like(W)).tobytes()
        # idempotence
        B = _pack(back, dtype, mask, no_reorder=not reorder)
        assert all(B.arrays()[k].tobytes() == got[k].tobytes() for k in got)
        A.free()
        B.free()


def test_named_workload_counts_and_strip_order():
    for wl, nnz in ((gen.c1_single_fp32(), 8192), (gen.c2_vgg_conv(N=8), 73728), (gen.c3_lstm_gates(), 786432)):
        A = _pack(wl.W, wl.dtype, wl.mask)
        assert A.view().nnz == nnz
    mask = gen.random_mask(512, 4608, 32, 32, (4, 8, 16), (4, 8, 16), seed=5)
    A = _pack(gen.normal_weights(512, 4608, gen.BF16, 5), gen.BF16, mask)
    order = A.arrays()["strip_order"]
    work = pack_ref.strip_work(mask)
    assert sorted(order.tolist()) == list(range(16))
    assert (np.diff(work[order]) <= 0).all()              # work is non-increasing after the reorder


def test_pack_preserves_special_values_and_ignores_pruned_ones():
    M, K, BR, BC = 4, 6, 2, 3
    mask = gen.mask_from_sets(M, K, BR, BC, [[0], [0, 1], [1], [0, 1]], [[0, 2], [1], [1], [0, 2]])
    W = np.arange(1, 25, dtype=np.float32).reshape(M, K)
    W[0, 0] = -0.0
    W[0, 2] = np.nan
    W[3, 1] = 0.0
    W[1, 1] = np.inf                                        # pruned position: must not matter
    A = _pack(W, gen.F32, mask)
    w = A.arrays()["weights"]
    assert w.view(np.uint32).tolist() == np.array([0.0, 16, 18, 22, 24, -0.0, np.nan, 5, 11],
                                                  dtype=np.float32).view(np.uint32).tolist()
    back = A.unpack()
    assert back[1, 1] == 0 and not np.signbit(back[1, 1]) and np.signbit(back[0, 0]) and np.isnan(back[0, 2])


def test_leading_dimension():
    mask = gen.random_mask(32, 64, 16, 32, 4, 8, seed=30)
    W = gen.normal_weights(32, 80, gen.F16, seed=31)
    # pack the left 64 columns of an 80-column array through the raw ABI
    lib = g.load_library()
    out = ctypes.c_void_p()
    opt = binding.Options(0, 1, 0)
    st = lib.grim_bcr_pack(W.ctypes.data_as(ctypes.c_void_p), 1, 32, 64, 80, 16, 32,
                           mask.row_ptr.ctypes.data_as(ctypes.c_void_p), mask.row_idx.ctypes.data_as(ctypes.c_void_p),
                           mask.col_ptr.ctypes.data_as(ctypes.c_void_p), mask.col_idx.ctypes.data_as(ctypes.c_void_p),
                           ctypes.byref(opt), ctypes.byref(out))
    assert st == 0
    B = binding.BcrMatrix(out.value, lib)
    ref = pack_ref.pack(np.ascontiguousarray(W[:, :64]), mask)
    assert B.arrays()["weights"].tobytes() == ref["weights"].tobytes()


def _raw_pack(W, dt, M, K, ldw, BR, BC, rp, ri, cp, ci):
    lib = g.load_library()
    out = ctypes.c_void_p(1234)
    opt = binding.Options(0, 1, 0)
    p = lambda a: None if a is None else a.ctypes.data_as(ctypes.c_void_p)
    st = lib.grim_bcr_pack(p(W), dt, M, K, ldw, BR, BC, p(rp), p(ri), p(cp), p(ci), ctypes.byref(opt), ctypes.byref(out))
    if st != 0:
        assert out.value is None                               # *out is NULL on error
    else:
        lib.grim_bcr_free(out)
    return binding.STATUS_NAMES[st]


def test_pack_rejects_malformed_arguments():
    M, K, BR, BC = 32, 64, 16, 32
    mask = gen.random_mask(M, K, BR, BC, 4, 8, seed=40)
    W = gen.normal_weights(M, K, gen.F16, seed=41)
    rp, ri, cp, ci = mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx
    ok = lambda **kw: _raw_pack(**{**dict(W=W, dt=1, M=M, K=K, ldw=K, BR=BR, BC=BC, rp=rp, ri=ri, cp=cp, ci=ci), **kw})
    assert ok() == "GRIM_OK"
    assert ok(W=None) == "GRIM_ERR_NULL"
    assert ok(rp=None) == "GRIM_ERR_NULL"
    assert ok(ci=None) == "GRIM_ERR_NULL"
    assert ok(dt=7) == "GRIM_ERR_DTYPE"
    assert ok(BR=12) == "GRIM_ERR_SHAPE"                     # block sizes must divide the matrix
    assert ok(BC=24) == "GRIM_ERR_SHAPE"
    assert ok(ldw=K - 1) == "GRIM_ERR_SHAPE"
    assert ok(M=0) == "GRIM_ERR_SHAPE"
    bad = ri.copy(); bad[3] = BR                               # out of range
    assert ok(ri=bad) == "GRIM_ERR_INDEX"
    bad = ci.copy(); bad[1] = bad[0]                           # not strictly ascending
    assert ok(ci=bad) == "GRIM_ERR_INDEX"
    bad = rp.copy(); bad[0] = 1
    assert ok(rp=bad) == "GRIM_ERR_INDEX"
    bad = cp.copy(); bad[2] = bad[1] - 1                       # not monotone
    assert ok(cp=bad) == "GRIM_ERR_INDEX"
    bad = rp.copy(); bad[1:] += BR + 1                         # more kept rows than the block has
    assert ok(rp=bad) == "GRIM_ERR_INDEX"
    lib = g.load_library()
    assert lib.grim_bcr_unpack(None, None, 0) == 1 and lib.grim_bcr_arrays(None, None) == 1
    lib.grim_bcr_free(None)                                     # no-op
    lib.grim_bcr_group_free(None)
    assert lib.grim_bcr_spmm(None, None, 1, 1, None, 1, None) == 1
    assert lib.grim_bcr_spmv(None, None, 1, 1, None, 1, None) == 1


def test_host_only_matrix_cannot_launch():
    wl = gen.c1_single_fp32()
    A = _pack(wl.W, wl.dtype, wl.mask)
    lib = g.load_library()
    buf = np.zeros(16, dtype=np.float32)
    addr = buf.ctypes.data
    assert lib.grim_bcr_spmm(A.handle, addr, 4, 4, addr, 4, None) == binding.STATUS_NAMES.index("GRIM_ERR_DEVICE")
    assert lib.grim_bcr_spmv(A.handle, addr, 1, 1, addr, 1, None) == binding.STATUS_NAMES.index("GRIM_ERR_DEVICE")
