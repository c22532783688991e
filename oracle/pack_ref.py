"""Reference construction of the canonical compact BCR arrays, in NumPy.

TEST INFRASTRUCTURE ONLY.  Written straight from the format's definition and
independent of the C++ packer; tests compare the two byte for byte.

Format (one weights array plus index arrays; all little endian).  It plays the
role of the paper's BCRC storage (Section 4.3) at block granularity: zero
weights are not stored, and the column indices of a block are stored once for
all of its kept rows (the redundancy BCRC removes with its hierarchical
index).  Row strips are stored in order of decreasing work so that strips with
the same amount of computation sit together (matrix reorder, Section 4.2).

  strip_order[nbr]  int32   strips sorted by work w_s = sum_c kr*kc, descending,
                            stable (equal work: smaller strip index first)
  row_ptr[nb+1]     int32   prefix sums of kept-row counts, in STORED block order
  row_idx[...]      uint16  kept rows, local to the block, ascending
  col_ptr[nb+1]     int32   same for kept columns
  col_idx[...]      uint16
  blk_ptr[nb+1]     int64   prefix sums of kr*kc in stored order (offsets into weights)
  weights[nnz]      dtype   every block row-major [kept row][kept column], bit copies

Stored block order: strips in strip_order; inside a strip, column blocks ascending.
"""
from __future__ import annotations

import numpy as np


def strip_work(mask) -> np.ndarray:
    kr = np.diff(np.asarray(mask.row_ptr, dtype=np.int64))
    kc = np.diff(np.asarray(mask.col_ptr, dtype=np.int64))
    return (kr * kc).reshape(mask.M // mask.BR, mask.K // mask.BC).sum(axis=1)


def pack(W: np.ndarray, mask, reorder: bool = True) -> dict:
    """W: dense M x K array in the storage dtype (uint16 for bf16 bit patterns)."""
    M, K, BR, BC = mask.M, mask.K, mask.BR, mask.BC
    assert W.shape == (M, K)
    nbr, nbc = M // BR, K // BC
    work = strip_work(mask)
    if reorder:
        order = sorted(range(nbr), key=lambda s: (-int(work[s]), s))
    else:
        order = list(range(nbr))
    row_ptr, col_ptr, blk_ptr = [0], [0], [0]
    row_idx, col_idx, chunks = [], [], []
    for s in order:
        for c in range(nbc):
            b = s * nbc + c
            R = np.asarray(mask.row_idx[mask.row_ptr[b]:mask.row_ptr[b + 1]], dtype=np.int64)
            C = np.asarray(mask.col_idx[mask.col_ptr[b]:mask.col_ptr[b + 1]], dtype=np.int64)
            row_idx.extend(int(r) for r in R)
            col_idx.extend(int(j) for j in C)
            row_ptr.append(row_ptr[-1] + len(R))
            col_ptr.append(col_ptr[-1] + len(C))
            blk_ptr.append(blk_ptr[-1] + len(R) * len(C))
            if len(R) and len(C):
                sub = W[s * BR:(s + 1) * BR, c * BC:(c + 1) * BC][np.ix_(R, C)]
                chunks.append(np.ascontiguousarray(sub).reshape(-1))
    weights = np.concatenate(chunks) if chunks else np.zeros(0, dtype=W.dtype)
    return {
        "strip_order": np.asarray(order, dtype=np.int32),
        "row_ptr": np.asarray(row_ptr, dtype=np.int32),
        "row_idx": np.asarray(row_idx, dtype=np.uint16),
        "col_ptr": np.asarray(col_ptr, dtype=np.int32),
        "col_idx": np.asarray(col_idx, dtype=np.uint16),
        "blk_ptr": np.asarray(blk_ptr, dtype=np.int64),
        "weights": weights.astype(W.dtype, copy=False),
    }


def unpack(arrays: dict, M: int, K: int, BR: int, BC: int, dtype) -> np.ndarray:
    """Inverse of pack: the masked dense matrix (pruned positions are +0)."""
    nbr, nbc = M // BR, K // BC
    out = np.zeros((M, K), dtype=dtype)
    t = 0
    for s in arrays["strip_order"]:
        for c in range(nbc):
            R = arrays["row_idx"][arrays["row_ptr"][t]:arrays["row_ptr"][t + 1]].astype(np.int64)
            C = arrays["col_idx"][arrays["col_ptr"][t]:arrays["col_ptr"][t + 1]].astype(np.int64)
            w = arrays["weights"][arrays["blk_ptr"][t]:arrays["blk_ptr"][t + 1]]
            if len(R) and len(C):
                out[np.ix_(int(s) * BR + R, c * BC + C)] = w.reshape(len(R), len(C))
            t += 1
    return out
