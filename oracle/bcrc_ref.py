"""Test infrastructure only -- reference construction of the paper's BCRC arrays.

Section 4.3 ("Compact Model Storage") describes six arrays: reorder, row offset, occurrence, column
stride, compact column and weights.  This module builds them straight from the DENSE picture -- the
boolean keep matrix of the mask and the dense weight matrix -- and never looks at the library's
compact arrays, so that the library's export can be checked against it byte for byte.

Reading of the text (its figure is not available): rows with the same set of kept columns form a
group; groups are ordered by the first original row that shows the pattern and rows inside a group
ascend -- which reproduces every value the text quotes (reorder starts 0, 3; row offset 0, 3; column
stride 0, 3; the first row's columns 0, 3, 6; occurrence 0, 2).  Rows that keep nothing form one group
with an empty list.  Parity of the group ORDER beyond those quoted values is unpinned by the paper.
"""
from __future__ import annotations

import numpy as np


def keep_matrix(mask) -> np.ndarray:
    """M x K boolean matrix: True where the BCR mask keeps the weight (Section 3.2)."""
    keep = np.zeros((mask.M, mask.K), dtype=bool)
    nbc = mask.K // mask.BC
    for b in range((mask.M // mask.BR) * nbc):
        s, c = divmod(b, nbc)
        rows = mask.row_idx[mask.row_ptr[b]:mask.row_ptr[b + 1]].astype(np.int64) + s * mask.BR
        cols = mask.col_idx[mask.col_ptr[b]:mask.col_ptr[b + 1]].astype(np.int64) + c * mask.BC
        if len(rows) and len(cols):
            keep[np.ix_(rows, cols)] = True
    return keep


def bcrc(W: np.ndarray, keep: np.ndarray) -> dict:
    """The six arrays for dense W (any dtype; values are copied bit for bit) under `keep`."""
    M, K = keep.shape
    order = {}
    groups = []
    for r in range(M):
        key = tuple(np.nonzero(keep[r])[0].tolist())
        if key not in order:
            order[key] = len(groups)
            groups.append((key, []))
        groups[order[key]][1].append(r)
    reorder, row_offset, occurrence, column_stride, compact_column, weights = [], [0], [0], [0], [], []
    for key, rows in groups:
        compact_column.extend(key)
        column_stride.append(len(compact_column))
        for r in rows:
            reorder.append(r)
            weights.append(W[r, list(key)])
            row_offset.append(row_offset[-1] + len(key))
        occurrence.append(len(reorder))
    w = np.concatenate(weights) if weights else np.zeros(0, dtype=W.dtype)
    return {"reorder": np.array(reorder, dtype=np.int32), "row_offset": np.array(row_offset, dtype=np.int64),
            "occurrence": np.array(occurrence, dtype=np.int32), "column_stride": np.array(column_stride, dtype=np.int64),
            "compact_column": np.array(compact_column, dtype=np.int32), "weights": w.astype(W.dtype)}


def to_dense(b: dict, M: int, K: int) -> np.ndarray:
    """Inverse: the masked dense matrix the six arrays describe."""
    W = np.zeros((M, K), dtype=b["weights"].dtype)
    for g in range(len(b["occurrence"]) - 1):
        cols = b["compact_column"][b["column_stride"][g]:b["column_stride"][g + 1]]
        for p in range(b["occurrence"][g], b["occurrence"][g + 1]):
            W[b["reorder"][p], cols] = b["weights"][b["row_offset"][p]:b["row_offset"][p + 1]]
    return W


def index_bytes(b: dict, M: int) -> dict:
    """Bytes of everything that is not a weight, for BCRC and for CSR of the same matrix (the quantity of the
    paper's BCRC-versus-CSR figure), 32-bit indices and offsets throughout as in the text's example."""
    nnz = int(b["row_offset"][-1])
    bcrc_b = 4 * (len(b["reorder"]) + len(b["row_offset"]) + len(b["occurrence"]) + len(b["column_stride"])
                  + len(b["compact_column"]))
    csr_b = 4 * (M + 1 + nnz)
    return {"bcrc": bcrc_b, "csr": csr_b, "saving": 1.0 - bcrc_b / csr_b if csr_b else 0.0}
