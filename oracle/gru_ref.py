"""Test infrastructure only -- fp64 reference of one GRU step around the BCR gate products.

Section 6.1 of the paper evaluates a two-layer GRU; Section 3.1 treats an RNN layer's gate matrices as
matrix-vector products.  The paper does not restate the cell; this is the standard GRU with the reset
gate applied to the hidden-side candidate product (the form torch.nn.GRUCell computes, which is what
pins this module in tests/test_gru.py).  Gate rows are stacked reset, update, candidate in both
products: gi = W_i x (3H x B), gh = W_h h (3H x B).
"""
from __future__ import annotations

import numpy as np


def sigmoid(v: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-v))


def cell(gi: np.ndarray, gh: np.ndarray, bias_i, bias_h, h: np.ndarray) -> np.ndarray:
    """gi, gh: 3H x B pre-activations of the input and hidden products; biases 3H or None; h: H x B.
    Returns the next hidden state, fp64."""
    gi = np.asarray(gi, dtype=np.float64)
    gh = np.asarray(gh, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    H = h.shape[0]
    if bias_i is not None:
        gi = gi + np.asarray(bias_i, dtype=np.float64)[:, None]
    if bias_h is not None:
        gh = gh + np.asarray(bias_h, dtype=np.float64)[:, None]
    r = sigmoid(gi[:H] + gh[:H])
    z = sigmoid(gi[H:2 * H] + gh[H:2 * H])
    n = np.tanh(gi[2 * H:] + r * gh[2 * H:])
    return (1.0 - z) * n + z * h


def step(Wi_masked64: np.ndarray, Wh_masked64: np.ndarray, x64: np.ndarray, hin64: np.ndarray, bias_i, bias_h,
         h: np.ndarray):
    """One step with the masked dense gate matrices (3H x I and 3H x H).  `hin64` is the hidden state as the
    product reads it (storage precision, widened), `h` the fp32 state the cell blends with."""
    gi = Wi_masked64 @ x64
    gh = Wh_masked64 @ hin64
    return gi, gh, cell(gi, gh, bias_i, bias_h, h)
