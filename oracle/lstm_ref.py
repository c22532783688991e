"""Test infrastructure only -- fp64 reference of one LSTM step around the BCR gate product.

Section 3.1 of the paper treats the gate matrices of an RNN layer as one matrix-vector product per
time step; the cell equations are the standard LSTM ones (the paper evaluates LSTM/GRU layers but does
not restate them).  Gate rows are stacked input, forget, cell candidate, output -- this build's
convention, the same as torch.nn.LSTMCell's, which is what pins this module (tests/test_lstm.py).
"""
from __future__ import annotations

import numpy as np


def sigmoid(v: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-v))


def cell(gates: np.ndarray, bias, c: np.ndarray):
    """gates: 4H x B pre-activations, bias: 4H or None, c: H x B  ->  (c_next, h_next), all fp64."""
    gates = np.asarray(gates, dtype=np.float64)
    H = gates.shape[0] // 4
    if bias is not None:
        gates = gates + np.asarray(bias, dtype=np.float64)[:, None]
    i, f = sigmoid(gates[:H]), sigmoid(gates[H:2 * H])
    g, o = np.tanh(gates[2 * H:3 * H]), sigmoid(gates[3 * H:])
    c_next = f * np.asarray(c, dtype=np.float64) + i * g
    return c_next, o * np.tanh(c_next)


def step(W_masked64: np.ndarray, xh64: np.ndarray, bias, c: np.ndarray):
    """One step with the masked dense gate matrix (4H x (I + H)) and the stacked input [x; h]."""
    gates = W_masked64 @ xh64
    c_next, h_next = cell(gates, bias, c)
    return gates, c_next, h_next
