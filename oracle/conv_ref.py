"""Test infrastructure only -- fp64 reference of a stride-1 "same" convolution with a BCR-pruned filter matrix.

Section 3.1 of the paper computes a CONV layer as the filter matrix (Cout rows; one column per (input channel,
kernel row, kernel column)) times the im2col matrix of the input feature map; Section 4.5 notes that the
generated code skips the rows of that matrix whose weights are all pruned.  This module states the result
directly, without forming the im2col matrix:

    Y[m, h, w] = sum over (cin, r, q) of  Wm[m, cin, r, q] * F[cin, h + r - kh // 2, w + q - kw // 2]

with F taken as zero outside the image, Wm the BCR-masked filter matrix reshaped to [M][Cin][kh][kw] -- column
k = cin * kh * kw + r * kw + q, this build's reading (the paper does not fix the order; it is the order of the
common unfold / weight.reshape(Cout, -1) convention, which is what pins it against the library routine).
"""
from __future__ import annotations

import numpy as np


def conv_same(Wm64: np.ndarray, F64: np.ndarray, kh: int, kw: int) -> np.ndarray:
    """Wm64: M x (Cin * kh * kw) masked filter matrix, F64: Cin x H x W  ->  Y: M x H x W (fp64)."""
    Cin, H, W = F64.shape
    M = Wm64.shape[0]
    Wr = Wm64.reshape(M, Cin, kh, kw)
    ph, pw = kh // 2, kw // 2
    Fp = np.zeros((Cin, H + 2 * ph, W + 2 * pw), dtype=np.float64)
    Fp[:, ph:ph + H, pw:pw + W] = F64
    Y = np.zeros((M, H, W), dtype=np.float64)
    for r in range(kh):
        for q in range(kw):
            # one kernel tap: a 1x1 convolution of the shifted image
            Y += np.einsum("mc,chw->mhw", Wr[:, :, r, q], Fp[:, r:r + H, q:q + W])
    return Y


def conv2d(Wm64: np.ndarray, F64: np.ndarray, kh: int, kw: int, stride: int = 1) -> np.ndarray:
    """A batch of images at a stride, padding kh // 2 and kw // 2 (the layers of the evaluated networks, Section 6.1):
    Wm64: M x (Cin * kh * kw), F64: B x Cin x H x W  ->  B x M x Ho x Wo with Ho = ceil(H / stride), Wo = ceil(W / stride),

        Y[b, m, ho, wo] = sum over (cin, r, q) of  Wm[m, cin, r, q] * F[b, cin, stride * ho + r - kh // 2, stride * wo + q - kw // 2]

    Written out per image and per kernel tap on the strided view of the padded image."""
    B, Cin, H, W = F64.shape
    M = Wm64.shape[0]
    Wr = Wm64.reshape(M, Cin, kh, kw)
    ph, pw = kh // 2, kw // 2
    Ho, Wo = -(-H // stride), -(-W // stride)
    Y = np.zeros((B, M, Ho, Wo), dtype=np.float64)
    for b in range(B):
        Fp = np.zeros((Cin, H + 2 * ph, W + 2 * pw), dtype=np.float64)
        Fp[:, ph:ph + H, pw:pw + W] = F64[b]
        for r in range(kh):
            for q in range(kw):
                # padded coordinates of tap (r, q) at output (ho, wo): (stride * ho + r, stride * wo + q)
                view = Fp[:, r:r + stride * (Ho - 1) + 1:stride, q:q + stride * (Wo - 1) + 1:stride]
                Y[b] += np.einsum("mc,chw->mhw", Wr[:, :, r, q], view)
    return Y


def abs_scale(Wm64: np.ndarray, F64: np.ndarray, kh: int, kw: int) -> np.ndarray:
    """S[m, h, w] = sum of |terms|, the scale the error is measured against."""
    return conv_same(np.abs(Wm64), np.abs(F64), kh, kw)


def im2col(F64: np.ndarray, kh: int, kw: int) -> np.ndarray:
    """The matrix of Section 3.1: (Cin * kh * kw) x (H * W), row k = cin * kh * kw + r * kw + q."""
    Cin, H, W = F64.shape
    ph, pw = kh // 2, kw // 2
    Fp = np.zeros((Cin, H + 2 * ph, W + 2 * pw), dtype=F64.dtype)
    Fp[:, ph:ph + H, pw:pw + W] = F64
    X = np.empty((Cin * kh * kw, H * W), dtype=F64.dtype)
    for cin in range(Cin):
        for r in range(kh):
            for q in range(kw):
                X[(cin * kh + r) * kw + q] = Fp[cin, r:r + H, q:q + W].reshape(-1)
    return X


def layer(W_masked64: np.ndarray, F64: np.ndarray, kh: int, kw: int, bias=None, relu: bool = False) -> np.ndarray:
    """A CONV layer as the evaluated networks chain them: convolution, bias per output channel, rectifier.
    fp64 throughout; the caller rounds to the storage type of the next layer's input."""
    Y = conv_same(W_masked64, F64, kh, kw)
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[:, None, None]
    return np.maximum(Y, 0.0) if relu else Y
