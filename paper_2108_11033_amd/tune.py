"""Block-size selection by measurement (Section 5.1 of the paper, "Block Size Optimization").

The paper chooses a layer's block size offline: for each candidate size it synthesises a layer of the same
shape whose weights are random but satisfy the pruning rate and the block size (latency depends on the rate,
not on where the survivors sit), times it on the target device, and walks the candidates while each next one
still buys a worthwhile speed-up; the last size that did is the answer -- the smallest block (best accuracy)
from which larger blocks no longer pay.  This module does the same on the GPU through the library: masks and
values come from the seeded generators, timing is by HIP events on the caller's stream.

Nothing here computes the product itself; it only packs, launches and times.
"""
from __future__ import annotations

import math
from typing import Callable, Iterable, List, Optional, Sequence, Tuple

import numpy as np


def kept_counts(BR: int, BC: int, rate: float, row_frac: Optional[float] = None) -> Tuple[int, int]:
    """Kept rows and columns per block for a compression `rate` (dense / kept): rows take `row_frac` of the block
    (default: the square root of the kept fraction, i.e. rows and columns pruned alike), columns what is left."""
    keep = 1.0 / rate
    f = math.sqrt(keep) if row_frac is None else row_frac
    kr = min(BR, max(1, round(BR * f)))
    kc = min(BC, max(1, round(BR * BC * keep / kr)))
    return kr, kc


def synthesize(M: int, K: int, N: int, BR: int, BC: int, rate: float, dtype: str, seed: int = 0, row_frac=None):
    """A layer of the given shape with random weights under a uniform random BCR mask of the given rate."""
    import bcr_inputs as gen
    kr, kc = kept_counts(BR, BC, rate, row_frac)
    mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=7000 + seed)
    W = gen.normal_weights(M, K, dtype, seed=7001 + seed)
    X = gen.normal_activations(K, N, dtype, seed=7002 + seed, relu=True) if N > 8 else gen.normal_activations(K, N, dtype, seed=7002 + seed)
    return W, X, mask


def choose(candidates: Sequence[Tuple[int, int]], latency_of: Callable[[Tuple[int, int]], float],
           threshold: float = 1.1):
    """Walk `candidates` in the caller's order (small blocks first) and keep moving to the next size while it is
    at least `threshold` times faster than the best so far; return (chosen size, [(size, latency), ...])."""
    trace: List[Tuple[Tuple[int, int], float]] = []
    best, best_t = None, math.inf
    for size in candidates:
        t = float(latency_of(size))
        trace.append((size, t))
        if best is not None and best_t / t < threshold:
            break
        best, best_t = size, t
    return best, trace


def time_layer(W, X, mask, dtype: str, steps: int = 50, warmup: int = 5, products: int = 1, **pack_kw) -> float:
    """Seconds per product of one synthesised layer on the current GPU (SpMM, or SpMV when X has <= 8 columns;
    `products` > 1 times that many independent copies through one batched SpMV launch)."""
    import torch
    import bcr_inputs as gen
    from . import binding
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    K, N = X.shape
    M = W.shape[0]

    def to_dev(a):
        if dtype == gen.BF16:
            return torch.from_numpy(a.view(np.int16).copy()).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    A = binding.pack(W, dtype, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, **pack_kw)
    if N <= 8 and products > 1:
        mats = [A] + [binding.pack(W, dtype, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx,
                                   **pack_kw) for _ in range(products - 1)]
        G = binding.group(mats)
        xd = to_dev(np.stack([X] * products))
        yd = torch.empty((products, M, N), dtype=torch.float32, device=dev)
        run = lambda: binding.spmv_batched(G, xd, K * N, N, N, yd, M * N, N, stream)   # noqa: E731
    else:
        xd = to_dev(X)
        yd = torch.empty((M, N), dtype=torch.float32, device=dev)
        run = lambda: binding.spmm(A, xd, N, N, yd, N, stream)                            # noqa: E731
        products = 1
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        run()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / steps / products


def find_block_size(M: int, K: int, N: int, rate: float, candidates: Iterable[Tuple[int, int]], dtype: str = "f16",
                    threshold: float = 1.1, products: int = 1, row_frac=None, **time_kw):
    """The paper's search for one layer shape: candidates that divide the layer, smallest block first."""
    sizes = [s for s in candidates if M % s[0] == 0 and K % s[1] == 0]

    def latency(size):
        W, X, mask = synthesize(M, K, N, size[0], size[1], rate, dtype, row_frac=row_frac)
        return time_layer(W, X, mask, dtype, products=products, **time_kw)
    return choose(sizes, latency, threshold)
