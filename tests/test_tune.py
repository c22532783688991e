"""Block-size selection (Section 5.1): the search rule on injected latencies (CPU), and one real search (GPU)."""
import math

import pytest

from paper_2108_11033_amd import tune


def test_kept_counts_hit_the_rate():
    for BR, BC, rate in ((16, 32, 8), (32, 32, 10), (16, 16, 4), (4, 4, 16), (64, 64, 10)):
        kr, kc = tune.kept_counts(BR, BC, rate)
        assert 1 <= kr <= BR and 1 <= kc <= BC
        assert abs(kr * kc / (BR * BC) - 1 / rate) <= 0.5 / min(BR, BC) + 0.02
    assert tune.kept_counts(16, 32, 8, row_frac=0.5) == (8, 8)          # c2's split: half the rows, a quarter of the columns


def test_search_stops_when_the_gain_is_small():
    lat = {(4, 4): 100.0, (8, 8): 60.0, (16, 16): 40.0, (32, 32): 38.0, (64, 64): 10.0}
    sizes = list(lat)
    best, trace = tune.choose(sizes, lat.__getitem__, threshold=1.1)
    assert best == (16, 16)                                             # 40 -> 38 is under 10 %: stop, keep 16x16
    assert [s for s, _ in trace] == sizes[:4]                           # 64x64 is never timed
    best, _ = tune.choose(sizes, lat.__getitem__, threshold=1.0)
    assert best == (64, 64)
    best, trace = tune.choose(sizes, lambda s: 5.0, threshold=1.1)      # flat latency: the smallest block wins
    assert best == (4, 4) and len(trace) == 2
    assert tune.choose([], lat.__getitem__) == (None, [])


@pytest.mark.gpu
def test_search_on_the_gpu():
    best, trace = tune.find_block_size(256, 1024, 512, 8.0, [(16, 16), (16, 32), (32, 32), (64, 64), (7, 7)],
                                       dtype="f16", threshold=1.05, steps=20, warmup=3, row_frac=0.5)
    assert best in {(16, 16), (16, 32), (32, 32), (64, 64)}
    assert all(math.isfinite(t) and t > 0 for _, t in trace) and (7, 7) not in [s for s, _ in trace]
