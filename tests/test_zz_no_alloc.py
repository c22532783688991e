"""grim_bcr_lstm_sequence_noalloc (the entry point for callers that cannot allocate: its exchange words live in a
static device array of the library) against grim_bcr_lstm_sequence on the same operands, bit for bit, on two calls in a
row, the second one smaller in every size -- the array keeps the first call's contents, which the second must not see."""
import numpy as np
import pytest

import bcr_inputs as gen

pytestmark = pytest.mark.gpu


def _case(torch, dev, g, dtype, H, I, T, seed):
    from helpers import to_device, pack_workload
    M, K = 4 * H, I + H
    mask = gen.random_mask(M, K, 32, 32, 8, 12, seed=seed)
    W = gen.normal_weights(M, K, dtype, seed=seed + 1)
    W = gen.round_to_storage(gen.storage_to_f64(W, dtype).astype(np.float32) * 4.0, dtype)
    A = pack_workload(g, W, dtype, mask)
    rng = np.random.default_rng(seed + 2)
    xs = to_device(np.ascontiguousarray(gen.normal_activations(I, T, dtype, seed=seed + 3).T), dtype)
    h0 = to_device(gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype), dtype)
    c0 = torch.from_numpy(rng.standard_normal(H).astype(np.float32)).to(dev)
    bias = torch.from_numpy((0.2 * rng.standard_normal(M)).astype(np.float32)).to(dev)
    return A, xs, h0, c0, bias


def _run(torch, dev, fn, A, xs, h0, c0, bias, H, I, T):
    c = c0.clone()
    hs = torch.full((T, H), 7.0, dtype=xs.dtype, device=dev)
    hs32 = torch.full((T, H), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    fn(A, xs, I, T, bias, h0, c, hs, H, hs32, H, status, 0, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    return hs.float().cpu().numpy(), hs32.cpu().numpy(), c.cpu().numpy()


def test_noalloc_sequence_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    import torch
    import paper_2108_11033_amd as g
    g.load_library()
    dev = torch.device("cuda:0")
    dtype = gen.F16
    for H, I, T, seed in [(1024, 512, 24, 1700), (256, 64, 5, 1710)]:      # the second call is smaller in H, I and T
        A, xs, h0, c0, bias = _case(torch, dev, g, dtype, H, I, T, seed)
        got = _run(torch, dev, g.lstm_sequence_noalloc, A, xs, h0, c0, bias, H, I, T)
        want = _run(torch, dev, g.lstm_sequence, A, xs, h0, c0, bias, H, I, T)
        for a, b, what in zip(got, want, ("h", "h in fp32", "c")):
            assert np.isfinite(a).all(), f"H={H}: {what} not finite"
            assert np.array_equal(a, b), f"H={H}: {what} differs from grim_bcr_lstm_sequence"
        assert np.abs(got[1][-1]).max() > 0.01


def test_noalloc_sequence_refuses_what_does_not_fit():
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload
    g.load_library()
    dev = torch.device("cuda:0")
    H, I = 64, 64
    m = gen.random_mask(4 * H, I + H, 32, 32, 10, 10, seed=1720)              # kept counts no sequence kernel is built for
    W = gen.normal_weights(4 * H, I + H, gen.F16, seed=1721)
    A = pack_workload(g, W, gen.F16, m)
    z16 = torch.zeros((4, H), dtype=torch.float16, device=dev)
    c = torch.zeros((H,), dtype=torch.float32, device=dev)
    status = torch.zeros((1,), dtype=torch.int32, device=dev)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence_noalloc(A, z16, I, 4, None, z16[0], c, z16.clone(), H, None, 0, status)
    assert "UNSUPPORTED" in str(e.value)
    torch.cuda.synchronize()
