"""LSTM cell around the BCR gate product (Section 3.1): pins of the fp64 reference (CPU) and parity of the GPU
cell kernel and of multi-step sequences against it (GPU)."""
import numpy as np
import pytest

import bcr_inputs as gen
from oracle import bcr_oracle as orc
from oracle import lstm_ref


# ------------------------------------------------------------------ pins of the reference (no GPU)
def test_reference_closed_forms():
    H, B = 5, 3
    c = np.linspace(-2, 2, H * B).reshape(H, B)
    # all pre-activations zero: i = f = o = 1/2, g = 0
    cn, hn = lstm_ref.cell(np.zeros((4 * H, B)), None, c)
    assert np.allclose(cn, 0.5 * c, rtol=0, atol=1e-15)
    assert np.allclose(hn, 0.5 * np.tanh(0.5 * c), rtol=0, atol=1e-15)
    # forget gate wide open, input gate shut, output gate open: the state passes through
    g = np.zeros((4 * H, B))
    g[:H] = -50.0
    g[H:2 * H] = 50.0
    g[3 * H:] = 50.0
    cn, hn = lstm_ref.cell(g, None, c)
    assert np.allclose(cn, c, atol=1e-12) and np.allclose(hn, np.tanh(c), atol=1e-12)
    # bias is added to the pre-activations: moving it between the two changes nothing
    rng = np.random.default_rng(3)
    gates, bias = rng.standard_normal((4 * H, B)), rng.standard_normal(4 * H)
    a = lstm_ref.cell(gates, bias, c)
    b = lstm_ref.cell(gates + bias[:, None], None, c)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    # tanh(x) = 2 sigmoid(2x) - 1
    x = np.linspace(-6, 6, 41)
    assert np.allclose(np.tanh(x), 2 * lstm_ref.sigmoid(2 * x) - 1, atol=1e-15)


def test_reference_matches_library_lstm_cell():
    """Same gate order and equations as torch.nn.LSTMCell (double precision, CPU)."""
    import torch
    I, H, B = 7, 6, 4
    rng = np.random.default_rng(11)
    cell = torch.nn.LSTMCell(I, H, bias=True, dtype=torch.float64)
    W = np.concatenate([cell.weight_ih.detach().numpy(), cell.weight_hh.detach().numpy()], axis=1)     # 4H x (I + H)
    bias = (cell.bias_ih + cell.bias_hh).detach().numpy()
    x, h, c = rng.standard_normal((B, I)), rng.standard_normal((B, H)), rng.standard_normal((B, H))
    h_t, c_t = cell(torch.from_numpy(x), (torch.from_numpy(h), torch.from_numpy(c)))
    xh = np.concatenate([x, h], axis=1).T                                                              # (I + H) x B
    _, c_ref, h_ref = lstm_ref.step(W, xh, bias, c.T)
    assert np.allclose(c_ref.T, c_t.detach().numpy(), rtol=0, atol=1e-14)
    assert np.allclose(h_ref.T, h_t.detach().numpy(), rtol=0, atol=1e-14)


# ------------------------------------------------------------------ GPU
def _gpu():
    import torch
    import paper_2108_11033_amd as g
    return torch, torch.device("cuda:0"), g


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("batch,pad", [(1, 0), (5, 2), (8, 0)])
def test_cell_kernel(dtype, batch, pad):
    from helpers import to_device
    torch, dev, g = _gpu()
    H = 300
    rng = np.random.default_rng(21)
    gates = (3.0 * rng.standard_normal((4 * H, batch))).astype(np.float32)
    gates[0, 0], gates[H, 0], gates[2 * H, 0], gates[3 * H, 0] = 90.0, -90.0, 40.0, -40.0      # saturated
    bias = rng.standard_normal(4 * H).astype(np.float32)
    c = rng.standard_normal((H, batch)).astype(np.float32)
    c_ref, h_ref = lstm_ref.cell(gates, bias, c)
    ld = batch + pad
    gd = torch.zeros((4 * H, ld), dtype=torch.float32, device=dev); gd[:, :batch] = torch.from_numpy(gates).to(dev)
    cd = torch.full((H, ld), 9.0, dtype=torch.float32, device=dev); cd[:, :batch] = torch.from_numpy(c).to(dev)
    tdt = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}[dtype]
    hd = torch.full((H, ld), 9.0, dtype=tdt, device=dev)
    h32 = torch.full((H, ld), 9.0, dtype=torch.float32, device=dev)
    g.lstm_cell(gd, ld, torch.from_numpy(bias).to(dev), cd, ld, hd, dtype, ld, h32, ld, H, batch, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.abs(cd[:, :batch].cpu().numpy() - c_ref).max() <= 2e-6 * max(1.0, np.abs(c_ref).max())
    assert np.abs(h32[:, :batch].cpu().numpy() - h_ref).max() <= 2e-6
    ulp = {gen.F32: 2e-6, gen.F16: 2.0 ** -10, gen.BF16: 2.0 ** -7}[dtype]          # storage rounding (fp32: the functions)
    assert np.abs(hd[:, :batch].float().cpu().numpy() - h_ref).max() <= ulp              # |h| < 1
    if pad:                                                                                   # nothing outside the batch columns
        assert (cd[:, batch:] == 9.0).all() and (hd[:, batch:].float() == 9.0).all() and (h32[:, batch:] == 9.0).all()
    # no bias, no h outputs
    cd2 = torch.from_numpy(c).to(dev).contiguous()
    g.lstm_cell(gd, ld, None, cd2, batch, None, dtype, 0, None, 0, H, batch, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.abs(cd2.cpu().numpy() - lstm_ref.cell(gates, None, c)[0]).max() <= 2e-6 * max(1.0, np.abs(c_ref).max())


@pytest.mark.gpu
@pytest.mark.parametrize("batch", [1, 4, 8, 32])
def test_sequence_of_steps(batch):
    """T steps of an LSTM layer whose gate matrix [W_ih | W_hh] is BCR-pruned: h is written by the cell straight into
    the lower part of the next step's input vector.  fp16 weights and activations, fp32 state."""
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    dtype, I, H, T = gen.F16, 64, 96, 6
    M, K, BR, BC = 4 * H, I + H, 32, 32
    mask = gen.random_mask(M, K, BR, BC, 8, 12, seed=600)
    W = gen.normal_weights(M, K, dtype, seed=601)
    W *= np.float16(8.0)                                       # pre-activations of order one
    xs = [gen.normal_activations(I, batch, dtype, seed=602 + t) for t in range(T)]
    bias = (0.1 * np.random.default_rng(603).standard_normal(M)).astype(np.float32)
    A = pack_workload(g, W, dtype, mask)
    Wm = orc.masked_dense(gen.storage_to_f64(W, dtype), BR, BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx)
    # device buffers: two [x; h] vectors used in turn
    xh = [torch.zeros((K, batch), dtype=torch.float16, device=dev) for _ in range(2)]
    gates = torch.empty((M, batch), dtype=torch.float32, device=dev)
    c = torch.zeros((H, batch), dtype=torch.float32, device=dev)
    h32 = torch.empty((H, batch), dtype=torch.float32, device=dev)
    bd = torch.from_numpy(bias).to(dev)
    stream = torch.cuda.current_stream()
    c_ref = np.zeros((H, batch)); h_ref = np.zeros((H, batch))
    for t in range(T):
        cur, nxt = xh[t % 2], xh[(t + 1) % 2]
        cur[:I] = to_device(xs[t], dtype)
        g.lstm_step(A, cur, batch, batch, gates, batch, bd, c, batch, nxt[I:], batch, h32, batch, stream)
        torch.cuda.synchronize()
        # the reference consumes what the device consumed: h rounded to fp16 as stored in the input vector
        xh_ref = np.concatenate([gen.storage_to_f64(xs[t], dtype), h_ref.astype(np.float16).astype(np.float64)], axis=0)
        _, c_ref, h_ref = lstm_ref.step(Wm, xh_ref, bias, c_ref)
        assert np.abs(c.cpu().numpy() - c_ref).max() <= TOL[dtype] * max(1.0, np.abs(c_ref).max()), f"c at step {t}"
        assert np.abs(h32.cpu().numpy() - h_ref).max() <= TOL[dtype], f"h at step {t}"
        assert np.abs(nxt[I:].float().cpu().numpy() - h_ref).max() <= TOL[dtype] + 2.0 ** -10
    assert np.abs(h_ref).max() > 0.05                          # the sequence did something
