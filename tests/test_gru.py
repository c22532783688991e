"""GRU cell around the BCR gate products (Section 6.1: the paper's RNN is a two-layer GRU): pins of the fp64
reference (CPU) and parity of the GPU cell kernel and of multi-step sequences against it (GPU)."""
import numpy as np
import pytest

import bcr_inputs as gen
from oracle import bcr_oracle as orc
from oracle import gru_ref


# ------------------------------------------------------------------ pins of the reference (no GPU)
def test_reference_closed_forms():
    H, B = 5, 3
    h = np.linspace(-1, 1, H * B).reshape(H, B)
    zero = np.zeros((3 * H, B))
    # all pre-activations zero: r = z = 1/2, n = 0  ->  h' = h / 2
    assert np.allclose(gru_ref.cell(zero, zero, None, None, h), 0.5 * h, rtol=0, atol=1e-15)
    # update gate wide open: the state passes through whatever the candidate is
    gi = np.random.default_rng(1).standard_normal((3 * H, B)); gi[H:2 * H] = 50.0
    assert np.allclose(gru_ref.cell(gi, zero, None, None, h), h, atol=1e-12)
    # update gate shut, reset gate shut: h' = tanh(input-side candidate); the hidden-side candidate is ignored
    gi = np.zeros((3 * H, B)); gh = np.zeros((3 * H, B))
    gi[:H] = -50.0; gi[H:2 * H] = -50.0
    gi[2 * H:] = np.linspace(-2, 2, H * B).reshape(H, B); gh[2 * H:] = 7.0
    assert np.allclose(gru_ref.cell(gi, gh, None, None, h), np.tanh(gi[2 * H:]), atol=1e-12)
    # reset gate open: the hidden-side candidate is added in full
    gi[:H] = 50.0; gh[2 * H:] = 0.3
    assert np.allclose(gru_ref.cell(gi, gh, None, None, h), np.tanh(gi[2 * H:] + 0.3), atol=1e-12)
    # the reset gate multiplies the hidden-side candidate INCLUDING its bias, not the input side's
    bh = np.zeros(3 * H); bh[2 * H:] = 0.4
    gi[:H] = 0.0                                                # r = 1/2
    assert np.allclose(gru_ref.cell(gi, gh, None, bh, h), np.tanh(gi[2 * H:] + 0.5 * (0.3 + 0.4)), atol=1e-12)
    bi = np.zeros(3 * H); bi[2 * H:] = 0.4
    assert np.allclose(gru_ref.cell(gi, gh, bi, None, h), np.tanh(gi[2 * H:] + 0.4 + 0.5 * 0.3), atol=1e-12)
    # biases of the r and z rows only enter through the sums
    rng = np.random.default_rng(3)
    gi, gh, bi, bh = rng.standard_normal((3 * H, B)), rng.standard_normal((3 * H, B)), rng.standard_normal(3 * H), rng.standard_normal(3 * H)
    a = gru_ref.cell(gi, gh, bi, bh, h)
    b = gru_ref.cell(gi + bi[:, None], gh + bh[:, None], None, None, h)
    assert np.array_equal(a, b)


def test_reference_matches_library_gru_cell():
    """Same gate order and equations as torch.nn.GRUCell (double precision, CPU)."""
    import torch
    I, H, B = 7, 6, 4
    rng = np.random.default_rng(11)
    cell = torch.nn.GRUCell(I, H, bias=True, dtype=torch.float64)
    Wi, Wh = cell.weight_ih.detach().numpy(), cell.weight_hh.detach().numpy()           # 3H x I, 3H x H
    bi, bh = cell.bias_ih.detach().numpy(), cell.bias_hh.detach().numpy()
    x, h = rng.standard_normal((B, I)), rng.standard_normal((B, H))
    h_t = cell(torch.from_numpy(x), torch.from_numpy(h)).detach().numpy()
    _, _, h_ref = gru_ref.step(Wi, Wh, x.T, h.T, bi, bh, h.T)
    assert np.allclose(h_ref.T, h_t, rtol=0, atol=1e-14)


# ------------------------------------------------------------------ GPU
def _gpu():
    import torch
    import paper_2108_11033_amd as g
    return torch, torch.device("cuda:0"), g


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("batch,pad", [(1, 0), (5, 2), (32, 0)])
def test_cell_kernel(dtype, batch, pad):
    torch, dev, g = _gpu()
    H = 300
    rng = np.random.default_rng(21)
    gi = (2.0 * rng.standard_normal((3 * H, batch))).astype(np.float32)
    gh = (2.0 * rng.standard_normal((3 * H, batch))).astype(np.float32)
    gi[0, 0], gi[H, 0], gi[2 * H, 0], gh[1, 0], gh[H + 1, 0] = 90.0, -90.0, 40.0, -90.0, 90.0      # saturated
    bi, bh = rng.standard_normal(3 * H).astype(np.float32), rng.standard_normal(3 * H).astype(np.float32)
    h = rng.standard_normal((H, batch)).astype(np.float32)
    h_ref = gru_ref.cell(gi, gh, bi, bh, h)
    ld = batch + pad
    def padded(a, fill=0.0):
        t = torch.full((a.shape[0], ld), fill, dtype=torch.float32, device=dev)
        t[:, :batch] = torch.from_numpy(a).to(dev)
        return t
    gid, ghd, h32 = padded(gi), padded(gh), padded(h, 9.0)
    tdt = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}[dtype]
    hd = torch.full((H, ld), 9.0, dtype=tdt, device=dev)
    g.gru_cell(gid, ld, ghd, ld, torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev), h32, ld, hd, dtype, ld, H, batch,
               torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.abs(h32[:, :batch].cpu().numpy() - h_ref).max() <= 4e-6 * max(1.0, np.abs(h_ref).max())
    ulp = {gen.F32: 4e-6, gen.F16: 2.0 ** -10, gen.BF16: 2.0 ** -7}[dtype]              # storage rounding (fp32: the functions)
    assert np.abs(hd[:, :batch].float().cpu().numpy() - h_ref).max() <= ulp * max(1.0, np.abs(h_ref).max())
    if pad:                                                                               # nothing outside the batch columns
        assert (h32[:, batch:] == 9.0).all() and (hd[:, batch:].float() == 9.0).all()
    # no biases, no typed copy
    h2 = torch.from_numpy(h).to(dev).contiguous()
    g.gru_cell(gid, ld, ghd, ld, None, None, h2, batch, None, dtype, 0, H, batch, torch.cuda.current_stream())
    torch.cuda.synchronize()
    r2 = gru_ref.cell(gi, gh, None, None, h)
    assert np.abs(h2.cpu().numpy() - r2).max() <= 4e-6 * max(1.0, np.abs(r2).max())


@pytest.mark.gpu
@pytest.mark.parametrize("batch", [1, 4, 12, 32, 60, 64])
def test_sequence_of_steps(batch):
    """T steps of a GRU layer whose two gate matrices are BCR-pruned; the cell writes the new state in fp16 into the
    buffer the next step's hidden-side product reads.  Batch 32 (the paper's GRU measurement) runs the products on the
    SpMM kernels -- 4 to 60 columns as one launch for both products (12: rows of X not 16-byte aligned), 64 as two --,
    1 on the SpMV kernels."""
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    dtype, I, H, T = gen.F16, 64, 96, 6
    M, BR, BC = 3 * H, 16, 32
    mi = gen.random_mask(M, I, BR, BC, 8, 12, seed=610)
    mh = gen.random_mask(M, H, BR, BC, 8, 12, seed=611)
    Wi = gen.normal_weights(M, I, dtype, seed=612) * np.float16(6.0)       # pre-activations of order one
    Wh = gen.normal_weights(M, H, dtype, seed=613) * np.float16(6.0)
    xs = [gen.normal_activations(I, batch, dtype, seed=614 + t) for t in range(T)]
    rng = np.random.default_rng(615)
    bi, bh = (0.1 * rng.standard_normal(M)).astype(np.float32), (0.1 * rng.standard_normal(M)).astype(np.float32)
    Ai, Ah = pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh)
    Wim = orc.masked_dense(gen.storage_to_f64(Wi, dtype), BR, BC, mi.row_ptr, mi.row_idx, mi.col_ptr, mi.col_idx)
    Whm = orc.masked_dense(gen.storage_to_f64(Wh, dtype), BR, BC, mh.row_ptr, mh.row_idx, mh.col_ptr, mh.col_idx)
    hbuf = torch.zeros((H, batch), dtype=torch.float16, device=dev)        # the state as the product reads it
    h32 = torch.zeros((H, batch), dtype=torch.float32, device=dev)
    gi = torch.empty((M, batch), dtype=torch.float32, device=dev)
    gh = torch.empty((M, batch), dtype=torch.float32, device=dev)
    bid, bhd = torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev)
    stream = torch.cuda.current_stream()
    h_ref = np.zeros((H, batch))
    for t in range(T):
        x = to_device(xs[t], dtype)
        g.gru_step(Ai, Ah, x, batch, hbuf, batch, batch, gi, batch, gh, batch, bid, bhd, h32, batch, hbuf, batch, stream)
        torch.cuda.synchronize()
        # the reference consumes what the device consumed: the state rounded to fp16 for the product, fp32 for the blend
        hin = h_ref.astype(np.float16).astype(np.float64)
        _, _, h_ref = gru_ref.step(Wim, Whm, gen.storage_to_f64(xs[t], dtype), hin, bi, bh, h_ref)
        assert np.abs(h32.cpu().numpy() - h_ref).max() <= 2 * TOL[dtype], f"h at step {t}"
        assert np.abs(hbuf.float().cpu().numpy() - h_ref).max() <= 2 * TOL[dtype] + 2.0 ** -10
    assert np.abs(h_ref).max() > 0.05                          # the sequence did something


@pytest.mark.gpu
@pytest.mark.parametrize("batch,uniform,x_first", [(1, True, True), (1, False, False), (4, True, False), (8, False, True),
                                                   (3, True, True)])
def test_sequence_equal_widths_one_launch(batch, uniform, x_first):
    """Input width = hidden width and at most 8 columns: both gate products leave in one launch, the hidden-side
    operands addressed as the input-side ones plus a stride.  Both signs of the stride (x before h and after it in
    memory, likewise the two results), uniformly and unevenly pruned matrices (different kernels)."""
    from helpers import pack_workload, TOL
    torch, dev, g = _gpu()
    dtype, H, T = gen.F16, 96, 5
    M, BR, BC = 3 * H, 16, 32
    kept = (8, 12) if uniform else ((4, 8, 16), (8, 12, 20))
    mi = gen.random_mask(M, H, BR, BC, kept[0], kept[1], seed=620)
    mh = gen.random_mask(M, H, BR, BC, kept[0], kept[1], seed=621)
    Wi = gen.normal_weights(M, H, dtype, seed=622) * np.float16(6.0)
    Wh = gen.normal_weights(M, H, dtype, seed=623) * np.float16(6.0)
    xs = [gen.normal_activations(H, batch, dtype, seed=624 + t) for t in range(T)]
    rng = np.random.default_rng(625)
    bi, bh = (0.1 * rng.standard_normal(M)).astype(np.float32), (0.1 * rng.standard_normal(M)).astype(np.float32)
    Ai, Ah = pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh)
    Wim = orc.masked_dense(gen.storage_to_f64(Wi, dtype), BR, BC, mi.row_ptr, mi.row_idx, mi.col_ptr, mi.col_idx)
    Whm = orc.masked_dense(gen.storage_to_f64(Wh, dtype), BR, BC, mh.row_ptr, mh.row_idx, mh.col_ptr, mh.col_idx)
    xh = torch.zeros((2, H, batch), dtype=torch.float16, device=dev)       # x and the state in one allocation
    gates = torch.full((2, M, batch), float("nan"), dtype=torch.float32, device=dev)
    xbuf, hbuf = (xh[0], xh[1]) if x_first else (xh[1], xh[0])
    gi, gh = (gates[0], gates[1]) if x_first else (gates[1], gates[0])
    h32 = torch.zeros((H, batch), dtype=torch.float32, device=dev)
    bid, bhd = torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev)
    stream = torch.cuda.current_stream()
    h_ref = np.zeros((H, batch))
    for t in range(T):
        xbuf.copy_(torch.from_numpy(xs[t]).to(dev))
        g.gru_step(Ai, Ah, xbuf, batch, hbuf, batch, batch, gi, batch, gh, batch, bid, bhd, h32, batch, hbuf, batch, stream)
        torch.cuda.synchronize()
        hin = h_ref.astype(np.float16).astype(np.float64)
        gi_ref, gh_ref, h_ref = gru_ref.step(Wim, Whm, gen.storage_to_f64(xs[t], dtype), hin, bi, bh, h_ref)
        assert np.abs(h32.cpu().numpy() - h_ref).max() <= 2 * TOL[dtype], f"h at step {t}"
        assert np.abs(hbuf.float().cpu().numpy() - h_ref).max() <= 2 * TOL[dtype] + 2.0 ** -10
    # the two products of the last step, element by element, against separate products of the same operands
    gi2 = torch.empty((M, batch), dtype=torch.float32, device=dev)
    g.spmv(Ai, xbuf, batch, batch, gi2, batch, stream)
    torch.cuda.synchronize()
    if batch != 8:                                             # (a lone product of 8 columns runs on the matrix cores)
        assert torch.equal(gi, gi2)                            # same kernel, same order of additions
    assert np.abs(gi2.cpu().numpy() - gi_ref).max() <= 2 * TOL[dtype] * np.abs(gi_ref).max()
    assert np.abs(gi.cpu().numpy() - gi_ref).max() <= 2 * TOL[dtype] * np.abs(gi_ref).max()
    assert np.abs(h_ref).max() > 0.05


@pytest.mark.gpu
def test_step_refusals():
    from helpers import pack_workload
    from paper_2108_11033_amd import GrimError
    torch, dev, g = _gpu()
    dtype, H = gen.F16, 32
    A3 = pack_workload(g, gen.normal_weights(3 * H, 64, dtype, seed=1), dtype, gen.random_mask(3 * H, 64, 16, 32, 8, 8, seed=2))
    Ah = pack_workload(g, gen.normal_weights(3 * H, H, dtype, seed=3), dtype, gen.random_mask(3 * H, H, 16, 32, 8, 8, seed=4))
    Abad = pack_workload(g, gen.normal_weights(3 * H, 64, dtype, seed=5), dtype, gen.random_mask(3 * H, 64, 16, 32, 8, 8, seed=6))
    x = torch.zeros((64, 1), dtype=torch.float16, device=dev)
    h = torch.zeros((H, 1), dtype=torch.float16, device=dev)
    gi = torch.zeros((3 * H, 1), dtype=torch.float32, device=dev)
    gh = torch.zeros((3 * H, 1), dtype=torch.float32, device=dev)
    h32 = torch.full((H, 1), 5.0, dtype=torch.float32, device=dev)
    with pytest.raises(GrimError) as e:                        # hidden-side matrix must be 3H x H
        g.gru_step(A3, Abad, x, 1, h, 1, 1, gi, 1, gh, 1, None, None, h32, 1, h, 1)
    assert e.value.name == "GRIM_ERR_SHAPE"
    with pytest.raises(GrimError) as e:
        g.gru_step(A3, Ah, x, 1, h, 1, 0, gi, 1, gh, 1, None, None, h32, 1, h, 1)
    assert e.value.name == "GRIM_ERR_SHAPE"
    with pytest.raises(GrimError) as e:
        g.gru_step(A3, Ah, x, 1, h, 1, 1, gi, 1, gh, 1, None, None, None, 1, h, 1)
    assert e.value.name == "GRIM_ERR_NULL"
    torch.cuda.synchronize()
    assert (h32 == 5.0).all()
