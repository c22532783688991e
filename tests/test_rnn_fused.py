"""Recurrent steps as ONE launch: the gate product(s) with the LSTM / GRU cell in the epilogue (Section 3.1: an RNN layer
is one matrix-vector product per time step; the cell is the elementwise rest).  The fused step is compared with the
product followed by the cell kernel on the same operands (gate pre-activations bit for bit: same kernel family, same
order of additions) and with the fp64 references over sequences, the new state going to a second buffer each step."""
import numpy as np
import pytest

import bcr_inputs as gen
from oracle import bcr_oracle as orc
from oracle import gru_ref, lstm_ref

pytestmark = pytest.mark.gpu


def _gpu():
    import torch
    import paper_2108_11033_amd as g
    g.load_library()
    return torch, torch.device("cuda:0"), g


def _tdt(torch, dtype):
    return {gen.F16: torch.float16, gen.BF16: torch.bfloat16}[dtype]


def _masked(W, dtype, m):
    return orc.masked_dense(gen.storage_to_f64(W, dtype), m.BR, m.BC, m.row_ptr, m.row_idx, m.col_ptr, m.col_idx)


def _round(a, dtype):
    return gen.storage_to_f64(gen.round_to_storage(np.asarray(a, dtype=np.float32), dtype), dtype)


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,BC,kr,kc,ld", [
    (128, 64, 32, 32, 8, 12, 1),      # the LSTM workload's block shape, 4 workgroups
    (96, 32, 16, 32, 8, 8, 1),        # 16-row blocks: 6 hidden-unit groups
    (64, 192, 32, 32, 4, 16, 3),      # strided vectors (element-wise staging of x), one segment of 8 blocks
    (32, 2272, 32, 32, 16, 8, 1),     # 72 column blocks: two segments per strip, one workgroup
])
def test_lstm_step_in_one_launch(dtype, H, I, BR, BC, kr, kc, ld):
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    M, K = 4 * H, I + H
    mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=900 + H)
    W = gen.normal_weights(M, K, dtype, seed=901)
    W = gen.round_to_storage(gen.storage_to_f64(W, dtype).astype(np.float32) * 6.0, dtype)
    A = pack_workload(g, W, dtype, mask)
    assert g.rnn_step_launches(A, None, 1) == 1 and g.rnn_step_launches(A, None, 8) == 1 and g.rnn_step_launches(A, None, 64) == 2
    rng = np.random.default_rng(902)
    xh = gen.normal_activations(K, 1, dtype, seed=903)
    bias = (0.2 * rng.standard_normal(M)).astype(np.float32)
    c0 = rng.standard_normal((H, 1)).astype(np.float32)
    stream = torch.cuda.current_stream()

    def bufs():
        x = torch.zeros((K, ld), dtype=_tdt(torch, dtype), device=dev); x[:, :1] = to_device(xh, dtype)
        gates = torch.full((M, ld), float("nan"), dtype=torch.float32, device=dev)
        c = torch.full((H, ld), 7.0, dtype=torch.float32, device=dev); c[:, :1] = torch.from_numpy(c0).to(dev)
        h = torch.full((H, ld), 7.0, dtype=_tdt(torch, dtype), device=dev)
        h32 = torch.full((H, ld), 7.0, dtype=torch.float32, device=dev)
        return x, gates, c, h, h32
    bd = torch.from_numpy(bias).to(dev)
    # fused: h goes to a buffer of its own
    x1, g1, c1, h1, h321 = bufs()
    g.lstm_step(A, x1, 1, ld, g1, ld, bd, c1, ld, h1, ld, h321, ld, stream)
    # the same step as product, then cell
    x2, g2, c2, h2, h322 = bufs()
    g.spmv(A, x2, 1, ld, g2, ld, stream)
    g.lstm_cell(g2, ld, bd, c2, ld, h2, dtype, ld, h322, ld, H, 1, stream)
    torch.cuda.synchronize()
    assert torch.equal(g1[:, 0], g2[:, 0])
    assert torch.allclose(c1[:, 0], c2[:, 0], rtol=0, atol=2e-6) and torch.allclose(h321[:, 0], h322[:, 0], rtol=0, atol=2e-6)
    assert torch.allclose(h1[:, 0].float(), h2[:, 0].float(), rtol=0, atol=2.0 ** -7)
    if ld > 1:      # nothing outside the first column
        for tns in (c1, h1.float(), h321):
            assert (tns[:, 1:] == 7.0).all()
        assert torch.isnan(g1[:, 1:]).all()
    # against the fp64 reference
    _, c_ref, h_ref = lstm_ref.step(_masked(W, dtype, mask), gen.storage_to_f64(xh, dtype), bias, c0.astype(np.float64))
    assert np.abs(c1[:, :1].cpu().numpy() - c_ref).max() <= TOL[dtype] * max(1.0, np.abs(c_ref).max())
    assert np.abs(h321[:, :1].cpu().numpy() - h_ref).max() <= TOL[dtype]
    # no bias, no fp32 copy of h
    x3, g3, c3, h3, _ = bufs()
    g.lstm_step(A, x3, 1, ld, g3, ld, None, c3, ld, h3, ld, None, 0, stream)
    torch.cuda.synchronize()
    _, c_ref0, h_ref0 = lstm_ref.step(_masked(W, dtype, mask), gen.storage_to_f64(xh, dtype), None, c0.astype(np.float64))
    assert np.abs(c3[:, :1].cpu().numpy() - c_ref0).max() <= TOL[dtype] * max(1.0, np.abs(c_ref0).max())
    assert np.abs(h3[:, :1].float().cpu().numpy() - h_ref0).max() <= TOL[dtype] + 2.0 ** -7


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,BR,kr,kc,x_first", [(128, 32, 8, 12, True), (96, 16, 8, 8, False), (1024, 32, 8, 12, True)])
def test_gru_step_in_one_launch(dtype, H, BR, kr, kc, x_first):
    from helpers import pack_workload, TOL
    torch, dev, g = _gpu()
    M, BC = 3 * H, 32
    mi = gen.random_mask(M, H, BR, BC, kr, kc, seed=910)
    mh = gen.random_mask(M, H, BR, BC, kr, kc, seed=911)
    scale = 6.0 if H < 512 else 2.0
    Wi = gen.round_to_storage(gen.storage_to_f64(gen.normal_weights(M, H, dtype, seed=912), dtype).astype(np.float32) * scale, dtype)
    Wh = gen.round_to_storage(gen.storage_to_f64(gen.normal_weights(M, H, dtype, seed=913), dtype).astype(np.float32) * scale, dtype)
    Ai, Ah = pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh)
    assert g.rnn_step_launches(Ai, Ah, 1) == 1 and g.rnn_step_launches(Ai, Ah, 4) == 1 and g.rnn_step_launches(Ai, Ah, 64) >= 2
    rng = np.random.default_rng(914)
    x = gen.normal_activations(H, 1, dtype, seed=915)
    h0 = (0.5 * rng.standard_normal((H, 1))).astype(np.float32)
    bi, bh = (0.1 * rng.standard_normal(M)).astype(np.float32), (0.1 * rng.standard_normal(M)).astype(np.float32)
    stream = torch.cuda.current_stream()
    tdt = _tdt(torch, dtype)

    def run(separate_out):
        xh = torch.zeros((2, H, 1), dtype=tdt, device=dev)                 # x and the state in one allocation
        xb, hb = (xh[0], xh[1]) if x_first else (xh[1], xh[0])
        xb.copy_(torch.from_numpy(x).to(dev).view(tdt) if dtype == gen.BF16 else torch.from_numpy(x).to(dev))
        hb.copy_(torch.from_numpy(h0).to(dev).to(tdt))
        gates = torch.full((2, M, 1), float("nan"), dtype=torch.float32, device=dev)
        gi, gh = (gates[0], gates[1]) if x_first else (gates[1], gates[0])
        h32 = torch.from_numpy(h0).to(dev).clone()
        hout = torch.full((H, 1), 7.0, dtype=tdt, device=dev) if separate_out else hb
        g.gru_step(Ai, Ah, xb, 1, hb, 1, 1, gi, 1, gh, 1, torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev), h32, 1,
                   hout, 1, stream)
        torch.cuda.synchronize()
        return gi.clone(), gh.clone(), h32, hout.clone(), hb
    gi1, gh1, h321, ho1, hb1 = run(True)       # one launch
    gi2, gh2, h322, ho2, _ = run(False)        # state updated in place: products, then the cell
    assert torch.equal(gi1, gi2) and torch.equal(gh1, gh2)
    assert torch.allclose(h321, h322, rtol=0, atol=2e-6) and torch.allclose(ho1.float(), ho2.float(), rtol=0, atol=2.0 ** -7)
    hin = gen.storage_to_f64(gen.round_to_storage(h0, dtype), dtype)
    assert np.array_equal(gen.storage_to_f64(hb1.cpu().view(torch.int16).numpy().view(np.uint16) if dtype == gen.BF16 else hb1.cpu().numpy(), dtype), hin)   # input state untouched
    _, _, h_ref = gru_ref.step(_masked(Wi, dtype, mi), _masked(Wh, dtype, mh), gen.storage_to_f64(x, dtype), hin, bi, bh,
                               h0.astype(np.float64))
    assert np.abs(h321.cpu().numpy() - h_ref).max() <= 2 * TOL[dtype]


def test_sequences_through_the_fused_steps():
    """Eight steps of an LSTM layer and of a GRU layer, every step one launch, states ping-ponging between two buffers."""
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    dtype, I, H, T, BR, BC = gen.F16, 64, 128, 8, 32, 32
    stream = torch.cuda.current_stream()
    # LSTM
    M, K = 4 * H, I + H
    mask = gen.random_mask(M, K, BR, BC, 8, 12, seed=920)
    W = gen.normal_weights(M, K, dtype, seed=921) * np.float16(8.0)
    A = pack_workload(g, W, dtype, mask)
    Wm = _masked(W, dtype, mask)
    xs = [gen.normal_activations(I, 1, dtype, seed=922 + t) for t in range(T)]
    bias = (0.1 * np.random.default_rng(923).standard_normal(M)).astype(np.float32)
    xh = [torch.zeros((K, 1), dtype=torch.float16, device=dev) for _ in range(2)]
    gates = torch.empty((M, 1), dtype=torch.float32, device=dev)
    c = torch.zeros((H, 1), dtype=torch.float32, device=dev)
    h32 = torch.empty((H, 1), dtype=torch.float32, device=dev)
    bd = torch.from_numpy(bias).to(dev)
    c_ref = np.zeros((H, 1)); h_ref = np.zeros((H, 1))
    assert g.rnn_step_launches(A, None, 1) == 1
    for t in range(T):
        cur, nxt = xh[t % 2], xh[(t + 1) % 2]
        cur[:I] = to_device(xs[t], dtype)
        g.lstm_step(A, cur, 1, 1, gates, 1, bd, c, 1, nxt[I:], 1, h32, 1, stream)
        torch.cuda.synchronize()
        xh_ref = np.concatenate([gen.storage_to_f64(xs[t], dtype), h_ref.astype(np.float16).astype(np.float64)], axis=0)
        _, c_ref, h_ref = lstm_ref.step(Wm, xh_ref, bias, c_ref)
        assert np.abs(c.cpu().numpy() - c_ref).max() <= TOL[dtype] * max(1.0, np.abs(c_ref).max()), f"c at step {t}"
        assert np.abs(h32.cpu().numpy() - h_ref).max() <= TOL[dtype], f"h at step {t}"
        assert np.abs(nxt[I:].float().cpu().numpy() - h_ref).max() <= TOL[dtype] + 2.0 ** -10
    assert np.abs(h_ref).max() > 0.05
    # GRU
    M = 3 * H
    mi, mh = gen.random_mask(M, H, BR, BC, 8, 12, seed=930), gen.random_mask(M, H, BR, BC, 8, 12, seed=931)
    Wi = gen.normal_weights(M, H, dtype, seed=932) * np.float16(6.0)
    Wh = gen.normal_weights(M, H, dtype, seed=933) * np.float16(6.0)
    Ai, Ah = pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh)
    Wim, Whm = _masked(Wi, dtype, mi), _masked(Wh, dtype, mh)
    xs = [gen.normal_activations(H, 1, dtype, seed=934 + t) for t in range(T)]
    rng = np.random.default_rng(935)
    bi, bh = (0.1 * rng.standard_normal(M)).astype(np.float32), (0.1 * rng.standard_normal(M)).astype(np.float32)
    hb = [torch.zeros((H, 1), dtype=torch.float16, device=dev) for _ in range(2)]
    h32 = torch.zeros((H, 1), dtype=torch.float32, device=dev)
    gi = torch.empty((M, 1), dtype=torch.float32, device=dev)
    gh = torch.empty((M, 1), dtype=torch.float32, device=dev)
    bid, bhd = torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev)
    h_ref = np.zeros((H, 1))
    assert g.rnn_step_launches(Ai, Ah, 1) == 1
    for t in range(T):
        x = to_device(xs[t], dtype)
        g.gru_step(Ai, Ah, x, 1, hb[t % 2], 1, 1, gi, 1, gh, 1, bid, bhd, h32, 1, hb[(t + 1) % 2], 1, stream)
        torch.cuda.synchronize()
        hin = h_ref.astype(np.float16).astype(np.float64)
        _, _, h_ref = gru_ref.step(Wim, Whm, gen.storage_to_f64(xs[t], dtype), hin, bi, bh, h_ref)
        assert np.abs(h32.cpu().numpy() - h_ref).max() <= 2 * TOL[dtype], f"h at step {t}"
        assert np.abs(hb[(t + 1) % 2].float().cpu().numpy() - h_ref).max() <= 2 * TOL[dtype] + 2.0 ** -10
    assert np.abs(h_ref).max() > 0.05


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,kr,kc,B,ld", [(128, 64, 32, 8, 12, 3, 3), (256, 256, 16, 8, 8, 8, 8), (1024, 1024, 32, 8, 12, 32, 40)])
def test_lstm_step_of_several_columns_in_one_launch(dtype, H, I, BR, kr, kc, B, ld):
    """A set of workgroups per column while the sets fit the GPU at once: every column gets the bits the one-column step
    gives; with more columns the step is the product and the cell kernel.  Either way nothing lands outside the B
    columns and the values agree with the fp64 reference."""
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    M, K = 4 * H, I + H
    mask = gen.random_mask(M, K, BR, 32, kr, kc, seed=950 + H)
    W = gen.normal_weights(M, K, dtype, seed=951)
    W = gen.round_to_storage(gen.storage_to_f64(W, dtype).astype(np.float32) * (6.0 if H < 512 else 2.0), dtype)
    A = pack_workload(g, W, dtype, mask)
    # one launch while all sets of workgroups fit the compute units at once (H / BR workgroups per column)
    fused = g.rnn_step_launches(A, None, B) == 1
    assert fused == (B <= 8)
    rng = np.random.default_rng(952)
    xh = gen.normal_activations(K, B, dtype, seed=953)
    bias = (0.2 * rng.standard_normal(M)).astype(np.float32)
    c0 = rng.standard_normal((H, B)).astype(np.float32)
    stream = torch.cuda.current_stream()
    tdt = _tdt(torch, dtype)
    bd = torch.from_numpy(bias).to(dev)
    x = torch.zeros((K, ld), dtype=tdt, device=dev); x[:, :B] = to_device(xh, dtype)
    gates = torch.full((M, ld), float("nan"), dtype=torch.float32, device=dev)
    c = torch.full((H, ld), 7.0, dtype=torch.float32, device=dev); c[:, :B] = torch.from_numpy(c0).to(dev)
    h = torch.full((H, ld), 7.0, dtype=tdt, device=dev)
    h32 = torch.full((H, ld), 7.0, dtype=torch.float32, device=dev)
    g.lstm_step(A, x, B, ld, gates, ld, bd, c, ld, h, ld, h32, ld, stream)
    torch.cuda.synchronize()
    if ld > B:
        assert torch.isnan(gates[:, B:]).all()
        for tns in (c, h.float(), h32):
            assert (tns[:, B:] == 7.0).all()
    Wm = _masked(W, dtype, mask)
    for b in sorted({0, 1, B // 2, B - 1}):
        x1 = x[:, b:b + 1].contiguous()
        g1 = torch.empty((M, 1), dtype=torch.float32, device=dev)
        c1 = torch.from_numpy(c0[:, b:b + 1].copy()).to(dev)
        h1 = torch.empty((H, 1), dtype=tdt, device=dev)
        h321 = torch.empty((H, 1), dtype=torch.float32, device=dev)
        g.lstm_step(A, x1, 1, 1, g1, 1, bd, c1, 1, h1, 1, h321, 1, stream)
        torch.cuda.synchronize()
        if fused:
            assert torch.equal(gates[:, b], g1[:, 0]) and torch.equal(c[:, b], c1[:, 0]), f"column {b}"
            assert torch.equal(h32[:, b], h321[:, 0]) and torch.equal(h[:, b], h1[:, 0]), f"column {b}"
        _, c_ref, h_ref = lstm_ref.step(Wm, gen.storage_to_f64(xh[:, b:b + 1], dtype), bias, c0[:, b:b + 1].astype(np.float64))
        assert np.abs(c[:, b:b + 1].cpu().numpy() - c_ref).max() <= TOL[dtype] * max(1.0, np.abs(c_ref).max())
        assert np.abs(h32[:, b:b + 1].cpu().numpy() - h_ref).max() <= TOL[dtype]
    assert not torch.equal(h32[:, 0], h32[:, 1])


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,BR,kr,kc,B,ld", [(128, 32, 8, 12, 5, 8), (1024, 32, 8, 12, 8, 8), (1024, 32, 8, 12, 32, 32)])
def test_gru_step_of_several_columns_in_one_launch(dtype, H, BR, kr, kc, B, ld):
    from helpers import to_device, pack_workload, TOL
    torch, dev, g = _gpu()
    M, BC = 3 * H, 32
    mi = gen.random_mask(M, H, BR, BC, kr, kc, seed=960)
    mh = gen.random_mask(M, H, BR, BC, kr, kc, seed=961)
    scale = 6.0 if H < 512 else 2.0
    Wi = gen.round_to_storage(gen.storage_to_f64(gen.normal_weights(M, H, dtype, seed=962), dtype).astype(np.float32) * scale, dtype)
    Wh = gen.round_to_storage(gen.storage_to_f64(gen.normal_weights(M, H, dtype, seed=963), dtype).astype(np.float32) * scale, dtype)
    Ai, Ah = pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh)
    fused = g.rnn_step_launches(Ai, Ah, B) == 1
    assert fused == (B <= 8)
    rng = np.random.default_rng(964)
    xv = gen.normal_activations(H, B, dtype, seed=965)
    h0 = (0.5 * rng.standard_normal((H, B))).astype(np.float32)
    bi, bh = (0.1 * rng.standard_normal(M)).astype(np.float32), (0.1 * rng.standard_normal(M)).astype(np.float32)
    bid, bhd = torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev)
    stream = torch.cuda.current_stream()
    tdt = _tdt(torch, dtype)
    xh = torch.zeros((2, H, ld), dtype=tdt, device=dev)                    # x and the state in one allocation
    xh[0, :, :B] = to_device(xv, dtype)
    xh[1, :, :B] = torch.from_numpy(h0).to(dev).to(tdt)
    gates = torch.full((2, M, ld), float("nan"), dtype=torch.float32, device=dev)
    h32 = torch.full((H, ld), 7.0, dtype=torch.float32, device=dev); h32[:, :B] = torch.from_numpy(h0).to(dev)
    hout = torch.full((H, ld), 7.0, dtype=tdt, device=dev)
    g.gru_step(Ai, Ah, xh[0], ld, xh[1], ld, B, gates[0], ld, gates[1], ld, bid, bhd, h32, ld, hout, ld, stream)
    torch.cuda.synchronize()
    Wim, Whm = _masked(Wi, dtype, mi), _masked(Wh, dtype, mh)
    hin_bits = xh[1, :, :B].float().cpu().numpy().astype(np.float64)
    for b in sorted({0, 1, B // 2, B - 1}):
        x1 = torch.zeros((2, H, 1), dtype=tdt, device=dev)
        x1[0, :, 0] = xh[0, :, b]; x1[1, :, 0] = xh[1, :, b]
        g1 = torch.empty((2, M, 1), dtype=torch.float32, device=dev)
        h321 = torch.from_numpy(h0[:, b:b + 1].copy()).to(dev)
        ho1 = torch.empty((H, 1), dtype=tdt, device=dev)
        g.gru_step(Ai, Ah, x1[0], 1, x1[1], 1, 1, g1[0], 1, g1[1], 1, bid, bhd, h321, 1, ho1, 1, stream)
        torch.cuda.synchronize()
        if fused:
            assert torch.equal(gates[0, :, b], g1[0, :, 0]) and torch.equal(gates[1, :, b], g1[1, :, 0]), f"column {b}"
            assert torch.equal(h32[:, b], h321[:, 0]) and torch.equal(hout[:, b], ho1[:, 0]), f"column {b}"
        _, _, h_ref = gru_ref.step(Wim, Whm, gen.storage_to_f64(xv[:, b:b + 1], dtype), hin_bits[:, b:b + 1], bi, bh,
                                   h0[:, b:b + 1].astype(np.float64))
        assert np.abs(h32[:, b:b + 1].cpu().numpy() - h_ref).max() <= 2 * TOL[dtype]
    if ld > B:
        assert (h32[:, B:] == 7.0).all() and (hout[:, B:].float() == 7.0).all()
        assert torch.isnan(gates[:, :, B:]).all()
