"""A recurrent layer over a whole sequence in one launch (Section 3.1: one matrix-vector product per time step; the
kernel keeps the compact weights in registers for all steps and passes the hidden state between workgroups through
tagged words).  Compared with the fp64 references step by step (h fed back rounded to the element type, as the device
feeds it back), with the chain of one-step calls on the device, and exercised on its bounded wait."""
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


def _scaled_weights(M, K, dtype, seed, scale):
    W = gen.normal_weights(M, K, dtype, seed=seed)
    return gen.round_to_storage(gen.storage_to_f64(W, dtype).astype(np.float32) * scale, dtype)


def _inputs(T, I, dtype, seed):
    """T x I inputs in storage type (row t = x_t)."""
    return np.ascontiguousarray(gen.normal_activations(I, T, dtype, seed=seed).T)


def _lstm_case(g, dtype, H, I, BR, BC, kr, kc, seed, scale=6.0):
    from helpers import pack_workload
    M, K = 4 * H, I + H
    mask = gen.random_mask(M, K, BR, BC, kr, kc, seed=seed)
    W = _scaled_weights(M, K, dtype, seed + 1, scale)
    return pack_workload(g, W, dtype, mask), _masked(W, dtype, mask)


def _lstm_reference(Wm, xs, dtype, bias, h0, c0):
    T = xs.shape[0]
    h = gen.storage_to_f64(h0, dtype).reshape(-1, 1)
    c = c0.astype(np.float64).reshape(-1, 1)
    hs = []
    for t in range(T):
        xh = np.concatenate([gen.storage_to_f64(xs[t], dtype).reshape(-1, 1), _round(h, dtype)], axis=0)
        _, c, h = lstm_ref.step(Wm, xh, bias, c)
        hs.append(h[:, 0].copy())
    return np.stack(hs), c[:, 0]


def _run_lstm(torch, dev, g, A, xs, dtype, bias, h0, c0, ldxs=None, ldhs=None, max_polls=0):
    from helpers import to_device
    T, I = xs.shape
    H = h0.shape[0]
    ldxs = I if ldxs is None else ldxs
    ldhs = H if ldhs is None else ldhs
    xp = np.zeros((T, ldxs), dtype=xs.dtype); xp[:, :I] = xs
    xd = to_device(xp, dtype)
    hd = to_device(h0, dtype)
    c = torch.from_numpy(c0.astype(np.float32)).to(dev)
    hs = torch.full((T, ldhs), 7.0, dtype=_tdt(torch, dtype), device=dev)
    hs32 = torch.full((T, ldhs), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    bd = None if bias is None else torch.from_numpy(bias).to(dev)
    g.lstm_sequence(A, xd, ldxs, T, bd, hd, c, hs, ldhs, hs32, ldhs, status, max_polls, torch.cuda.current_stream())
    torch.cuda.synchronize()
    if ldhs > H:
        assert (hs[:, H:].float() == 7.0).all() and torch.isnan(hs32[:, H:]).all(), "wrote outside the H outputs of a step"
    return int(status.item()), hs[:, :H].float().cpu().numpy(), hs32[:, :H].cpu().numpy(), c.cpu().numpy()


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,BC,kr,kc,T,pad", [
    (96, 64, 32, 32, 8, 12, 12, 0),       # 3 workgroups, 5 column blocks
    (128, 72, 16, 8, 4, 4, 9, 3),         # 8 workgroups, 25 column blocks, x rows not 16-byte aligned (ldxs = I + 3)
    (1024, 1024, 32, 32, 8, 12, 6, 0),    # the LSTM workload's gate matrix (4096 x 2048): 32 workgroups, 64 blocks
    (512, 32, 32, 16, 16, 8, 5, 8),       # 34 column blocks, padded outputs
])
def test_lstm_sequence_against_reference(dtype, H, I, BR, BC, kr, kc, T, pad):
    from helpers import TOL
    torch, dev, g = _gpu()
    scale = 6.0 if H < 512 else 2.0
    A, Wm = _lstm_case(g, dtype, H, I, BR, BC, kr, kc, seed=1200 + H, scale=scale)
    assert g.rnn_sequence_supported(A)
    rng = np.random.default_rng(1201)
    xs = _inputs(T, I, dtype, 1202)
    bias = (0.2 * rng.standard_normal(4 * H)).astype(np.float32)
    h0 = gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype)
    c0 = rng.standard_normal(H).astype(np.float32)
    status, hs, hs32, c = _run_lstm(torch, dev, g, A, xs, dtype, bias, h0, c0, ldxs=I + pad, ldhs=H + pad)
    assert status == 0
    hs_ref, c_ref = _lstm_reference(Wm, xs, dtype, bias, h0, c0)
    # the reference follows the device's own rounding of h only approximately (a last-place difference in a rounded
    # h moves later steps a little), so the bound grows slowly with the step
    for t in range(T):
        tol = TOL[dtype] * (1 + t)
        assert np.abs(hs32[t] - hs_ref[t]).max() <= tol, f"h32 at step {t}"
        assert np.abs(hs[t] - hs_ref[t]).max() <= tol + 2.0 ** -9, f"h at step {t}"
    assert np.abs(c - c_ref).max() <= TOL[dtype] * (1 + T) * max(1.0, np.abs(c_ref).max())
    assert np.abs(hs_ref[-1]).max() > 0.05


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
def test_lstm_sequence_equals_the_chain_of_steps(dtype):
    """Same arithmetic in the same order as grim_bcr_lstm_step called T times: the outputs agree bit for bit."""
    from helpers import to_device
    torch, dev, g = _gpu()
    H, I, T = 256, 192, 10
    A, _ = _lstm_case(g, dtype, H, I, 32, 32, 8, 12, seed=1300)
    rng = np.random.default_rng(1301)
    xs = _inputs(T, I, dtype, 1302)
    bias = (0.2 * rng.standard_normal(4 * H)).astype(np.float32)
    h0 = gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype)
    c0 = rng.standard_normal(H).astype(np.float32)
    status, hs, hs32, c = _run_lstm(torch, dev, g, A, xs, dtype, bias, h0, c0)
    assert status == 0
    # the chain: two [x; h] vectors used in turn
    K = I + H
    xh = [torch.zeros((K, 1), dtype=_tdt(torch, dtype), device=dev) for _ in range(2)]
    xh[0][I:, 0] = to_device(h0, dtype)
    gates = torch.empty((4 * H, 1), dtype=torch.float32, device=dev)
    cd = torch.from_numpy(c0.reshape(H, 1).copy()).to(dev)
    h32 = torch.empty((H, 1), dtype=torch.float32, device=dev)
    bd = torch.from_numpy(bias).to(dev)
    stream = torch.cuda.current_stream()
    xsd = to_device(xs, dtype)
    for t in range(T):
        cur, nxt = xh[t % 2], xh[(t + 1) % 2]
        cur[:I, 0] = xsd[t]
        g.lstm_step(A, cur, 1, 1, gates, 1, bd, cd, 1, nxt[I:], 1, h32, 1, stream)
        torch.cuda.synchronize()
        assert np.array_equal(h32[:, 0].cpu().numpy(), hs32[t]), f"fp32 h at step {t}"
        assert np.array_equal(nxt[I:, 0].float().cpu().numpy(), hs[t]), f"h at step {t}"
    assert np.array_equal(cd[:, 0].cpu().numpy(), c)


def _gru_case(g, dtype, H, I, BR, BC, kr, kc, seed, scale=5.0):
    from helpers import pack_workload
    mi = gen.random_mask(3 * H, I, BR, BC, kr, kc, seed=seed)
    mh = gen.random_mask(3 * H, H, BR, BC, kr, kc, seed=seed + 1)
    Wi = _scaled_weights(3 * H, I, dtype, seed + 2, scale)
    Wh = _scaled_weights(3 * H, H, dtype, seed + 3, scale)
    return pack_workload(g, Wi, dtype, mi), pack_workload(g, Wh, dtype, mh), _masked(Wi, dtype, mi), _masked(Wh, dtype, mh)


def _run_gru(torch, dev, g, Ai, Ah, xs, dtype, bi, bh, h0, h32_0, max_polls=0):
    from helpers import to_device
    T, I = xs.shape
    H = h0.shape[0]
    xd = to_device(xs, dtype)
    hd = to_device(h0, dtype)
    h32 = torch.from_numpy(h32_0.astype(np.float32)).to(dev)
    hs = torch.full((T, H), 7.0, dtype=_tdt(torch, dtype), device=dev)
    hs32 = torch.full((T, H), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    bid = None if bi is None else torch.from_numpy(bi).to(dev)
    bhd = None if bh is None else torch.from_numpy(bh).to(dev)
    g.gru_sequence(Ai, Ah, xd, I, T, bid, bhd, hd, h32, hs, H, hs32, H, status, max_polls, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return int(status.item()), hs.float().cpu().numpy(), hs32.cpu().numpy(), h32.cpu().numpy()


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,BC,kr,kc,T", [
    (128, 96, 16, 32, 8, 8, 10),          # input and hidden sizes differ: 3 and 4 column blocks
    (1024, 1024, 32, 32, 8, 12, 6),       # the paper's hidden size (Section 6.1), 32 workgroups of 6 waves
    (512, 160, 32, 16, 4, 16, 7),         # the paper's 152-wide input rounded up to whole blocks
])
def test_gru_sequence_against_reference(dtype, H, I, BR, BC, kr, kc, T):
    from helpers import TOL
    torch, dev, g = _gpu()
    Ai, Ah, Wim, Whm = _gru_case(g, dtype, H, I, BR, BC, kr, kc, seed=1400 + H, scale=5.0 if H < 512 else 2.0)
    assert g.rnn_sequence_supported(Ai, Ah)
    rng = np.random.default_rng(1401)
    xs = _inputs(T, I, dtype, 1402)
    bi = (0.2 * rng.standard_normal(3 * H)).astype(np.float32)
    bh = (0.2 * rng.standard_normal(3 * H)).astype(np.float32)
    h32_0 = (0.5 * rng.standard_normal(H)).astype(np.float32)
    h0 = gen.round_to_storage(h32_0, dtype)
    status, hs, hs32, h_last = _run_gru(torch, dev, g, Ai, Ah, xs, dtype, bi, bh, h0, h32_0)
    assert status == 0
    h = h32_0.astype(np.float64).reshape(-1, 1)
    for t in range(T):
        x64 = gen.storage_to_f64(xs[t], dtype).reshape(-1, 1)
        hin = _round(h, dtype) if t else gen.storage_to_f64(h0, dtype).reshape(-1, 1)
        h = gru_ref.step(Wim, Whm, x64, hin, bi, bh, h)[-1]
        tol = TOL[dtype] * (1 + t)
        assert np.abs(hs32[t] - h[:, 0]).max() <= tol, f"h32 at step {t}"
        assert np.abs(hs[t] - h[:, 0]).max() <= tol + 2.0 ** -9, f"h at step {t}"
    assert np.array_equal(h_last, hs32[-1])
    assert np.abs(h).max() > 0.05


def test_sequence_calls_in_a_row_and_a_tiny_wait_limit():
    """The exchange words are cleared by every call (a shorter sequence after a longer one must not see old tags), and
    a wait limit of one re-read either completes with the right values or gives up cleanly: status 1, the kernel
    returns, and the next call with the default limit is right again."""
    from helpers import TOL
    torch, dev, g = _gpu()
    dtype, H, I = gen.F16, 512, 64
    A, Wm = _lstm_case(g, dtype, H, I, 32, 32, 8, 12, seed=1500)
    rng = np.random.default_rng(1501)
    h0 = gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype)
    c0 = rng.standard_normal(H).astype(np.float32)
    for T, polls in [(40, 0), (7, 0), (200, 1), (9, 0)]:
        xs = _inputs(T, I, dtype, 1502 + T)
        status, hs, hs32, c = _run_lstm(torch, dev, g, A, xs, dtype, None, h0, c0, max_polls=polls)
        assert status in (0, 1)
        assert polls == 1 or status == 0
        if status == 0:
            hs_ref, _ = _lstm_reference(Wm, xs, dtype, None, h0, c0)
            for t in range(min(T, 12)):
                assert np.abs(hs32[t] - hs_ref[t]).max() <= TOL[dtype] * (1 + t), f"T={T}: h32 at step {t}"


def test_sequence_refusals():
    from helpers import pack_workload
    torch, dev, g = _gpu()
    dtype, H, I = gen.F16, 64, 64
    # blocks keeping different counts: no sequence kernel
    m = gen.random_mask(4 * H, I + H, 32, 32, 8, 12, seed=1600)
    W = gen.normal_weights(4 * H, I + H, dtype, seed=1601)
    A = pack_workload(g, W, dtype, m)
    assert g.rnn_sequence_supported(A)
    m2 = gen.random_mask(4 * H, I + H, 32, 32, (4, 8), (8, 12), seed=1602)
    xs = torch.zeros((3, I), dtype=torch.float16, device=dev)
    h0 = torch.zeros((H,), dtype=torch.float16, device=dev)
    c = torch.zeros((H,), dtype=torch.float32, device=dev)
    hs = torch.zeros((3, H), dtype=torch.float16, device=dev)
    status = torch.zeros((1,), dtype=torch.int32, device=dev)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence(A, xs, I, 0, None, h0, c, hs, H, None, 0, status)           # no steps
    assert "SHAPE" in str(e.value)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence(A, xs, I - 1, 3, None, h0, c, hs, H, None, 0, status)       # rows of xs overlap
    assert "SHAPE" in str(e.value)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence(A, xs, I, 3, None, h0, c, None, H, None, 0, status)
    assert "NULL" in str(e.value)
    A2 = pack_workload(g, W, dtype, m2)
    assert not g.rnn_sequence_supported(A2)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence(A2, xs, I, 3, None, h0, c, hs, H, None, 0, status)
    assert "UNSUPPORTED" in str(e.value)
    # kept counts outside the compiled pairs
    m3 = gen.random_mask(4 * H, I + H, 32, 32, 10, 10, seed=1603)
    A3 = pack_workload(g, W, dtype, m3)
    assert not g.rnn_sequence_supported(A3)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence(A3, xs, I, 3, None, h0, c, hs, H, None, 0, status)
    assert "UNSUPPORTED" in str(e.value)
    torch.cuda.synchronize()


# ---- several sequences side by side (batch): every sequence gets the bits of a call of its own

def _run_lstm_batch(torch, dev, g, A, xs, dtype, bias, h0, c0, pad=0, max_polls=0):
    """xs [T, B, I], h0 [B, H] storage bits, c0 [B, H]: returns status, hs [T, B, H], hs32 [T, B, H], c [B, H]."""
    from helpers import to_device
    T, B, I = xs.shape
    H = h0.shape[1]
    ldxs, ldhs = I + pad, H + pad
    xp = np.zeros((T * B, ldxs), dtype=xs.dtype); xp[:, :I] = xs.reshape(T * B, I)
    xd = to_device(xp, dtype)
    hd = to_device(np.ascontiguousarray(h0), dtype)
    c = torch.from_numpy(np.ascontiguousarray(c0, dtype=np.float32)).to(dev)
    hs = torch.full((T * B, ldhs), 7.0, dtype=_tdt(torch, dtype), device=dev)
    hs32 = torch.full((T * B, ldhs), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    bd = None if bias is None else torch.from_numpy(bias).to(dev)
    g.lstm_sequence_batch(A, xd, ldxs, T, B, bd, hd, c, hs, ldhs, hs32, ldhs, status, max_polls, torch.cuda.current_stream())
    torch.cuda.synchronize()
    if pad:
        assert (hs[:, H:].float() == 7.0).all() and torch.isnan(hs32[:, H:]).all(), "wrote outside the H outputs of a row"
    return (int(status.item()), hs[:, :H].float().cpu().numpy().reshape(T, B, H), hs32[:, :H].cpu().numpy().reshape(T, B, H),
            c.cpu().numpy())


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,BC,kr,kc,T,B,pad", [
    (96, 64, 32, 32, 8, 12, 9, 2, 0),        # one pair of sequences
    (128, 72, 16, 8, 4, 4, 7, 3, 3),         # an odd batch (the second pair is half empty), unaligned rows of xs
    (256, 64, 8, 16, 4, 8, 6, 5, 8),         # strips of 8 rows: 3 cell threads per hidden unit
    (1024, 1024, 32, 32, 8, 12, 5, 8, 0),    # the LSTM workload's gate matrix, full batch: two rounds of exchange reads
    (512, 1536, 32, 32, 8, 12, 4, 8, 0),     # 16 workgroups per sequence
    # more workgroups per sequence than an eighth of the GPU: workgroups carry several sequences in turn
    (1024, 64, 8, 32, 4, 8, 4, 5, 0),        # 128 workgroups: two sets, of 3 and 2 sequences
    (2016, 32, 8, 32, 4, 8, 3, 3, 8),        # 252 workgroups: one set carries all three
    (1024, 1024, 8, 32, 4, 8, 3, 8, 3),      # four sequences per workgroup, inputs copied element by element
    (1024, 1024, 32, 32, 8, 12, 3, 32, 0),   # the LSTM workload at the batch of Section 6.3: 8 sets, four sequences each
    (1024, 256, 32, 32, 8, 12, 4, 20, 0),    # 7 sets: six of three sequences (two per pass, then one), one of two
])
def test_lstm_sequence_batch_equals_sequences_of_their_own(dtype, H, I, BR, BC, kr, kc, T, B, pad):
    from helpers import TOL
    torch, dev, g = _gpu()
    scale = 6.0 if H < 512 else 2.0
    A, Wm = _lstm_case(g, dtype, H, I, BR, BC, kr, kc, seed=1700 + H, scale=scale)
    assert g.rnn_sequence_supported(A, None, B)
    rng = np.random.default_rng(1701 + B)
    xs = np.stack([_inputs(T, I, dtype, 1710 + b) for b in range(B)], axis=1)           # [T, B, I]
    bias = (0.2 * rng.standard_normal(4 * H)).astype(np.float32)
    h0 = np.stack([gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype) for _ in range(B)])
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    status, hs, hs32, c = _run_lstm_batch(torch, dev, g, A, xs, dtype, bias, h0, c0, pad=pad)
    assert status == 0
    for b in range(B):
        s1, hs1, hs32_1, c1 = _run_lstm(torch, dev, g, A, np.ascontiguousarray(xs[:, b]), dtype, bias, h0[b], c0[b])
        assert s1 == 0
        assert np.array_equal(hs32[:, b], hs32_1), f"sequence {b}: fp32 outputs"
        assert np.array_equal(hs[:, b], hs1), f"sequence {b}: outputs"
        assert np.array_equal(c[b], c1), f"sequence {b}: cell state"
    # and one of them against the fp64 reference, so the pair of calls cannot be wrong together
    b = B - 1
    hs_ref, c_ref = _lstm_reference(Wm, np.ascontiguousarray(xs[:, b]), dtype, bias, h0[b], c0[b])
    for t in range(T):
        assert np.abs(hs32[t, b] - hs_ref[t]).max() <= TOL[dtype] * (1 + t), f"h32 at step {t}"
    assert np.abs(hs_ref[-1]).max() > 0.05
    # sequences differ from each other
    assert not np.array_equal(hs32[:, 0], hs32[:, 1])


@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("H,I,BR,BC,kr,kc,T,B", [
    (128, 96, 16, 32, 8, 8, 8, 4),
    (1024, 1024, 32, 32, 8, 12, 5, 8),       # the paper's hidden size (Section 6.1)
    (512, 160, 32, 16, 4, 16, 6, 7),
    (1024, 96, 8, 32, 4, 8, 5, 4),           # 128 workgroups per sequence: two sets of two sequences
    (1024, 96, 8, 32, 4, 8, 4, 7),           # sets of 4 and 3
    (1024, 1024, 32, 32, 8, 12, 3, 32),      # Section 6.3's batch: 8 sets of four sequences
])
def test_gru_sequence_batch_equals_sequences_of_their_own(dtype, H, I, BR, BC, kr, kc, T, B):
    from helpers import TOL, to_device
    torch, dev, g = _gpu()
    Ai, Ah, Wim, Whm = _gru_case(g, dtype, H, I, BR, BC, kr, kc, seed=1800 + H, scale=5.0 if H < 512 else 2.0)
    assert g.rnn_sequence_supported(Ai, Ah, B)
    rng = np.random.default_rng(1801 + B)
    xs = np.stack([_inputs(T, I, dtype, 1810 + b) for b in range(B)], axis=1)
    bi = (0.2 * rng.standard_normal(3 * H)).astype(np.float32)
    bh = (0.2 * rng.standard_normal(3 * H)).astype(np.float32)
    h32_0 = (0.5 * rng.standard_normal((B, H))).astype(np.float32)
    h0 = np.stack([gen.round_to_storage(h32_0[b], dtype) for b in range(B)])
    xd = to_device(np.ascontiguousarray(xs.reshape(T * B, I)), dtype)
    hd = to_device(np.ascontiguousarray(h0), dtype)
    h32 = torch.from_numpy(h32_0.copy()).to(dev)
    hs = torch.full((T * B, H), 7.0, dtype=_tdt(torch, dtype), device=dev)
    hs32 = torch.full((T * B, H), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    g.gru_sequence_batch(Ai, Ah, xd, I, T, B, torch.from_numpy(bi).to(dev), torch.from_numpy(bh).to(dev), hd, h32, hs, H, hs32, H,
                         status, 0, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    hsn = hs.float().cpu().numpy().reshape(T, B, H)
    hs32n = hs32.cpu().numpy().reshape(T, B, H)
    for b in range(B):
        s1, hs1, hs32_1, last1 = _run_gru(torch, dev, g, Ai, Ah, np.ascontiguousarray(xs[:, b]), dtype, bi, bh, h0[b], h32_0[b])
        assert s1 == 0
        assert np.array_equal(hs32n[:, b], hs32_1), f"sequence {b}: fp32 outputs"
        assert np.array_equal(hsn[:, b], hs1), f"sequence {b}: outputs"
        assert np.array_equal(h32[b].cpu().numpy(), last1), f"sequence {b}: final state"
    b = 0
    h = h32_0[b].astype(np.float64).reshape(-1, 1)
    for t in range(T):
        x64 = gen.storage_to_f64(xs[t, b], dtype).reshape(-1, 1)
        hin = _round(h, dtype) if t else gen.storage_to_f64(h0[b], dtype).reshape(-1, 1)
        h = gru_ref.step(Wim, Whm, x64, hin, bi, bh, h)[-1]
        assert np.abs(hs32n[t, b] - h[:, 0]).max() <= TOL[dtype] * (1 + t), f"h32 at step {t}"
    assert not np.array_equal(hs32n[:, 0], hs32n[:, 1])


def test_sequence_batch_limits_and_a_tiny_wait_limit():
    torch, dev, g = _gpu()
    dtype, H, I = gen.F16, 256, 64
    A, _ = _lstm_case(g, dtype, H, I, 32, 32, 8, 12, seed=1900)
    assert g.rnn_sequence_supported(A, None, 8) and g.rnn_sequence_supported(A, None, 32) and not g.rnn_sequence_supported(A, None, 33)
    assert not g.rnn_sequence_supported(A, None, 0)
    rng = np.random.default_rng(1901)
    B, T = 8, 150
    xs = np.stack([_inputs(T, I, dtype, 1910 + b) for b in range(B)], axis=1)
    h0 = np.stack([gen.round_to_storage((0.5 * rng.standard_normal(H)).astype(np.float32), dtype) for _ in range(B)])
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    ok = _run_lstm_batch(torch, dev, g, A, xs, dtype, None, h0, c0)
    assert ok[0] == 0
    # one re-read allowed: the call completes with the same bits or gives up cleanly, and the next call is right again
    status, _, hs32, _ = _run_lstm_batch(torch, dev, g, A, xs, dtype, None, h0, c0, max_polls=1)
    assert status in (0, 1)
    if status == 0:
        assert np.array_equal(hs32, ok[2])
    again = _run_lstm_batch(torch, dev, g, A, xs[:5], dtype, None, h0, c0)
    assert again[0] == 0 and np.array_equal(again[2], ok[2][:5])
    xd = torch.zeros((33 * 3, I), dtype=torch.float16, device=dev)
    hd = torch.zeros((33, H), dtype=torch.float16, device=dev)
    c = torch.zeros((33, H), dtype=torch.float32, device=dev)
    hs = torch.zeros((33 * 3, H), dtype=torch.float16, device=dev)
    st = torch.zeros((1,), dtype=torch.int32, device=dev)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence_batch(A, xd, I, 3, 33, None, hd, c, hs, H, None, 0, st)
    assert "UNSUPPORTED" in str(e.value)
    with pytest.raises(g.GrimError) as e:
        g.lstm_sequence_batch(A, xd, I, 3, 0, None, hd, c, hs, H, None, 0, st)
    assert "SHAPE" in str(e.value)
    torch.cuda.synchronize()
