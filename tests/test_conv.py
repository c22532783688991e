"""Convolution with the im2col matrix never materialised (Section 3.1 / 4.5): pins of the fp64 reference (CPU)
and parity of grim_bcr_conv2d against it (GPU)."""
import numpy as np
import pytest

import bcr_inputs as gen
from oracle import bcr_oracle as orc
from oracle import conv_ref


def _masked(W, dtype, mask):
    return orc.masked_dense(gen.storage_to_f64(W, dtype), mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx)


# ------------------------------------------------------------------ pins of the reference (no GPU)
@pytest.mark.parametrize("kh,kw", [(3, 3), (1, 1), (3, 1), (1, 3)])
def test_reference_equals_im2col_product_and_library_conv(kh, kw):
    import torch
    Cin, H, W, M = 6, 7, 9, 8
    rng = np.random.default_rng(31)
    Wm = rng.standard_normal((M, Cin * kh * kw))
    Wm[rng.random(Wm.shape) < 0.6] = 0.0
    F = rng.standard_normal((Cin, H, W))
    Y = conv_ref.conv_same(Wm, F, kh, kw)
    # the GEMM view of Section 3.1: filter matrix times the im2col matrix
    assert np.allclose(Y.reshape(M, -1), Wm @ conv_ref.im2col(F, kh, kw), rtol=0, atol=1e-12)
    # the library routine, double precision, zero padding kh // 2, kw // 2
    Yt = torch.nn.functional.conv2d(torch.from_numpy(F)[None], torch.from_numpy(Wm.reshape(M, Cin, kh, kw)),
                                    padding=(kh // 2, kw // 2))[0].numpy()
    assert np.allclose(Y, Yt, rtol=0, atol=1e-12)


def test_reference_special_cases():
    Cin, H, W, M = 3, 5, 8, 4
    rng = np.random.default_rng(32)
    F = rng.standard_normal((Cin, H, W))
    # a 1 x 1 kernel is a plain matrix product over channels
    W1 = rng.standard_normal((M, Cin))
    assert np.allclose(conv_ref.conv_same(W1, F, 1, 1).reshape(M, -1), W1 @ F.reshape(Cin, -1), atol=1e-13)
    # a single centre tap of a 3 x 3 kernel copies the channel; the corner tap shifts it by one row and one column
    Wc = np.zeros((1, Cin * 9)); Wc[0, 1 * 9 + 4] = 1.0
    assert np.array_equal(conv_ref.conv_same(Wc, F, 3, 3)[0], F[1])
    Wk = np.zeros((1, Cin * 9)); Wk[0, 2 * 9 + 0] = 1.0          # (r, q) = (0, 0): Y[h, w] = F[h - 1, w - 1]
    Yk = conv_ref.conv_same(Wk, F, 3, 3)[0]
    assert np.array_equal(Yk[1:, 1:], F[2, :-1, :-1]) and not Yk[0].any() and not Yk[:, 0].any()
    # integer data: exact, and the scale bounds the result
    Wi = rng.integers(-3, 4, (M, Cin * 9)).astype(np.float64)
    Fi = rng.integers(-3, 4, (Cin, H, W)).astype(np.float64)
    Yi = conv_ref.conv_same(Wi, Fi, 3, 3)
    assert np.array_equal(Yi, np.round(Yi)) and (np.abs(Yi) <= conv_ref.abs_scale(Wi, Fi, 3, 3)).all()


def test_layer_reference_matches_library_conv_with_bias_and_relu():
    import torch
    Cin, H, W, M = 5, 6, 9, 7
    rng = np.random.default_rng(33)
    Wm, F, b = rng.standard_normal((M, Cin * 9)), rng.standard_normal((Cin, H, W)), rng.standard_normal(M)
    Yt = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(F)[None], torch.from_numpy(Wm.reshape(M, Cin, 3, 3)),
                                               bias=torch.from_numpy(b), padding=1))[0].numpy()
    assert np.allclose(conv_ref.layer(Wm, F, 3, 3, b, True), Yt, rtol=0, atol=1e-12)
    assert (conv_ref.layer(Wm, F, 3, 3, b, True) >= 0).all() and (conv_ref.layer(Wm, F, 3, 3, b, False) < 0).any()
    assert np.array_equal(conv_ref.layer(Wm, F, 3, 3), conv_ref.conv_same(Wm, F, 3, 3))



@pytest.mark.parametrize("kh,kw,stride,H,W", [(3, 3, 2, 8, 10), (3, 3, 2, 7, 9), (1, 1, 2, 5, 6), (5, 5, 2, 9, 9), (3, 3, 1, 6, 5)])
def test_batched_strided_reference_equals_library_conv_and_plain_loops(kh, kw, stride, H, W):
    import torch
    B, Cin, M = 2, 3, 4
    rng = np.random.default_rng(34)
    Wm = rng.standard_normal((M, Cin * kh * kw))
    Wm[rng.random(Wm.shape) < 0.5] = 0.0
    F = rng.standard_normal((B, Cin, H, W))
    Y = conv_ref.conv2d(Wm, F, kh, kw, stride)
    Yt = torch.nn.functional.conv2d(torch.from_numpy(F), torch.from_numpy(Wm.reshape(M, Cin, kh, kw)), stride=stride,
                                    padding=(kh // 2, kw // 2)).numpy()
    assert Y.shape == Yt.shape == (B, M, -(-H // stride), -(-W // stride))
    assert np.allclose(Y, Yt, rtol=0, atol=1e-12)
    # the definition, term by term
    Wr = Wm.reshape(M, Cin, kh, kw)
    for b, m, ho, wo in [(0, 0, 0, 0), (1, 3, Y.shape[2] - 1, Y.shape[3] - 1), (1, 2, 1, 2), (0, 1, Y.shape[2] - 1, 0)]:
        s = 0.0
        for cin in range(Cin):
            for r in range(kh):
                for q in range(kw):
                    h, w = stride * ho + r - kh // 2, stride * wo + q - kw // 2
                    if 0 <= h < H and 0 <= w < W:
                        s += Wr[m, cin, r, q] * F[b, cin, h, w]
        assert abs(Y[b, m, ho, wo] - s) <= 1e-12
    # stride 1, one image: the single-image reference
    if stride == 1:
        assert np.array_equal(Y[1], conv_ref.conv_same(Wm, F[1], kh, kw))
    else:
        # a strided convolution is the stride-1 result read at every stride-th position
        assert np.allclose(Y[0], conv_ref.conv_same(Wm, F[0], kh, kw)[:, ::stride, ::stride], rtol=0, atol=1e-12)


# ------------------------------------------------------------------ GPU
def _run(g, A, F, dtype, M, Cin, H, W, kh, kw, ldy=None):
    import torch
    from helpers import to_device
    dev = torch.device("cuda:0")
    N = H * W
    ldy = N if ldy is None else ldy
    Fd = to_device(np.ascontiguousarray(F.reshape(Cin, N)), dtype)
    Yd = torch.full((M, ldy), float("nan"), dtype=torch.float32, device=dev)
    g.conv2d(A, Fd, Cin, H, W, kh, kw, Yd, ldy, torch.cuda.current_stream())
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    if ldy > N:
        assert np.isnan(Y[:, N:]).all()
    return Y[:, :N].reshape(M, H, W)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("Cin,H,W,kh,kw,BR,BC", [
    (32, 14, 14, 3, 3, 16, 32),      # 14 x 14: image rows of 28 bytes, every alignment of the window occurs
    (16, 12, 20, 3, 3, 4, 16),       # the paper's 4 x 16 blocks
    (64, 8, 8, 1, 1, 16, 32),        # 1 x 1: a plain product, one tile exactly
    (24, 9, 16, 3, 1, 16, 24),
    (8, 10, 13, 1, 3, 32, 8),        # odd width (130 positions)
])
def test_conv_parity(dtype, Cin, H, W, kh, kw, BR, BC):
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    M, K = 96, Cin * kh * kw
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, BR // 2, BR})), tuple(sorted({1, BC // 4 + 1, BC})), seed=700 + Cin)
    Wt = gen.normal_weights(M, K, dtype, seed=701)
    F = gen.normal_activations(Cin, H * W, dtype, seed=702, relu=True).reshape(Cin, H, W)
    A = pack_workload(g, Wt, dtype, mask)
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    Yref, S = conv_ref.conv_same(Wm, F64, kh, kw), conv_ref.abs_scale(Wm, F64, kh, kw)
    Y = _run(g, A, F, dtype, M, Cin, H, W, kh, kw)
    assert np.isfinite(Y).all()
    assert (Y[S == 0] == 0).all()
    pos = S > 0
    assert (np.abs(Y - Yref)[pos] / S[pos]).max() <= TOL[dtype]
    assert np.abs(Y - Yref).max() <= TOL[dtype] * np.abs(Yref).max()
    Y2 = _run(g, A, F, dtype, M, Cin, H, W, kh, kw, ldy=H * W + 5)
    assert Y2.tobytes() == Y.tobytes()


@pytest.mark.gpu
@pytest.mark.parametrize("Cin,H,W,M,BC,keep_c,form", [
    (8, 96, 116, 96, 8, (2, 8), "a (tile, strip) pair per wave: strips of a few steps, thousands of pairs, idle waves in a tile's last workgroup"),
    (64, 16, 24, 64, 32, (24, 32), "twelve waves per strip: long strips, at most 256 (tile, strip) pairs"),
    (64, 48, 116, 64, 32, (24, 32), "eight waves per strip: long strips, 348 (tile, strip) pairs"),
])
@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
def test_conv_launch_forms(dtype, Cin, H, W, M, BC, keep_c, form):
    """The other launch forms of the convolution kernel (same arithmetic per step, different split of the work)."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    K = Cin * 9
    mask = gen.random_mask(M, K, 16, BC, (0, 8, 16), keep_c, seed=770 + Cin)
    Wt = gen.normal_weights(M, K, dtype, seed=771)
    F = gen.normal_activations(Cin, H * W, dtype, seed=772, relu=True).reshape(Cin, H, W)
    bias = (0.05 * np.random.default_rng(773).standard_normal(M)).astype(np.float32)
    A = pack_workload(g, Wt, dtype, mask)
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    ref = conv_ref.layer(Wm, F64, 3, 3, bias, True)
    S = conv_ref.abs_scale(Wm, F64, 3, 3) + np.abs(bias)[:, None, None]
    out = _run_act(g, A, F, dtype, M, Cin, H, W, 3, 3, bias, True, gen.F32)
    assert (np.abs(out - ref) <= TOL[dtype] * S + 1e-30).all(), form
    plain = _run(g, A, F, dtype, M, Cin, H, W, 3, 3)
    Sp = conv_ref.abs_scale(Wm, F64, 3, 3)
    assert (np.abs(plain - conv_ref.conv_same(Wm, F64, 3, 3)) <= TOL[dtype] * Sp + 1e-30).all(), form


@pytest.mark.gpu
def test_conv_random_geometries():
    """Seeded sweep over image sizes (widths of every parity and alignment, so that windows start at odd and even
    elements, wrap to the next image row inside a piece, and reach outside the feature map in the first and last
    tiles), kernel shapes and channel counts; integer data, so every result must equal the reference exactly."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload
    rng = np.random.default_rng(760)
    dtype = gen.F16
    for case in range(14):
        kh, kw = [(3, 3), (1, 3), (3, 1), (5, 3), (1, 1), (3, 5)][case % 6]
        W = int(rng.integers(8, 41))
        H = int(rng.integers(max(2, (64 + W - 1) // W), 30))
        BC = [8, 16, 32][case % 3]
        Cin = BC * int(rng.integers(1, 5)) // np.gcd(BC, kh * kw) * 1
        while (Cin * kh * kw) % BC:
            Cin += 1
        M, K = 32, Cin * kh * kw
        mask = gen.random_mask(M, K, 16, BC, (0, 5, 16), tuple(sorted({1, BC // 2, BC})), seed=761 + case)
        Wt = gen.small_int_values((M, K), dtype, seed=762 + case)
        F = gen.small_int_values((Cin, H, W), dtype, seed=763 + case)
        A = pack_workload(g, Wt, dtype, mask)
        Yref = conv_ref.conv_same(_masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype), kh, kw)
        Y = _run(g, A, F, dtype, M, Cin, H, W, kh, kw)
        assert np.array_equal(Y.astype(np.float64), Yref), (case, Cin, H, W, kh, kw, BC)


@pytest.mark.gpu
@pytest.mark.parametrize("Cin,H,W,kh,kw,BC", [
    (32, 7, 7, 3, 3, 32),       # 7 x 7, the last stage of an ImageNet ResNet: 49 positions, one partly filled tile
    (64, 7, 7, 1, 1, 32),
    (32, 4, 4, 3, 3, 32),
    (16, 2, 2, 3, 3, 16),       # narrower and lower than the kernel
    (16, 1, 1, 3, 3, 16),       # one position: only the centre tap is ever valid
    (16, 1, 9, 1, 3, 16),
    (32, 30, 3, 3, 3, 32),      # rows of 3: a piece of 8 positions spans three or four image rows
    (24, 13, 5, 5, 3, 8),
    (16, 50, 2, 3, 5, 16),      # 100 positions, rows narrower than the kernel
    (16, 11, 12, 5, 5, 16),     # 25 taps
    (16, 9, 10, 3, 7, 16),      # 21 taps
    (32, 6, 20, 1, 9, 32),
])
def test_conv_small_and_narrow_maps(Cin, H, W, kh, kw, BC):
    """Maps of fewer than 64 positions (one tile whose columns past H * W are never stored) and image rows shorter than a
    piece of 8 positions or than the kernel; integer data, exact.  Also through the layer epilogue with a padded fp16
    output, where nothing past a row's H * W positions may be written."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload
    dtype, M = gen.F16, 48
    K = Cin * kh * kw
    mask = gen.random_mask(M, K, 16, BC, (0, 5, 16), tuple(sorted({1, BC // 2, BC})), seed=770 + H * W)
    Wt = gen.small_int_values((M, K), dtype, seed=771)
    F = gen.small_int_values((Cin, H, W), dtype, seed=772 + H)
    A = pack_workload(g, Wt, dtype, mask)
    Yref = conv_ref.conv_same(_masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype), kh, kw)
    Y = _run(g, A, F, dtype, M, Cin, H, W, kh, kw, ldy=H * W + 5)
    assert np.array_equal(Y.astype(np.float64), Yref), (Cin, H, W, kh, kw)
    bias = np.arange(M, dtype=np.float32) - 20.0
    out = _run_act(g, A, F, dtype, M, Cin, H, W, kh, kw, bias, True, gen.F16, ldo=H * W + 3)
    ref = np.maximum(Yref + bias[:, None, None], 0.0)
    assert np.array_equal(out.astype(np.float64), ref.astype(np.float16).astype(np.float64)), (Cin, H, W, kh, kw)


@pytest.mark.gpu
def test_conv_wave_per_strip_long_strips():
    """Nine steps per strip and 4096 (tile, strip) pairs (a 256 x 256 map, 64 output channels): every wave takes a
    pair of its own and runs three batches of steps.  Integer data, exact, every entry."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload
    dtype, Cin, H, W, M = gen.F16, 32, 256, 256, 64
    K = Cin * 9
    mask = gen.random_mask(M, K, 16, 32, (4, 8, 16), 32, seed=780)       # every column kept: 9 steps in every strip
    Wt = gen.small_int_values((M, K), dtype, seed=781)
    F = gen.small_int_values((Cin, H, W), dtype, seed=782)
    A = pack_workload(g, Wt, dtype, mask)
    Yref = conv_ref.conv_same(_masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype), 3, 3)
    Y = _run(g, A, F, dtype, M, Cin, H, W, 3, 3)
    assert np.array_equal(Y.astype(np.float64), Yref)


@pytest.mark.gpu
def test_conv_integer_data_is_exact_and_equals_the_im2col_product():
    """Small integers: every sum is exact, so the fused path, the library's own product on the materialised
    im2col matrix and the reference must agree bit for bit."""
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, run_spmm
    dtype, Cin, H, W, M = gen.F16, 32, 16, 24, 64
    K = Cin * 9
    mask = gen.random_mask(M, K, 16, 32, (0, 4, 8), (0, 8, 16), seed=710)
    Wt = gen.small_int_values((M, K), dtype, seed=711)
    F = gen.small_int_values((Cin, H, W), dtype, seed=712)
    A = pack_workload(g, Wt, dtype, mask)
    Yref = conv_ref.conv_same(_masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype), 3, 3)
    Y = _run(g, A, F, dtype, M, Cin, H, W, 3, 3)
    assert np.array_equal(Y.astype(np.float64), Yref)
    X = conv_ref.im2col(F, 3, 3)
    Yx = run_spmm(g, A, X, dtype, M, H * W)
    assert Yx.tobytes() == np.ascontiguousarray(Y.reshape(M, -1)).tobytes()


@pytest.mark.gpu
def test_conv_full_size_sampled():
    """The configuration bench.py --conv times (c2's weights on a 256 x 56 x 56 map): sampled output rows against the
    reference, every border position included, and the whole result against the product on the materialised matrix
    (same kernel family, same summation order: bit for bit)."""
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, run_spmm, TOL
    wl = gen.c2_vgg_conv(64)
    dtype, Cin, H, W, M = wl.dtype, 256, 56, 56, wl.M
    A = pack_workload(g, wl.W, dtype, wl.mask)
    F = gen.normal_activations(Cin, H * W, dtype, seed=77, relu=True).reshape(Cin, H, W)
    Y = _run(g, A, F, dtype, M, Cin, H, W, 3, 3)
    Wm, F64 = _masked(wl.W, dtype, wl.mask), gen.storage_to_f64(F, dtype)
    rows = np.array([0, 7, 8, 100, 129, 255])
    Yref, S = conv_ref.conv_same(Wm[rows], F64, 3, 3), conv_ref.abs_scale(Wm[rows], F64, 3, 3)
    assert (np.abs(Y[rows] - Yref) <= TOL[dtype] * np.maximum(S, 1e-30)).all()
    assert np.abs(Y[rows] - Yref).max() <= TOL[dtype] * np.abs(Yref).max()
    X = conv_ref.im2col(F, 3, 3)
    Yx = run_spmm(g, A, X, dtype, M, H * W, kernel=3)
    assert Yx.tobytes() == np.ascontiguousarray(Y.reshape(M, -1)).tobytes()


@pytest.mark.gpu
@pytest.mark.parametrize("layer", [1, 3])
def test_conv_vgg_layers_at_224_and_112_sampled(layer):
    """VGG-16 layers 2 (64 channels at 224 x 224) and 4 (128 channels at 112 x 112) on the layers' own matrices, as fused
    convolutions at full size: sampled output channels (every row strip touched) against the reference at every
    position, borders included."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    M, K, N = gen.VGG16_LAYERS[layer]
    Cin, H = K // 9, int(round(N ** 0.5))
    wl = gen.c4_vgg16_layer(layer, N=64)
    dtype = wl.dtype
    A = pack_workload(g, wl.W, dtype, wl.mask)
    F = gen.normal_activations(Cin, H * H, dtype, seed=300 + layer, relu=True).reshape(Cin, H, H)
    Y = _run(g, A, F, dtype, M, Cin, H, H, 3, 3)
    rng = np.random.default_rng(310 + layer)
    rows = np.sort(np.concatenate([s * 16 + rng.choice(16, 2, replace=False) for s in range(M // 16)]))
    Wm, F64 = _masked(wl.W, dtype, wl.mask), gen.storage_to_f64(F, dtype)
    Yref, S = conv_ref.conv_same(Wm[rows], F64, 3, 3), conv_ref.abs_scale(Wm[rows], F64, 3, 3)
    assert np.isfinite(Y).all()
    assert (np.abs(Y[rows] - Yref) <= TOL[dtype] * np.maximum(S, 1e-30)).all()
    assert np.abs(Y[rows] - Yref).max() <= TOL[dtype] * np.abs(Yref).max()


def _run_act(g, A, F, dtype, M, Cin, H, W, kh, kw, bias, relu, out_dtype, ldo=None):
    import torch
    from helpers import to_device
    dev = torch.device("cuda:0")
    N = H * W
    ldo = N if ldo is None else ldo
    Fd = to_device(np.ascontiguousarray(F.reshape(Cin, N)), dtype)
    tdt = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}[out_dtype]
    out = torch.full((M, ldo), 7.0, dtype=tdt, device=dev)
    bd = None if bias is None else torch.from_numpy(bias).to(dev)
    g.conv2d_act(A, Fd, Cin, H, W, kh, kw, bd, relu, out, out_dtype, ldo, torch.cuda.current_stream())
    torch.cuda.synchronize()
    if ldo > N:
        assert (out[:, N:].float() == 7.0).all()
    return out[:, :N].float().cpu().numpy().reshape(M, H, W)


@pytest.mark.gpu
@pytest.mark.parametrize("out_dtype", [gen.F32, gen.F16, gen.BF16])
@pytest.mark.parametrize("relu,with_bias,pad", [(True, True, 0), (False, True, 3), (True, False, 4)])
def test_conv_layer_epilogue(out_dtype, relu, with_bias, pad):
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    dtype, Cin, H, W, M, BR, BC = gen.F16, 32, 12, 14, 96, 16, 32
    K = Cin * 9
    mask = gen.random_mask(M, K, BR, BC, (0, 8, 16), (4, 8, 32), seed=720)
    Wt = gen.normal_weights(M, K, dtype, seed=721)
    F = gen.normal_activations(Cin, H * W, dtype, seed=722, relu=True).reshape(Cin, H, W)
    bias = (0.05 * np.random.default_rng(723).standard_normal(M)).astype(np.float32) if with_bias else None
    A = pack_workload(g, Wt, dtype, mask)
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    ref = conv_ref.layer(Wm, F64, 3, 3, bias, relu)
    S = conv_ref.abs_scale(Wm, F64, 3, 3) + (0 if bias is None else np.abs(bias)[:, None, None])
    out = _run_act(g, A, F, dtype, M, Cin, H, W, 3, 3, bias, relu, out_dtype, ldo=H * W + pad)
    ulp = {gen.F32: 0.0, gen.F16: 2.0 ** -11, gen.BF16: 2.0 ** -8}[out_dtype]      # half an ulp of the output rounding, relative
    assert np.isfinite(out).all()
    assert (np.abs(out - ref) <= TOL[dtype] * S + ulp * np.abs(ref) + 1e-30).all()
    if relu:
        assert (out >= 0).all() and (out[ref < -TOL[dtype] * S] == 0).all()
    else:
        assert (out < 0).any()
    if out_dtype == gen.F32 and not relu and bias is None:
        pass
    # fp32, no bias, no rectifier: the same bits as grim_bcr_conv2d
    plain = _run(g, A, F, dtype, M, Cin, H, W, 3, 3)
    same = _run_act(g, A, F, dtype, M, Cin, H, W, 3, 3, None, False, gen.F32)
    assert plain.tobytes() == same.tobytes()


@pytest.mark.gpu
def test_three_conv_layers_chained_in_fp16():
    """Three pruned 3x3 CONV + bias + ReLU layers, each writing the next one's fp16 feature map directly.  The reference
    runs the same chain in fp64 and rounds every layer's output to fp16 where the device does, so that each layer is
    compared on identical inputs."""
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, to_device, TOL
    dev = torch.device("cuda:0")
    dtype, H, W = gen.F16, 16, 24
    chans = [32, 64, 64, 32]
    N = H * W
    F = gen.normal_activations(chans[0], N, dtype, seed=730, relu=True).reshape(chans[0], H, W)
    cur = to_device(np.ascontiguousarray(F.reshape(chans[0], N)), dtype)
    ref_in = gen.storage_to_f64(F, dtype)
    for li in range(3):
        Cin, M = chans[li], chans[li + 1]
        K = Cin * 9
        mask = gen.random_mask(M, K, 16, 32, (8, 16), (8, 16), seed=731 + li)
        Wt = gen.normal_weights(M, K, dtype, seed=741 + li) * np.float16(6.0)          # keeps activations of order one
        bias = (0.1 * np.random.default_rng(751 + li).standard_normal(M)).astype(np.float32)
        A = pack_workload(g, Wt, dtype, mask)
        out = torch.empty((M, N), dtype=torch.float16, device=dev)
        g.conv2d_act(A, cur, Cin, H, W, 3, 3, torch.from_numpy(bias).to(dev), True, out, dtype, N, torch.cuda.current_stream())
        torch.cuda.synchronize()
        Wm = _masked(Wt, dtype, mask)
        ref = conv_ref.layer(Wm, ref_in, 3, 3, bias, True)
        S = conv_ref.abs_scale(Wm, ref_in, 3, 3) + np.abs(bias)[:, None, None]
        got = out.float().cpu().numpy().reshape(M, H, W)
        assert (np.abs(got - ref) <= TOL[dtype] * S + 2.0 ** -11 * np.abs(ref) + 1e-30).all(), f"layer {li}"
        assert got.max() > 0.1, f"layer {li} died"
        # the next layer consumes what the device wrote
        ref_in = got.astype(np.float64)
        cur = out



def _run_plan(g, A, F, dtype, M, kh, kw, stride, bias=None, relu=False, out_dtype=gen.F32, pad=0):
    """F: B x Cin x H x W storage-typed.  Returns (B x M x Ho x Wo) in fp64 and the raw output tensor."""
    import torch
    from helpers import to_device
    dev = torch.device("cuda:0")
    B, Cin, H, W = F.shape
    Ho, Wo = -(-H // stride), -(-W // stride)
    plan = g.ConvPlan(A, Cin, H, W, kh, kw, stride)
    assert plan.out_hw == (Ho, Wo)
    fstride = Cin * H * W + pad
    Fp = np.zeros((B, fstride), dtype=F.dtype); Fp[:, :Cin * H * W] = F.reshape(B, -1)
    Fd = to_device(Fp, dtype)
    ldo = Ho * Wo + pad
    ostride = M * ldo + pad
    tdt = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}[out_dtype]
    out = torch.full((B, ostride), 7.0, dtype=tdt, device=dev)
    bd = None if bias is None else torch.from_numpy(bias).to(dev)
    g.conv2d_plan(plan, Fd, B, fstride, bd, relu, out, out_dtype, ldo, ostride, torch.cuda.current_stream())
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().astype(np.float64)
    body = o[:, :M * ldo].reshape(B, M, ldo)
    if pad:
        assert (body[:, :, Ho * Wo:] == 7.0).all() and (o[:, M * ldo:] == 7.0).all(), "wrote outside the outputs"
    return body[:, :, :Ho * Wo].reshape(B, M, Ho, Wo)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [gen.F16, gen.BF16])
@pytest.mark.parametrize("Cin,H,W,kh,kw,BR,BC,stride,B,pad", [
    (16, 24, 24, 3, 3, 16, 16, 1, 3, 0),     # a batch at stride 1
    (16, 12, 20, 3, 3, 4, 16, 1, 2, 3),      # odd image strides: the second image starts 2 bytes off a dword
    (32, 32, 40, 3, 3, 16, 32, 2, 2, 0),     # stride 2, W a multiple of 8: every second row skipped
    (8, 15, 13, 3, 3, 16, 8, 2, 2, 1),       # stride 2, odd sizes: all rows walked, odd outputs dropped
    (32, 7, 7, 1, 1, 16, 32, 2, 3, 0),       # 1 x 1 at stride 2 (a down-sampling shortcut), fewer than 64 positions
    (4, 56, 56, 5, 5, 16, 20, 2, 1, 0),
    (24, 9, 16, 3, 1, 16, 24, 2, 2, 5),
])
def test_conv_plan_batch_and_stride(dtype, Cin, H, W, kh, kw, BR, BC, stride, B, pad):
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    M, K = 96, Cin * kh * kw
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, BR // 2, BR})), tuple(sorted({1, BC // 4 + 1, BC})), seed=740 + Cin)
    Wt = gen.normal_weights(M, K, dtype, seed=741)
    F = gen.normal_activations(Cin, B * H * W, dtype, seed=742, relu=True).reshape(Cin, B, H, W).transpose(1, 0, 2, 3).copy()
    A = pack_workload(g, Wt, dtype, mask)
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    Yref = conv_ref.conv2d(Wm, F64, kh, kw, stride)
    S = conv_ref.conv2d(np.abs(Wm), np.abs(F64), kh, kw, stride)
    Y = _run_plan(g, A, F, dtype, M, kh, kw, stride, pad=pad)
    assert np.isfinite(Y).all()
    assert (Y[S == 0] == 0).all()
    pos = S > 0
    assert (np.abs(Y - Yref)[pos] / S[pos]).max() <= TOL[dtype]
    assert np.abs(Y - Yref).max() <= TOL[dtype] * np.abs(Yref).max()
    if stride == 1:
        # the planned convolution adds the same terms in the same order as the unplanned one, image by image
        for b in range(B):
            Yb = _run(g, A, F[b], dtype, M, Cin, H, W, kh, kw)
            assert np.array_equal(Yb, Y[b].astype(np.float32))


@pytest.mark.gpu
def test_conv_plan_layer_epilogue_and_refusals():
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    dtype, Cin, H, W, M, stride, B = gen.F16, 16, 16, 16, 48, 2, 2
    K = Cin * 9
    mask = gen.random_mask(M, K, 16, 16, (4, 8), (4, 8), seed=760)
    Wt = gen.normal_weights(M, K, dtype, seed=761)
    F = gen.normal_activations(Cin, B * H * W, dtype, seed=762).reshape(Cin, B, H, W).transpose(1, 0, 2, 3).copy()
    bias = np.random.default_rng(763).standard_normal(M).astype(np.float32) * 0.05
    A = pack_workload(g, Wt, dtype, mask)
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    ref = np.maximum(conv_ref.conv2d(Wm, F64, 3, 3, stride) + bias.astype(np.float64)[None, :, None, None], 0.0)
    for out_dtype, slack in [(gen.F32, 0.0), (gen.F16, 2.0 ** -11), (gen.BF16, 2.0 ** -8)]:
        Y = _run_plan(g, A, F, dtype, M, 3, 3, stride, bias=bias, relu=True, out_dtype=out_dtype, pad=2)
        assert (Y >= 0).all()
        assert np.abs(Y - ref).max() <= (TOL[dtype] + slack) * max(1.0, np.abs(ref).max())
    with pytest.raises(g.GrimError) as e:
        g.ConvPlan(A, Cin, H, W, 3, 3, 3)                      # stride 3
    assert "SHAPE" in str(e.value)
    with pytest.raises(g.GrimError) as e:
        g.ConvPlan(A, Cin + 1, H, W, 3, 3, 1)                  # K does not match
    assert "SHAPE" in str(e.value)
    plan = g.ConvPlan(A, Cin, H, W, 3, 3, 2)
    dev = torch.device("cuda:0")
    Fd = torch.zeros((B, Cin * H * W), dtype=torch.float16, device=dev)
    out = torch.zeros((B, M * 64), dtype=torch.float32, device=dev)
    with pytest.raises(g.GrimError) as e:
        g.conv2d_plan(plan, Fd, B, Cin * H * W, None, False, out, gen.F32, 63, M * 64)       # ldo < Ho * Wo
    assert "SHAPE" in str(e.value)
    with pytest.raises(g.GrimError) as e:
        g.conv2d_plan(plan, Fd, B, Cin * H * W - 1, None, False, out, gen.F32, 64, M * 64)   # images overlap
    assert "SHAPE" in str(e.value)
    torch.cuda.synchronize()


@pytest.mark.gpu
def test_conv_plan_on_the_large_nonuniform_workload_as_a_batch_of_images():
    """The largest SpMM workload is a 3 x 3 convolution of 512 channels on a batch of 8 images of 56 x 56
    (K = 4608, N = 8 * 3136): as a planned convolution on the feature maps, compared with the reference on sampled
    output channels, and with the product on the materialised im2col matrix of one image."""
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, to_device, TOL
    wl = gen.c5_nonuniform()
    dtype, M, Cin, H, W, B = wl.dtype, wl.M, 512, 56, 56, 8
    assert wl.K == Cin * 9 and wl.N == B * H * W
    A = pack_workload(g, wl.W, dtype, wl.mask)
    F = gen.normal_activations(Cin, B * H * W, dtype, seed=770, relu=True).reshape(Cin, B, H, W).transpose(1, 0, 2, 3).copy()
    Y = _run_plan(g, A, F, dtype, M, 3, 3, 1)
    Wm, F64 = _masked(wl.W, dtype, wl.mask), gen.storage_to_f64(F, dtype)
    rows = np.array([0, 1, 31, 32, 255, 300, 511])
    for b in (0, 3, 7):
        ref = conv_ref.conv_same(Wm[rows], F64[b], 3, 3)
        S = conv_ref.abs_scale(Wm[rows], F64[b], 3, 3)
        got = Y[b][rows]
        pos = S > 0
        assert (np.abs(got - ref)[pos] / S[pos]).max() <= TOL[dtype]
        assert (got[~pos] == 0).all()
    # image 5 through the SpMM entry point on its im2col matrix: the same sums up to the order of additions
    X = gen.round_to_storage(conv_ref.im2col(F64[5], 3, 3).astype(np.float32), dtype)
    dev = torch.device("cuda:0")
    Xd = to_device(X, dtype)
    Yd = torch.empty((M, H * W), dtype=torch.float32, device=dev)
    g.spmm(A, Xd, H * W, H * W, Yd, H * W, torch.cuda.current_stream())
    torch.cuda.synchronize()
    Ym = Yd.cpu().numpy().astype(np.float64).reshape(M, H, W)
    assert np.abs(Ym - Y[5]).max() <= TOL[dtype] * np.abs(Ym).max()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,M,Cin,H,W,kh,kw,BR,BC,B,epi", [
    (gen.F16, 128, 8, 224, 224, 3, 3, 16, 24, 1, None),       # 8 strips, 192-column tiles: 256 + a rest of 1024 positions
    (gen.BF16, 256, 16, 112, 112, 3, 3, 32, 16, 2, None),     # 32-row blocks, 96-column tiles that straddle the two images
    (gen.F16, 272, 16, 160, 160, 5, 5, 16, 20, 1, gen.F16),   # 17 strips = two groups; 5 x 5; bias + rectifier + fp16 out
    (gen.BF16, 128, 4, 3073, 16, 3, 3, 16, 12, 1, gen.BF16),  # 16 positions past the whole round: the rest overlaps it
    (gen.F16, 256, 32, 96, 88, 1, 1, 32, 32, 3, gen.F32),     # 1 x 1, three images
])
def test_conv_on_the_wide_tile_kernel(dtype, M, Cin, H, W, kh, kw, BR, BC, B, epi):
    """Layers with at least one round of 256 workgroups' worth of positions run on the wide-tile kernel with the
    fetching waves building the im2col rows from the feature maps; compared with the reference in full."""
    import paper_2108_11033_amd as g
    from helpers import pack_workload, TOL
    K = Cin * kh * kw
    mask = gen.random_mask(M, K, BR, BC, tuple(sorted({0, 1, BR // 2, BR})), tuple(sorted({1, BC // 4 + 1, BC})), seed=780 + M)
    Wt = gen.normal_weights(M, K, dtype, seed=781)
    F = gen.normal_activations(Cin, B * H * W, dtype, seed=782, relu=True).reshape(Cin, B, H, W).transpose(1, 0, 2, 3).copy()
    A = pack_workload(g, Wt, dtype, mask)
    assert g.conv2d_kernel_name(A, Cin, H, W, kh, kw, B, 1) == "bcr_conv_wide"
    assert g.conv2d_kernel_name(A, Cin, H, W, kh, kw, B, 2) == "bcr_conv_gather"
    Wm, F64 = _masked(Wt, dtype, mask), gen.storage_to_f64(F, dtype)
    Yref = conv_ref.conv2d(Wm, F64, kh, kw, 1)
    S = conv_ref.conv2d(np.abs(Wm), np.abs(F64), kh, kw, 1)
    if epi is None:
        Y = _run_plan(g, A, F, dtype, M, kh, kw, 1)
        assert np.isfinite(Y).all()
        assert (Y[S == 0] == 0).all()
        pos = S > 0
        assert (np.abs(Y - Yref)[pos] / S[pos]).max() <= TOL[dtype]
        assert np.abs(Y - Yref).max() <= TOL[dtype] * np.abs(Yref).max()
    else:
        bias = (0.05 * np.random.default_rng(783).standard_normal(M)).astype(np.float32)
        ref = np.maximum(Yref + bias.astype(np.float64)[None, :, None, None], 0.0)
        Y = _run_plan(g, A, F, dtype, M, kh, kw, 1, bias=bias, relu=True, out_dtype=epi, pad=4)
        slack = {gen.F32: 0.0, gen.F16: 2.0 ** -11, gen.BF16: 2.0 ** -8}[epi]
        assert (Y >= 0).all()
        assert np.abs(Y - ref).max() <= (TOL[dtype] + slack) * max(1.0, np.abs(ref).max())
    if B == 1:
        # the unplanned entry point takes the same route and writes the same bits
        import torch
        from helpers import to_device
        dev = torch.device("cuda:0")
        Fd = to_device(np.ascontiguousarray(F[0].reshape(Cin, H * W)), dtype)
        Yd = torch.full((M, H * W), float("nan"), dtype=torch.float32, device=dev)
        g.conv2d(A, Fd, Cin, H, W, kh, kw, Yd, H * W, torch.cuda.current_stream())
        torch.cuda.synchronize()
        Y1 = Yd.cpu().numpy().reshape(M, H, W)
        assert np.isfinite(Y1).all()
        assert np.abs(Y1 - Yref[0]).max() <= TOL[dtype] * np.abs(Yref).max()
        if epi is None:
            assert np.array_equal(Y1, Y[0].astype(np.float32))


@pytest.mark.gpu
def test_conv_refusals():
    import torch
    import paper_2108_11033_amd as g
    from helpers import pack_workload, to_device
    from paper_2108_11033_amd import GrimError
    dev = torch.device("cuda:0")
    wl = gen.c2_vgg_conv(64)
    A = pack_workload(g, wl.W, wl.dtype, wl.mask)                 # K = 2304 = 256 * 9
    F = torch.zeros((256, 64), dtype=torch.float16, device=dev)
    Y = torch.full((256, 64), 5.0, dtype=torch.float32, device=dev)
    for args, name in (((255, 8, 8, 3, 3), "GRIM_ERR_SHAPE"),      # Cin * kh * kw != K
                       ((256, 8, 8, 2, 2), "GRIM_ERR_SHAPE"),      # even kernel
                       ((256, 0, 8, 3, 3), "GRIM_ERR_SHAPE"),      # empty map
                       ((2304, 8, 8, 1, 1), "GRIM_ERR_SHAPE")):    # output row shorter than the map is checked below
        with pytest.raises(GrimError) as e:
            g.conv2d(A, F, *args, Y, 64 if args[0] != 2304 else 63)
        assert e.value.name == name, args
    # 25 taps in one kernel row: the division of the tap number by the kernel width is not exact in the kernel's form
    m25 = gen.random_mask(32, 32 * 25, 16, 32, 8, 8, seed=790)
    A25 = pack_workload(g, gen.normal_weights(32, 32 * 25, gen.F16, seed=791), gen.F16, m25)
    with pytest.raises(GrimError) as e:
        g.conv2d(A25, F, 32, 8, 8, 1, 25, Y, 64)
    assert e.value.name == "GRIM_ERR_UNSUPPORTED"
    torch.cuda.synchronize()
    assert (Y == 5.0).all()
