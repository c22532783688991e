#!/usr/bin/env python3
"""Benchmark of the BCR sparse product on one MI355X.

A step is one pass of the hot path -- one grim_bcr_spmm launch -- over one batch of
synthetic input of the headline workload: the VGG-style 3x3 convolution as an im2col
BCR SpMM (M=256, K=2304, N=3136, fp16 in / fp32 accumulate, 16x32 blocks keeping
8/16 rows and 8/32 columns).  Inputs are resident in HBM before the timed region; the
steps rotate over enough (X, Y) buffer sets that no step finds its operands in the
256 MB last-level cache.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--extra]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
# HBM bytes per c2 launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by
# what the same counter reads for a device copy of known size (x 2.0 fetched, x 1.0 written); per kernel family, from
# profiles/bcr_spmm_gather_c2.md and profiles/bcr_spmm_mma_c2.md
C2_TRAFFIC_BYTES = {
    "bcr_spmm_gather": (7765.9 * 2.0 + 3136.0) * 1024,
    "bcr_spmm_mma": (7834.0 * 2.0 + 3136.0) * 1024,
}
METRIC = "BCR SpMM/SpMV useful TFLOP/s, HBM GB/s, % of roofline vs oracle"


def spmm_algorithmic_bytes(view, N: int, esz: int) -> int:
    """Bytes one SpMM must move: X once, Y once, the compact weights and their indices."""
    idx = 2 * (view["n_row_idx"] + view["n_col_idx"]) + 4 * 2 * (view["nb"] + 1) + 8 * (view["nb"] + 1) + 4 * view["nbr"]
    return esz * view["K"] * N + 4 * view["M"] * N + esz * view["nnz"] + idx


def spmv_algorithmic_bytes(view, batch: int, esz: int) -> int:
    """Bytes one SpMV must move: compact weights, 8 bytes of bit masks per block, x and y."""
    return esz * view["nnz"] + 8 * view["nb"] + 4 * view["nbr"] + esz * view["K"] * batch + 4 * view["M"] * batch


def view_dict(A) -> dict:
    v = A.view()
    a = A.arrays()
    return dict(M=v.M, K=v.K, nnz=v.nnz, nb=v.nb, nbr=v.nbr, n_row_idx=len(a["row_idx"]), n_col_idx=len(a["col_idx"]),
                dev_bytes_mma=v.dev_bytes_mma)


def time_launches(torch, fn, steps: int, warmup: int):
    """Average seconds per launch by HIP events on the stream the kernels run on."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for i in range(steps):
        fn(warmup + i)
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return start.elapsed_time(stop) * 1e-3 / steps, wall / steps


def cpu_baseline(wl, reps: int = 3) -> dict:
    """The oracle as it stands, timed on the host cores on the whole headline workload."""
    import bcr_inputs as gen
    from oracle import bcr_oracle as orc
    W64 = gen.storage_to_f64(wl.W, wl.dtype)
    X64 = gen.storage_to_f64(wl.X, wl.dtype)
    Wm = orc.masked_dense(W64, wl.mask.BR, wl.mask.BC, wl.mask.row_ptr, wl.mask.row_idx, wl.mask.col_ptr, wl.mask.col_idx)
    best = float("inf")
    for _ in range(reps):
        t0 = time.perf_counter()
        orc.matmul(Wm, X64, want_scale=False, skip_zero=True)
        best = min(best, time.perf_counter() - t0)
    return {"value": wl.useful_flops() / best / 1e12, "unit": "TFLOP/s", "cores": orc.threads(), "kind": "oracle",
            "sample": f"whole {wl.name} product (M={wl.M}, K={wl.K}, N={wl.N}), fp64 zero-skipping triple loop, "
                      f"best of {reps}, {best * 1e3:.1f} ms"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--sets", type=int, default=32, help="(X, Y) buffer sets the steps rotate over")
    ap.add_argument("--tile-n", type=int, default=0)
    ap.add_argument("--strips-per-wg", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 choose, 2 staged matrix-core kernel, 3 row-gathering one")
    ap.add_argument("--extra", action="store_true", help="also time the SpMV and large non-uniform workloads")
    ap.add_argument("--conv", action="store_true",
                    help="also time c2's layer as a convolution on the feature map (no im2col matrix)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--sweep", action="store_true",
                    help="also run the block-size search of the paper on a 1024x1024 layer at 10x pruning, and the "
                         "strip-reorder ablation on the non-uniform workload")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the product would shard over the columns of X with no "
              "exchange between GPUs); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import bcr_inputs as gen
    import paper_2108_11033_amd as g
    from paper_2108_11033_amd import binding

    g.load_library()                      # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    def pack(wl):
        m = wl.mask
        return g.pack(wl.W, wl.dtype, m.BR, m.BC, m.row_ptr, m.row_idx, m.col_ptr, m.col_idx)

    def dev_tensor(a, dtype):
        if dtype == gen.BF16:
            return torch.from_numpy(a.view(np.int16).copy()).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---------------- headline: c2 ----------------
    wl = gen.c2_vgg_conv()
    A = pack(wl)
    vd = view_dict(A)
    X0 = dev_tensor(wl.X, wl.dtype)
    sets = max(1, args.sets)
    Xs = [X0] + [X0.clone() for _ in range(sets - 1)]
    Ys = [torch.empty((wl.M, wl.N), dtype=torch.float32, device=dev) for _ in range(sets)]
    tune = dict(tile_n=args.tile_n, strips_per_wg=args.strips_per_wg, kernel=args.kernel)
    kernel_name = g.spmm_kernel_name(A, Xs[0], wl.N, wl.N, **tune)

    def step(i):
        j = i % sets
        g.spmm(A, Xs[j], wl.N, wl.N, Ys[j], wl.N, stream, **tune)

    t_cold, wall_cold = time_launches(torch, step, args.steps, args.warmup)
    t_warm, _ = time_launches(torch, lambda i: g.spmm(A, Xs[0], wl.N, wl.N, Ys[0], wl.N, stream, **tune),
                              args.steps, args.warmup)
    flops = wl.useful_flops()
    abytes = spmm_algorithmic_bytes(vd, wl.N, 2)
    value = flops / t_cold / 1e12
    achieved = abytes / t_cold / 1e9
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_cold * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "c2: VGG-style 3x3 conv as im2col BCR SpMM, M=256 K=2304 N=3136, fp16 in / fp32 acc, "
                               "16x32 blocks keep 8/16 rows x 8/32 cols (density 1/8)",
                   "buffer_sets": sets, "useful_gflop_per_step": flops / 1e9, "algorithmic_mb_per_step": abytes / 1e6},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": C2_TRAFFIC_BYTES.get(kernel_name),
                     "kernel": kernel_name, "launch_us": t_cold * 1e6},
        "warm_cache": {"ms_per_step": t_warm * 1e3, "useful_tflops": flops / t_warm / 1e12,
                       "algorithmic_gbs": abytes / t_warm / 1e9,
                       "note": "same X/Y every step: operands stay in the 256 MB last-level cache"},
        "wall_ms_per_step": wall_cold * 1e3,
    }

    if args.calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = 256 << 20
        del src, dst

    if args.extra:
        extra = {}
        # ---- c3: LSTM gate SpMV, batch 1 and 8: (A) same W, (B) rotating copies, (C) one batched launch
        for batch in (1, 8):
            w3 = gen.c3_lstm_gates(batch)
            copies = 256
            mats = [pack(w3) for _ in range(copies)]
            v3 = view_dict(mats[0])
            xs = dev_tensor(np.stack([w3.X] * copies), w3.dtype)
            ys = torch.empty((copies, w3.M, batch), dtype=torch.float32, device=dev)
            b3 = spmv_algorithmic_bytes(v3, batch, 2)
            # single calls: raw addresses, so that the host side of a call is the C entry point and little else
            xa = [int(xs[j].data_ptr()) for j in range(copies)]
            ya = [int(ys[j].data_ptr()) for j in range(copies)]
            sh = int(stream.cuda_stream)
            tA, _ = time_launches(torch, lambda i: g.spmv(mats[0], xa[0], batch, batch, ya[0], batch, sh), 1000, 50)
            tB, _ = time_launches(torch, lambda i: g.spmv(mats[i % copies], xa[i % copies], batch, batch, ya[i % copies], batch, sh), 1000, 50)
            # the same 1000 independent calls recorded once into a HIP graph and replayed (no host work per call)
            gstream = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(gstream):
                gh = int(gstream.cuda_stream)
                for i in range(20):
                    g.spmv(mats[i % copies], xa[i % copies], batch, batch, ya[i % copies], batch, gh)
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=gstream):
                    for i in range(1000):
                        g.spmv(mats[i % copies], xa[i % copies], batch, batch, ya[i % copies], batch, gh)
            torch.cuda.synchronize()
            tD = float("inf")
            for _ in range(3):
                t0 = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                tD = min(tD, (time.perf_counter() - t0) / 1000)
            del graph
            G = binding.group(mats)
            tC, _ = time_launches(torch, lambda i: g.spmv_batched(G, xs, w3.K * batch, batch, batch, ys, w3.M * batch, batch, stream), 20, 3)
            tC /= copies
            extra[f"c3_b{batch}"] = {
                "algorithmic_mb": b3 / 1e6, "useful_mflop": w3.useful_flops() / 1e6,
                "A_same_W_us": tA * 1e6, "A_gbs": b3 / tA / 1e9,
                "B_rotating_us": tB * 1e6, "B_gbs": b3 / tB / 1e9, "B_frac_hbm": b3 / tB / 1e9 / HBM_PEAK_GBS,
                "C_batched_us_per_product": tC * 1e6, "C_gbs": b3 / tC / 1e9, "C_frac_hbm": b3 / tC / 1e9 / HBM_PEAK_GBS,
                "C_products_per_launch": copies,
                "D_graph_of_1000_calls_us_per_call": tD * 1e6, "D_gbs": b3 / tD / 1e9,
            }
            # the same matrix as an LSTM layer (hidden = input = 1024): one step = gate product + cell
            Hh = w3.M // 4
            xh = [dev_tensor(w3.X, w3.dtype).clone() for _ in range(2)]
            gates = torch.empty((w3.M, batch), dtype=torch.float32, device=dev)
            cst = torch.zeros((Hh, batch), dtype=torch.float32, device=dev)

            def lstm(i):
                g.lstm_step(mats[0], xh[i % 2], batch, batch, gates, batch, None, cst, batch, xh[(i + 1) % 2][w3.K - Hh:],
                            batch, None, 0, stream)
            tL, _ = time_launches(torch, lstm, 1000, 50)
            extra[f"c3_b{batch}"]["lstm_step_us"] = tL * 1e6
            del G, mats
        # ---- a GRU layer of the paper's size (Section 5: hidden 1024, both gate matrices 3072 x 1024, pruned 10x,
        #      32 x 32 blocks): one step = two products + the cell, at batch 1, 8 and 32 (the paper quotes batch 32)
        from paper_2108_11033_amd import tune
        Hg = 1024
        Wgi, _, mgi = tune.synthesize(3 * Hg, Hg, 1, 32, 32, 10.0, "f16", seed=1)
        Wgh, _, mgh = tune.synthesize(3 * Hg, Hg, 1, 32, 32, 10.0, "f16", seed=2)
        Agi = g.pack(Wgi, "f16", 32, 32, mgi.row_ptr, mgi.row_idx, mgi.col_ptr, mgi.col_idx)
        Agh = g.pack(Wgh, "f16", 32, 32, mgh.row_ptr, mgh.row_idx, mgh.col_ptr, mgh.col_idx)
        gru = {}
        for batch in (1, 8, 32):
            xg = dev_tensor(gen.normal_activations(Hg, batch, "f16", seed=9), "f16")
            hb = torch.zeros((Hg, batch), dtype=torch.float16, device=dev)
            h32 = torch.zeros((Hg, batch), dtype=torch.float32, device=dev)
            gi_ = torch.empty((3 * Hg, batch), dtype=torch.float32, device=dev)
            gh_ = torch.empty((3 * Hg, batch), dtype=torch.float32, device=dev)
            tG, _ = time_launches(torch, lambda i: g.gru_step(Agi, Agh, xg, batch, hb, batch, batch, gi_, batch, gh_, batch,
                                                              None, None, h32, batch, hb, batch, stream), 500, 50)
            gru[f"b{batch}_step_us"] = tG * 1e6
        gru["kernel_b32"] = g.spmm_kernel_name(Agi, xg, 32, 32)
        # the three GRU matrix sizes the paper counts register loads on (Section 5.3), pruned 10.7x: one product each
        shapes = {}
        for (Mg, Kg, BRg, BCg, krg, kcg) in ((152, 1024, 8, 32, 4, 6), (512, 1024, 32, 32, 8, 12), (1024, 1024, 32, 32, 8, 12)):
            mk = gen.random_mask(Mg, Kg, BRg, BCg, krg, kcg, seed=40 + Mg)
            Wg = gen.normal_weights(Mg, Kg, "f16", seed=41 + Mg)
            Ag = g.pack(Wg, "f16", BRg, BCg, mk.row_ptr, mk.row_idx, mk.col_ptr, mk.col_idx)
            rec = {}
            for batch in (1, 32):
                xg2 = dev_tensor(gen.normal_activations(Kg, batch, "f16", seed=9), "f16")
                yg2 = torch.empty((Mg, batch), dtype=torch.float32, device=dev)
                xa2, ya2, sh2 = int(xg2.data_ptr()), int(yg2.data_ptr()), int(stream.cuda_stream)
                tg, _ = time_launches(torch, lambda i: g.spmm(Ag, xa2, batch, batch, ya2, batch, sh2), 500, 50)
                rec[f"b{batch}_us"] = tg * 1e6
                rec[f"b{batch}_kernel"] = g.spmm_kernel_name(Ag, xg2, batch, batch)
            shapes[f"{Mg}x{Kg}"] = rec
            del Ag
        gru["paper_shapes"] = shapes
        extra["gru_1024"] = gru
        del Agi, Agh
        # ---- c5: large non-uniform bf16 SpMM
        w5 = gen.c5_nonuniform()
        A5 = pack(w5)
        v5 = view_dict(A5)
        X5 = dev_tensor(w5.X, w5.dtype)
        X5b = X5.clone()
        Y5 = [torch.empty((w5.M, w5.N), dtype=torch.float32, device=dev) for _ in range(2)]
        XX = [X5, X5b]
        t5, _ = time_launches(torch, lambda i: g.spmm(A5, XX[i % 2], w5.N, w5.N, Y5[i % 2], w5.N, stream), 50, 5)
        b5 = spmm_algorithmic_bytes(v5, w5.N, 2)
        extra["c5"] = {"us": t5 * 1e6, "useful_tflops": w5.useful_flops() / t5 / 1e12, "algorithmic_mb": b5 / 1e6,
                       "gbs": b5 / t5 / 1e9, "frac_hbm": b5 / t5 / 1e9 / HBM_PEAK_GBS, "nnz": v5["nnz"],
                       "mma_layout_mb": v5["dev_bytes_mma"] / 1e6}
        extra["c5"]["kernel"] = g.spmm_kernel_name(A5, X5, w5.N, w5.N)
        del X5, X5b, Y5, XX, A5
        # ---- c2's layer at a large N (224 x 224 positions): the same weights, 16x the columns
        wb = gen.c2_vgg_conv(50176)
        Ab = pack(wb)
        vb = view_dict(Ab)
        Xb = [dev_tensor(wb.X, wb.dtype)]
        Xb.append(Xb[0].clone())
        Yb = [torch.empty((wb.M, wb.N), dtype=torch.float32, device=dev) for _ in range(2)]
        tb, _ = time_launches(torch, lambda i: g.spmm(Ab, Xb[i % 2], wb.N, wb.N, Yb[i % 2], wb.N, stream), 30, 3)
        bb = spmm_algorithmic_bytes(vb, wb.N, 2)
        extra["c2_N50176"] = {"us": tb * 1e6, "useful_tflops": wb.useful_flops() / tb / 1e12, "algorithmic_mb": bb / 1e6,
                              "gbs": bb / tb / 1e9, "frac_hbm": bb / tb / 1e9 / HBM_PEAK_GBS,
                              "kernel": g.spmm_kernel_name(Ab, Xb[0], wb.N, wb.N)}
        del Xb, Yb, Ab
        # ---- c4: the 13 VGG-16 conv layers
        layers = []
        tot_t = tot_b = tot_f = 0.0
        for li in range(13):
            w4 = gen.c4_vgg16_layer(li)
            A4 = pack(w4)
            v4 = view_dict(A4)
            nset = 4
            X4 = [dev_tensor(w4.X, w4.dtype)]
            X4 += [X4[0].clone() for _ in range(nset - 1)]
            Y4 = [torch.empty((w4.M, w4.N), dtype=torch.float32, device=dev) for _ in range(nset)]
            t4, _ = time_launches(torch, lambda i: g.spmm(A4, X4[i % nset], w4.N, w4.N, Y4[i % nset], w4.N, stream), 100, 10)
            b4 = spmm_algorithmic_bytes(v4, w4.N, 2)
            layers.append({"layer": li + 1, "M": w4.M, "K": w4.K, "N": w4.N, "us": t4 * 1e6,
                           "useful_tflops": w4.useful_flops() / t4 / 1e12, "gbs": b4 / t4 / 1e9,
                           "kernel": g.spmm_kernel_name(A4, X4[0], w4.N, w4.N)})
            tot_t += t4; tot_b += b4; tot_f += w4.useful_flops()
            del X4, Y4, A4
        extra["c4"] = {"layers": layers, "total_us": tot_t * 1e6, "useful_tflops": tot_f / tot_t / 1e12,
                       "gbs": tot_b / tot_t / 1e9, "frac_hbm": tot_b / tot_t / 1e9 / HBM_PEAK_GBS}
        out["extra"] = extra

    if args.conv:
        # c2's layer fed with the feature map it stands for: 256 channels of 56 x 56, 3 x 3 kernel, same padding
        Cin, Hc, Wc = 256, 56, 56
        F0 = dev_tensor(gen.normal_activations(Cin, Hc * Wc, wl.dtype, seed=77, relu=True), wl.dtype)
        Fs = [F0] + [F0.clone() for _ in range(sets - 1)]
        tc, _ = time_launches(torch, lambda i: g.conv2d(A, Fs[i % sets], Cin, Hc, Wc, 3, 3, Ys[i % sets], wl.N, stream),
                              args.steps, args.warmup)
        cbytes = abytes - wl.K * wl.N * 2 + Cin * Hc * Wc * 2
        # context: what forming the matrix costs with the library routine of the framework that owns the buffers
        unfold = lambda i: torch.nn.functional.unfold(Fs[i % sets].view(1, Cin, Hc, Wc), 3, padding=1)
        tu, _ = time_launches(torch, unfold, 100, 10)
        out["conv"] = {"workload": "c2's weights on a 256 x 56 x 56 fp16 feature map, 3x3, zero padding 1",
                       "us": tc * 1e6, "useful_tflops": flops / tc / 1e12, "algorithmic_mb": cbytes / 1e6,
                       "gbs": cbytes / tc / 1e9, "product_on_materialised_im2col_us": t_cold * 1e6,
                       "torch_unfold_us": tu * 1e6, "im2col_matrix_mb": wl.K * wl.N * 2 / 1e6}
        # the layer as networks chain it: bias + rectifier in the epilogue, fp16 out (the next layer's feature map)
        bias_c = torch.zeros(wl.M, dtype=torch.float32, device=dev)
        Os = [torch.empty((wl.M, wl.N), dtype=torch.float16, device=dev) for _ in range(sets)]
        ta, _ = time_launches(torch, lambda i: g.conv2d_act(A, Fs[i % sets], Cin, Hc, Wc, 3, 3, bias_c, True, Os[i % sets],
                                                            "f16", wl.N, stream), args.steps, args.warmup)
        out["conv"]["bias_relu_fp16_out_us"] = ta * 1e6
        del Os
        # the same layer on a 224 x 224 map (N = 50176): the matrix would be 231 MB
        Hb = 224
        Fb = [dev_tensor(gen.normal_activations(Cin, Hb * Hb, wl.dtype, seed=78 + i, relu=True), wl.dtype) for i in range(2)]
        Yb_ = [torch.empty((wl.M, Hb * Hb), dtype=torch.float32, device=dev) for _ in range(2)]
        tcb, _ = time_launches(torch, lambda i: g.conv2d(A, Fb[i % 2], Cin, Hb, Hb, 3, 3, Yb_[i % 2], Hb * Hb, stream), 30, 3)
        tub, _ = time_launches(torch, lambda i: torch.nn.functional.unfold(Fb[i % 2].view(1, Cin, Hb, Hb), 3, padding=1), 10, 2)
        out["conv"]["at_224x224"] = {"us": tcb * 1e6, "useful_tflops": 2.0 * vd["nnz"] * Hb * Hb / tcb / 1e12,
                                     "torch_unfold_us": tub * 1e6, "im2col_matrix_mb": wl.K * Hb * Hb * 2 / 1e6}
        del Fb, Yb_
        # the 13 VGG-16 conv layers (c4's weights) as fused layers: convolution + bias + rectifier + fp16 output,
        # each from a feature map of its input size (pooling between the stages is not part of this library)
        stack = []
        tot = 0.0
        for li in range(13):
            Mv, Kv, Nv = gen.VGG16_LAYERS[li]
            Cv, Hv = Kv // 9, int(round(Nv ** 0.5))
            w4 = gen.c4_vgg16_layer(li, N=64)
            A4 = pack(w4)
            Fv = [dev_tensor(gen.normal_activations(Cv, Nv, "f16", seed=90 + li + 20 * i, relu=True), "f16") for i in range(2)]
            Ov = [torch.empty((Mv, Nv), dtype=torch.float16, device=dev) for _ in range(2)]
            bv = torch.zeros(Mv, dtype=torch.float32, device=dev)
            tv, _ = time_launches(torch, lambda i: g.conv2d_act(A4, Fv[i % 2], Cv, Hv, Hv, 3, 3, bv, True, Ov[i % 2], "f16", Nv, stream),
                                  50, 5)
            stack.append(tv * 1e6)
            tot += tv
            del A4, Fv, Ov
        out["conv"]["vgg16_13_fused_layers_us"] = stack
        out["conv"]["vgg16_13_fused_layers_total_us"] = tot * 1e6
        del Fs

    if args.sweep:
        from paper_2108_11033_amd import tune
        sweep = {}
        sizes = [(4, 4), (8, 8), (16, 16), (16, 32), (32, 32), (16, 64), (32, 64), (64, 64), (16, 128), (32, 128)]
        # matrix-vector layer (the paper's RNN case), 256 independent products per launch; and the same layer as a GEMM
        for name, n, products in (("spmv_256_products", 1, 256), ("spmm_N3136", 3136, 1)):
            cand = [s for s in sizes if n > 8 or (s[0] <= 32 and s[1] <= 32)]
            best, trace = tune.find_block_size(1024, 1024, n, 10.0, cand, dtype="f16", threshold=1.1,
                                               products=products, steps=30, warmup=3)
            # the search stops early; time the remaining sizes too so that the whole curve is on record
            seen = {s for s, _ in trace}
            rest = []
            for sz in cand:
                if sz not in seen:
                    W_, X_, m_ = tune.synthesize(1024, 1024, n, sz[0], sz[1], 10.0, "f16")
                    rest.append((sz, tune.time_layer(W_, X_, m_, "f16", products=products, steps=30, warmup=3)))
            sweep[name] = {"chosen": list(best) if best else None,
                           "searched_us": [[list(sz), t * 1e6] for sz, t in trace],
                           "not_searched_us": [[list(sz), t * 1e6] for sz, t in rest]}
        # strip reorder on / off on c5 (work per strip varies there)
        w5 = gen.c5_nonuniform()
        t_on = tune.time_layer(w5.W, w5.X, w5.mask, w5.dtype, steps=30, warmup=3)
        t_off = tune.time_layer(w5.W, w5.X, w5.mask, w5.dtype, steps=30, warmup=3, no_reorder=True)
        sweep["c5_reorder"] = {"reordered_us": t_on * 1e6, "natural_order_us": t_off * 1e6, "ratio": t_off / t_on}
        out["sweep"] = sweep

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
