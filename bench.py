#!/usr/bin/env python3
"""Benchmark of the BCR sparse product on one MI355X.

A step is one pass of the hot path -- one grim_bcr_spmm call: weight + index load, activation
gather, sub-block contraction, scatter-accumulate and store -- over one batch of synthetic input of
the headline workload, the largest configured one: the non-uniform BCR SpMM c5 (M=512, K=4608,
N=25088 = batch 8 at 56x56, bf16 in / fp32 accumulate, 32x32 blocks whose kept-row and kept-column
fractions are drawn from {1/8, 1/4, 1/2}).  Inputs are resident in HBM before the timed region and
the steps alternate between two (X, Y) buffer sets (565 MB, more than the 256 MB last-level cache).
The same JSON line carries, under "configs", the other configured workloads (c1, c2, c3 at batch 1
and 8 in the three call forms, the 13 layers of c4, c2's layer at N = 50176) with time, algorithmic
GB/s, fraction of the HBM roof and the kernel that ran.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--headline-only] [--extra] [--conv] [--sweep]
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
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by what
# the same counter reads for a device copy of known size (x 2.0 fetched, x 1.0 written), keyed by (workload, kernel);
# the profile under profiles/ that holds the two counter runs is named beside each entry.  A (workload, kernel) pair
# that no committed profile covers reports null and says so.
TRAFFIC_BYTES = {
    ("c2", "bcr_spmm_gather"): ((7765.9 * 2.0 + 3136.0) * 1024, "profiles/bcr_spmm_gather_c2.md"),
    ("c2", "bcr_spmm_mma"): ((7834.0 * 2.0 + 3136.0) * 1024, "profiles/bcr_spmm_mma_c2.md"),
    # one step = one launch: wide-tile workgroups on 24576 columns, row-gathering workgroups on the last 512
    ("c5", "bcr_spmm_wide"): ((117914.7 * 2.0 + 50264.6) * 1024, "profiles/bcr_spmm_wide_c5.md"),
}


def traffic_of(workload: str, kernel: str):
    hit = TRAFFIC_BYTES.get((workload, kernel))
    if hit is None:
        return None, f"no committed rocprofv3 counter run covers kernel {kernel} on {workload}"
    return hit[0], hit[1]

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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tile-n", type=int, default=0)
    ap.add_argument("--strips-per-wg", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 choose, 2 staged matrix-core kernel, 3 row-gathering one")
    ap.add_argument("--headline-only", action="store_true", help="time the headline workload only (no \"configs\" object)")
    ap.add_argument("--extra", action="store_true",
                    help="also time the recurrent steps (LSTM on c3's matrix, a GRU layer of the paper's size), the GRU "
                         "matrix sizes of the paper's register-load study and a HIP graph of 1000 SpMV calls")
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

    def spmm_record(wl, sets, steps, warmup, tune=None, key=None):
        """Time grim_bcr_spmm on a workload, rotating over `sets` (X, Y) buffer sets; returns (record, A, Xs, Ys)."""
        tune = tune or {}
        A = pack(wl)
        vd = view_dict(A)
        X0 = dev_tensor(wl.X, wl.dtype)
        Xs = [X0] + [X0.clone() for _ in range(sets - 1)]
        Ys = [torch.empty((wl.M, wl.N), dtype=torch.float32, device=dev) for _ in range(sets)]
        t, wall = time_launches(torch, lambda i: g.spmm(A, Xs[i % sets], wl.N, wl.N, Ys[i % sets], wl.N, stream, **tune),
                                steps, warmup)
        esz = gen.storage_itemsize(wl.dtype)
        ab = spmm_algorithmic_bytes(vd, wl.N, esz)
        kernel = g.spmm_kernel_name(A, Xs[0], wl.N, wl.N, **tune)
        traffic, src = traffic_of(key or wl.name, kernel)
        rec = {"us": t * 1e6, "useful_tflops": wl.useful_flops() / t / 1e12, "algorithmic_mb": ab / 1e6,
               "gbs": ab / t / 1e9, "frac_hbm": ab / t / 1e9 / HBM_PEAK_GBS, "kernel": kernel,
               "M": wl.M, "K": wl.K, "N": wl.N, "nnz": vd["nnz"], "buffer_sets": sets,
               "buffer_set_mb": (esz * wl.K * wl.N + 4 * wl.M * wl.N) / 1e6, "traffic": traffic, "traffic_source": src,
               "wall_us": wall * 1e6}
        return rec, A, Xs, Ys

    # ---------------- headline: c5, the largest configured workload ----------------
    wl = gen.c5_nonuniform()
    tune = dict(tile_n=args.tile_n, strips_per_wg=args.strips_per_wg, kernel=args.kernel)
    sets = 2
    head, A, Xs, Ys = spmm_record(wl, sets, args.steps, args.warmup, tune)
    t_cold = head["us"] * 1e-6
    flops = wl.useful_flops()
    abytes = head["algorithmic_mb"] * 1e6
    out = {
        "metric": METRIC, "value": head["useful_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t_cold * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c5: large non-uniform BCR SpMM, M=512 K=4608 N=25088 (batch 8 at 56x56), bf16 in / fp32 "
                               "acc, 32x32 blocks, per block kept-row and kept-col fractions drawn from {1/8,1/4,1/2}",
                   "buffer_sets": sets, "useful_gflop_per_step": flops / 1e9, "algorithmic_mb_per_step": abytes / 1e6,
                   "nnz": head["nnz"]},
        "roofline": {"bound": "hbm", "achieved": head["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["frac_hbm"], "traffic": head["traffic"], "traffic_source": head["traffic_source"],
                     "kernel": head["kernel"], "launch_us": head["us"],
                     "hbm_roof_useful_tflops": flops / (abytes / (HBM_PEAK_GBS * 1e9)) / 1e12,
                     "frac_of_mfma_peak": head["useful_tflops"] / 2500.0},
        "wall_ms_per_step": head["wall_us"] * 1e-3,
    }
    del A, Xs, Ys

    if args.calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = 256 << 20
        del src, dst

    c3_mats = {}
    if not args.headline_only:
        cfg = {}
        # ---- c1: the small fp32 case (latency-bound: 0.17 MB)
        r1, A1, X1, Y1 = spmm_record(gen.c1_single_fp32(), 1, 500, 50)
        cfg["c1"] = r1
        del A1, X1, Y1
        # ---- c2: rotating over 32 buffer sets (565 MB) and with the same operands every step (last-level cache)
        w2 = gen.c2_vgg_conv()
        r2, A2, X2, Y2 = spmm_record(w2, 32, 400, 40)
        tw, _ = time_launches(torch, lambda i: g.spmm(A2, X2[0], w2.N, w2.N, Y2[0], w2.N, stream), 400, 40)
        r2["warm_cache_us"] = tw * 1e6
        r2["warm_cache_gbs"] = r2["algorithmic_mb"] * 1e6 / tw / 1e9
        cfg["c2"] = r2
        del A2, X2, Y2
        # ---- c3: LSTM gate SpMV, batch 1 and 8: (A) same W back to back, (B) rotating over 256 packed copies,
        #      (C) the 256 products in one batched launch
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
            G = binding.group(mats)
            tC, _ = time_launches(torch, lambda i: g.spmv_batched(G, xs, w3.K * batch, batch, batch, ys, w3.M * batch, batch, stream), 20, 3)
            tC /= copies
            cfg[f"c3_b{batch}"] = {
                "algorithmic_mb": b3 / 1e6, "useful_mflop": w3.useful_flops() / 1e6, "calls_timed": 1000,
                "A_same_W_us": tA * 1e6, "A_gbs": b3 / tA / 1e9,
                "B_rotating_us": tB * 1e6, "B_gbs": b3 / tB / 1e9, "B_frac_hbm": b3 / tB / 1e9 / HBM_PEAK_GBS,
                "C_batched_us_per_product": tC * 1e6, "C_gbs": b3 / tC / 1e9, "C_frac_hbm": b3 / tC / 1e9 / HBM_PEAK_GBS,
                "C_products_per_launch": copies,
                "kernel": g.spmm_kernel_name(mats[0], xa[0], batch, batch),
            }
            del G
            c3_mats[batch] = (w3, mats, xs, ys, xa, ya)
            if not args.extra:
                c3_mats.pop(batch)
                del mats, xs, ys
        # ---- c2's layer at a large N (224 x 224 positions): the same weights, 16x the columns
        rb, Ab, Xb, Yb = spmm_record(gen.c2_vgg_conv(50176), 2, 30, 3, key="c2_N50176")
        cfg["c2_N50176"] = rb
        del Ab, Xb, Yb
        # ---- c4: the 13 VGG-16 conv layers
        layers = []
        tot_t = tot_b = tot_f = 0.0
        for li in range(13):
            w4 = gen.c4_vgg16_layer(li)
            r4, A4, X4, Y4 = spmm_record(w4, 4, 100, 10, key=f"c4_L{li + 1}")
            layers.append({"layer": li + 1, "M": w4.M, "K": w4.K, "N": w4.N, "us": r4["us"],
                           "useful_tflops": r4["useful_tflops"], "gbs": r4["gbs"], "frac_hbm": r4["frac_hbm"],
                           "kernel": r4["kernel"]})
            tot_t += r4["us"] * 1e-6; tot_b += r4["algorithmic_mb"] * 1e6; tot_f += w4.useful_flops()
            del X4, Y4, A4
        cfg["c4"] = {"layers": layers, "total_us": tot_t * 1e6, "useful_tflops": tot_f / tot_t / 1e12,
                     "algorithmic_mb": tot_b / 1e6, "gbs": tot_b / tot_t / 1e9, "frac_hbm": tot_b / tot_t / 1e9 / HBM_PEAK_GBS}
        out["configs"] = cfg

    if args.extra:
        extra = {}
        for batch in (1, 8):
            if batch not in c3_mats:
                w3 = gen.c3_lstm_gates(batch)
                copies = 256
                mats = [pack(w3) for _ in range(copies)]
                xs = dev_tensor(np.stack([w3.X] * copies), w3.dtype)
                ys = torch.empty((copies, w3.M, batch), dtype=torch.float32, device=dev)
                xa = [int(xs[j].data_ptr()) for j in range(copies)]
                ya = [int(ys[j].data_ptr()) for j in range(copies)]
            else:
                w3, mats, xs, ys, xa, ya = c3_mats.pop(batch)
                copies = len(mats)
            b3 = spmv_algorithmic_bytes(view_dict(mats[0]), batch, 2)
            # the 1000 independent calls recorded once into a HIP graph and replayed (no host work per call)
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
            extra[f"c3_b{batch}"] = {"D_graph_of_1000_calls_us_per_call": tD * 1e6, "D_gbs": b3 / tD / 1e9}
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
            extra[f"c3_b{batch}"]["lstm_step_launches"] = g.rnn_step_launches(mats[0], None, batch)
            if batch == 1 and g.rnn_sequence_supported(mats[0]):
                # T steps in one launch (weights stay in registers, h passes between workgroups through tagged words)
                Ih = w3.K - Hh
                status = torch.zeros((1,), dtype=torch.int32, device=dev)
                for T in (16, 256):
                    xs_t = dev_tensor(gen.normal_activations(Ih, T, w3.dtype, seed=11), w3.dtype).t().contiguous()
                    h0 = torch.zeros((Hh,), dtype=xs_t.dtype, device=dev)
                    cs = torch.zeros((Hh,), dtype=torch.float32, device=dev)
                    hs = torch.empty((T, Hh), dtype=xs_t.dtype, device=dev)
                    tS, _ = time_launches(torch, lambda i: g.lstm_sequence(mats[0], xs_t, Ih, T, None, h0, cs, hs, Hh, None, 0,
                                                                           status, 0, stream), 10, 2)
                    torch.cuda.synchronize()
                    assert int(status.item()) == 0
                    extra[f"c3_b{batch}"][f"lstm_sequence_T{T}_us_per_step"] = tS * 1e6 / T
                # 2 .. 32 sequences side by side in the same launch (up to 8 as sets of workgroups, then several per workgroup)
                T = 256
                for nb in (2, 4, 8, 16, 32):
                    if not g.rnn_sequence_supported(mats[0], None, nb):
                        continue
                    xs_b = dev_tensor(gen.normal_activations(Ih, T * nb, w3.dtype, seed=13), w3.dtype).t().contiguous()
                    h0 = torch.zeros((nb, Hh), dtype=xs_b.dtype, device=dev)
                    cs = torch.zeros((nb, Hh), dtype=torch.float32, device=dev)
                    hs = torch.empty((T * nb, Hh), dtype=xs_b.dtype, device=dev)
                    tS, _ = time_launches(torch, lambda i: g.lstm_sequence_batch(mats[0], xs_b, Ih, T, nb, None, h0, cs, hs, Hh,
                                                                                 None, 0, status, 0, stream), 10, 2)
                    torch.cuda.synchronize()
                    assert int(status.item()) == 0
                    extra[f"c3_b{batch}"][f"lstm_sequence_batch{nb}_T{T}_us_per_step"] = tS * 1e6 / T
            del mats, xs, ys
        # ---- a GRU layer of the paper's size (Section 6.1: hidden 1024, both gate matrices 3072 x 1024, 32 x 32 blocks
        #      keeping 8 rows x 12 columns = pruned 10.7x, the rate of Section 6.4): one step = two products + the cell,
        #      at batch 1, 8 and 32 (Section 6.3 quotes batch 32)
        from paper_2108_11033_amd import tune as tune_mod
        Hg = 1024
        Wgi, _, mgi = tune_mod.synthesize(3 * Hg, Hg, 1, 32, 32, 1024 / 96, "f16", seed=1, row_frac=0.25)
        Wgh, _, mgh = tune_mod.synthesize(3 * Hg, Hg, 1, 32, 32, 1024 / 96, "f16", seed=2, row_frac=0.25)
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
            gru[f"b{batch}_step_in_place_us"] = tG * 1e6          # new state over the old: products, then the cell kernel
            gru[f"b{batch}_step_launches"] = g.rnn_step_launches(Agi, Agh, batch)
            # new state into a second buffer: the step is then one launch (the cell in the products' kernel)
            hb2 = torch.zeros((Hg, batch), dtype=torch.float16, device=dev)
            hbs = [hb, hb2]
            tG1, _ = time_launches(torch, lambda i: g.gru_step(Agi, Agh, xg, batch, hbs[i % 2], batch, batch, gi_, batch, gh_,
                                                               batch, None, None, h32, batch, hbs[(i + 1) % 2], batch, stream),
                                   500, 50)
            gru[f"b{batch}_step_us"] = tG1 * 1e6
        if g.rnn_sequence_supported(Agi, Agh):
            status = torch.zeros((1,), dtype=torch.int32, device=dev)
            for T in (16, 256):
                xs_t = dev_tensor(gen.normal_activations(Hg, T, "f16", seed=12), "f16").t().contiguous()
                h0 = torch.zeros((Hg,), dtype=torch.float16, device=dev)
                hst = torch.zeros((Hg,), dtype=torch.float32, device=dev)
                hs = torch.empty((T, Hg), dtype=torch.float16, device=dev)
                tS, _ = time_launches(torch, lambda i: g.gru_sequence(Agi, Agh, xs_t, Hg, T, None, None, h0, hst, hs, Hg, None, 0,
                                                                      status, 0, stream), 10, 2)
                torch.cuda.synchronize()
                assert int(status.item()) == 0
                gru[f"sequence_T{T}_us_per_step"] = tS * 1e6 / T
            T = 256
            for nb in (2, 4, 8, 16, 32):
                if not g.rnn_sequence_supported(Agi, Agh, nb):
                    continue
                xs_b = dev_tensor(gen.normal_activations(Hg, T * nb, "f16", seed=14), "f16").t().contiguous()
                h0 = torch.zeros((nb, Hg), dtype=torch.float16, device=dev)
                hst = torch.zeros((nb, Hg), dtype=torch.float32, device=dev)
                hs = torch.empty((T * nb, Hg), dtype=torch.float16, device=dev)
                tS, _ = time_launches(torch, lambda i: g.gru_sequence_batch(Agi, Agh, xs_b, Hg, T, nb, None, None, h0, hst, hs, Hg,
                                                                            None, 0, status, 0, stream), 10, 2)
                torch.cuda.synchronize()
                assert int(status.item()) == 0
                gru[f"sequence_batch{nb}_T{T}_us_per_step"] = tS * 1e6 / T
        gru["kernel_b32"] = g.spmm_kernel_name(Agi, xg, 32, 32)
        # the three GRU matrix sizes the paper counts register loads on (Section 6.4), pruned 10.7x: one product each
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
        out["extra"] = extra

    if args.conv:
        # c2's layer fed with the feature map it stands for: 256 channels of 56 x 56, 3 x 3 kernel, same padding
        Cin, Hc, Wc = 256, 56, 56
        wc = gen.c2_vgg_conv()
        csets = 32
        rc, Ac, Xc, Yc = spmm_record(wc, csets, 400, 40)
        del Xc
        vdc = view_dict(Ac)
        F0 = dev_tensor(gen.normal_activations(Cin, Hc * Wc, wc.dtype, seed=77, relu=True), wc.dtype)
        Fs = [F0] + [F0.clone() for _ in range(csets - 1)]
        tc, _ = time_launches(torch, lambda i: g.conv2d(Ac, Fs[i % csets], Cin, Hc, Wc, 3, 3, Yc[i % csets], wc.N, stream),
                              400, 40)
        cbytes = rc["algorithmic_mb"] * 1e6 - wc.K * wc.N * 2 + Cin * Hc * Wc * 2
        # context: what forming the matrix costs with the library routine of the framework that owns the buffers
        unfold = lambda i: torch.nn.functional.unfold(Fs[i % csets].view(1, Cin, Hc, Wc), 3, padding=1)
        tu, _ = time_launches(torch, unfold, 100, 10)
        out["conv"] = {"workload": "c2's weights on a 256 x 56 x 56 fp16 feature map, 3x3, zero padding 1",
                       "us": tc * 1e6, "useful_tflops": wc.useful_flops() / tc / 1e12, "algorithmic_mb": cbytes / 1e6,
                       "gbs": cbytes / tc / 1e9, "product_on_materialised_im2col_us": rc["us"],
                       "torch_unfold_us": tu * 1e6, "im2col_matrix_mb": wc.K * wc.N * 2 / 1e6}
        # the layer as networks chain it: bias + rectifier in the epilogue, fp16 out (the next layer's feature map)
        bias_c = torch.zeros(wc.M, dtype=torch.float32, device=dev)
        Os = [torch.empty((wc.M, wc.N), dtype=torch.float16, device=dev) for _ in range(csets)]
        ta, _ = time_launches(torch, lambda i: g.conv2d_act(Ac, Fs[i % csets], Cin, Hc, Wc, 3, 3, bias_c, True, Os[i % csets],
                                                            "f16", wc.N, stream), 400, 40)
        out["conv"]["bias_relu_fp16_out_us"] = ta * 1e6
        del Os
        # the same layer through a convolution plan (window starts and taps split when the plan is made)
        plan_c = g.ConvPlan(Ac, Cin, Hc, Wc, 3, 3, 1)
        tp, _ = time_launches(torch, lambda i: g.conv2d_plan(plan_c, Fs[i % csets], 1, 0, None, False, Yc[i % csets], "f32",
                                                             wc.N, 0, stream), 400, 40)
        out["conv"]["planned_us"] = tp * 1e6
        # at stride 2 (28 x 28 outputs)
        plan_s2 = g.ConvPlan(Ac, Cin, Hc, Wc, 3, 3, 2)
        Ys2 = [torch.empty((wc.M, 28 * 28), dtype=torch.float32, device=dev) for _ in range(csets)]
        ts2, _ = time_launches(torch, lambda i: g.conv2d_plan(plan_s2, Fs[i % csets], 1, 0, None, False, Ys2[i % csets], "f32",
                                                              28 * 28, 0, stream), 400, 40)
        out["conv"]["planned_stride2_us"] = ts2 * 1e6
        del Ys2, plan_c, plan_s2
        # the largest SpMM workload as what it stands for: a 3 x 3 convolution of 512 channels on a batch of 8 images of
        # 56 x 56 (the im2col matrix would be 231 MB; the feature maps are 25.7 MB)
        w5 = gen.c5_nonuniform()
        A5 = pack(w5)
        B5, C5, H5 = 8, 512, 56
        plan5 = g.ConvPlan(A5, C5, H5, H5, 3, 3, 1)
        F5 = [dev_tensor(gen.normal_activations(C5, B5 * H5 * H5, w5.dtype, seed=79 + i, relu=True), w5.dtype) for i in range(4)]
        Y5 = [torch.empty((B5, w5.M, H5 * H5), dtype=torch.float32, device=dev) for _ in range(4)]
        t5, _ = time_launches(torch, lambda i: g.conv2d_plan(plan5, F5[i % 4], B5, C5 * H5 * H5, None, False, Y5[i % 4], "f32",
                                                             H5 * H5, w5.M * H5 * H5, stream), 50, 5)
        v5 = view_dict(A5)
        b5 = C5 * H5 * H5 * B5 * 2 + w5.M * w5.N * 4 + v5["nnz"] * 2
        out["conv"]["c5_as_batch_of_8_images"] = {"us": t5 * 1e6, "useful_tflops": 2.0 * v5["nnz"] * w5.N / t5 / 1e12,
                                                   "algorithmic_mb": b5 / 1e6, "gbs": b5 / t5 / 1e9,
                                                   "frac_hbm": b5 / t5 / 1e9 / HBM_PEAK_GBS}
        del F5, Y5, plan5, A5
        # the same layer on a 224 x 224 map (N = 50176): the matrix would be 231 MB
        Hb = 224
        Fb = [dev_tensor(gen.normal_activations(Cin, Hb * Hb, wc.dtype, seed=78 + i, relu=True), wc.dtype) for i in range(2)]
        Yb_ = [torch.empty((wc.M, Hb * Hb), dtype=torch.float32, device=dev) for _ in range(2)]
        tcb, _ = time_launches(torch, lambda i: g.conv2d(Ac, Fb[i % 2], Cin, Hb, Hb, 3, 3, Yb_[i % 2], Hb * Hb, stream), 30, 3)
        tub, _ = time_launches(torch, lambda i: torch.nn.functional.unfold(Fb[i % 2].view(1, Cin, Hb, Hb), 3, padding=1), 10, 2)
        out["conv"]["at_224x224"] = {"us": tcb * 1e6, "useful_tflops": 2.0 * vdc["nnz"] * Hb * Hb / tcb / 1e12,
                                     "torch_unfold_us": tub * 1e6, "im2col_matrix_mb": wc.K * Hb * Hb * 2 / 1e6}
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
        del Fs, Ac, Yc

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
