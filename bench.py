#!/usr/bin/env python3
"""Benchmark of the dithered-backprop hot path on one MI355X.

One "step" = the whole hot path on the largest configuration of BASELINE.json, configs[4] ("config 5"): the
VGG-16 conv3-shaped layer in the 8-bit mode (batch 32, 256 -> 256 channels, 3x3, 56x56; int8 activations, fp32
weights, Delta chosen for 90 % zero codes): one NSD pass over the preactivation gradient (Eq. (qdz)) and the two
products dX and dW of the convolutional analogue of Eqs. (qda), (qdw), through the C ABI entry point
dithered_conv2d_backward with DBP_PATH_AUTO.  Inputs are synthetic (workloads.py) and resident in HBM before the
timed region; two buffer sets (2 x 260 MB) are rotated so that the 256 MB Infinity Cache cannot stand in for HBM.

Timing: every step is bracketed by its own pair of events on the launch stream and the MEDIAN step time is reported
(independent of how far the clocks have settled after `--warmup` steps); the mean over the same steps is kept beside it.

Prints ONE JSON line: whole-job dense-equivalent TFLOP/s of that step, `roofline` for its dominant kernel (the
method's algorithmic work: 2*nnz*C*R*S flops against the fp32 vector peak and the compulsory bytes against 8 TB/s,
with the executed matrix-core work as a separate, labelled field), `cpu_baseline` (the CPU oracle on the host cores,
one thread and all threads) and rows for every other configuration: configs 1-4, the MLP chain of configs[1] with
its per-kernel times, sweeps over the sparsity (config 5: 50...99 %, MLP: c = 2...64), the gather kernels with their
fraction of the fp32 vector peak, structured (dead-plane) gradients, the same library's dense fp32 backward and
torch's dense backward (context), and the NSD pass on a 2^28-element tensor.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_I8_TOPS = 5000.0
PEAK_F32_VECTOR_TFLOPS = 157.3
FLAG_OFFSET = 16384 * 16            # the density gate's flag inside the format's scratch region


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sparsity", type=float, default=0.90, help="target fraction of zero codes of the headline step")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--headline-only", action="store_true", help="skip the rows of the other configurations")
    ap.add_argument("--probe", choices=["conv_dx", "conv_dw", "nsd", "fc2"], default=None,
                    help="counter probe: one 1 GiB device copy of known size, then only the named kernel "
                         "(for `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives are part of the hot path); use --gpus 1")

    import numpy as np
    import torch
    import paper_2004_04729_amd as dbp
    import workloads

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn, iters, warm=3):
        """Median / mean / min seconds per call, every call between its own pair of events."""
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        # after an idle phase (host-side set-up, the CPU baseline) the GPU takes a while to return to its working clocks: keep
        # warming until about 30 ms of calls have run, so that every row is a steady-state figure like the headline's
        t0 = time.perf_counter()
        i = warm
        while time.perf_counter() - t0 < 0.03:
            fn(i)
            i += 1
            if i % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for i in range(iters):
            fn(i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        d = [ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(iters)]
        return {"median": statistics.median(d), "mean": sum(d) / len(d), "min": min(d)}

    def med(fn, iters, warm=3):
        return timed(fn, iters, warm)["median"]

    def captured(call):
        """A HIP graph of call(stream_handle): the library allocates and synchronises nothing, so its calls can be captured; replays
        save the host's launch work and the gaps between dependent kernels."""
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            call(side.cuda_stream)                                   # eager first: one-time function attributes are set outside a capture
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            call(torch.cuda.current_stream().cuda_stream)
        return g

    def conv_buffers(p, sets=1):
        N, Cc, H, Wd = p.X.shape
        K, _, R, S = p.W.shape
        i8 = p.X.dtype == np.int8
        xd = dbp.I8 if i8 else dbp.F32
        out = []
        for s in range(sets):
            perm = np.random.default_rng(99 + s).permutation(N) if s else np.arange(N)   # same law, different bytes per set
            b = dict(d=torch.from_numpy(p.delta[perm]).to(dev), X=torch.from_numpy(p.X[perm]).to(dev),
                     W=torch.from_numpy(p.W).to(dev).clone(),
                     codes=torch.empty(p.delta.shape, dtype=torch.int8, device=dev),
                     dX=torch.empty(p.X.shape, dtype=torch.float32, device=dev),
                     dW=torch.empty(p.W.shape, dtype=torch.int32 if i8 else torch.float32, device=dev),
                     ws=torch.zeros(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, p.stride, p.pad, xd), dtype=torch.uint8, device=dev),
                     st=torch.zeros(32, dtype=torch.uint8, device=dev))
            out.append(b)
        dims = (N, Cc, H, Wd, K, R, S)
        return out, dims, xd

    def conv_call(b, dims, xd, p, step, path=dbp.PATH_AUTO, dX=True, dW=True, on=None):
        N, Cc, H, Wd, K, R, S = dims
        dbp.dithered_conv2d_backward(b["d"], b["W"], b["X"], xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, step, p.seed, 0, b["codes"],
                                     b["dX"] if dX else None, b["dW"] if dW else None, b["ws"], b["st"], path, stream if on is None else on)

    def gate_flag(ws, rows, cols):
        """-1: one family was launched; else the state the device chose: 0 matrix cores, 1 the gather kernels, 2 matrix
        cores for dX and the gather kernel for dW (three flags, one of them set)."""
        off = dbp.format_layout(rows, cols)["scratch_offset"] + FLAG_OFFSET
        v = ws[off:off + 12].cpu().numpy().view(np.int32)
        return -1 if v[0] == -1 else 1 if v[0] == 1 else 2 if v[1] == 1 else 0

    def arm_flag(ws, rows, cols):
        off = dbp.format_layout(rows, cols)["scratch_offset"] + FLAG_OFFSET
        ws[off:off + 4] = 255                                            # reads back as -1 unless a gated call writes it

    PATH_NAME = {-1: "matrix cores (one family launched)", 0: "matrix cores (device gate)", 1: "gather (device gate)",
                 2: "matrix cores for dX, gather for dW (device gate)"}

    # ------------------------------------------------------------------ headline workload: config 5
    p5 = workloads.config5(args.sparsity)
    sets5, dims5, xd5 = conv_buffers(p5, sets=2)
    N, Cc, H, Wd, K, R, S = dims5
    P, Q = p5.delta.shape[2:]
    n_codes = p5.delta.size
    dense_flops5 = 2 * 2.0 * n_codes * Cc * R * S                        # dX and dW, dense-equivalent

    if args.probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)                                     # 1 GiB read + 1 GiB written: calibrates the counters
        torch.cuda.synchronize()
        if args.probe == "conv_dx":
            b = sets5[0]
            dbp.nsd_quantize(b["d"], N * K, P * Q, p5.step, p5.seed, 0, b["codes"], None, None, stream)
            for _ in range(20):
                dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, b["dX"], None,
                                    b["ws"], dbp.PATH_MFMA, stream)
            for _ in range(20):                                            # and the opt-in two-plane form of the same kernel
                dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, b["dX"], None,
                                    b["ws"], dbp.PATH_MFMA | dbp.PATH_TWO_PLANES, stream)
            what = "20 launches of conv_dx_weight_prep_kernel + conv_dx_kernel on config 5 (90 % zeros), three planes, then 20 with two planes"
        elif args.probe == "conv_dw":
            b = sets5[0]
            dbp.nsd_quantize(b["d"], N * K, P * Q, p5.step, p5.seed, 0, b["codes"], None, None, stream)
            for _ in range(20):
                dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, None, b["dW"],
                                    b["ws"], dbp.PATH_MFMA, stream)
            what = "20 launches of conv_dw_i8_kernel + conv_dw_reduce_kernel on config 5 (90 % zeros)"
        elif args.probe == "nsd":
            fmt = torch.empty(dbp.format_layout(1 << 16, 1 << 12)["total_bytes"], dtype=torch.uint8, device=dev)
            codes = torch.empty(1 << 28, dtype=torch.int8, device=dev)
            st = torch.zeros(32, dtype=torch.uint8, device=dev)
            src.normal_(0.0, 1e-3)
            for _ in range(20):
                dbp.nsd_quantize(src, 1 << 16, 1 << 12, 8e-3, 1, 0, codes, fmt, st, stream)
            what = "20 launches of nsd_kernel (codes + tile-sparse format + statistics) on 2^28 elements"
        else:
            pl = workloads.config2(8.0)[1]
            Bq, iq, oq = pl.dims
            dq, Wq, Xq = (torch.from_numpy(a).to(dev) for a in (pl.delta, pl.W, pl.X))
            cq = torch.empty((Bq, oq), dtype=torch.int8, device=dev)
            dXq = torch.empty((Bq, iq), dtype=torch.float32, device=dev)
            dWq = torch.empty((oq, iq), dtype=torch.float32, device=dev)
            wsq = torch.empty(dbp.linear_workspace_bytes(Bq, iq, oq), dtype=torch.uint8, device=dev)
            dbp.nsd_quantize(dq, Bq, oq, pl.step, pl.seed, 0, cq, None, None, stream)
            for _ in range(50):
                dbp.linear_products(cq, None, pl.step, Wq, Xq, dbp.F32, Bq, iq, oq, dXq, dWq, wsq, dbp.PATH_MFMA, stream)
            what = "50 launches of fc2_pair_kernel + fc2_reduce_kernel on the 256x4096x4096 layer (91 % zeros)"
        torch.cuda.synchronize()
        print(json.dumps({"probe": "torch.mul on 2^28 floats (1 GiB read, 1 GiB written), then " + what}))
        return

    for b in sets5:
        arm_flag(b["ws"], N * K, P * Q)

    def step5(i):
        conv_call(sets5[i % 2], dims5, xd5, p5, p5.step)

    for i in range(args.warmup):
        step5(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record()
    for i in range(args.steps):
        step5(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    per_step = [ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(args.steps)]
    t_step = max(statistics.median(per_step), 1e-9)
    t_mean = ev[0].elapsed_time(ev[args.steps]) * 1e-3 / args.steps
    st5 = dbp.Stats.from_tensor(sets5[0]["st"])
    nnz5 = st5.nnz
    value = dense_flops5 / t_step / 1e12
    path5 = PATH_NAME[gate_flag(sets5[0]["ws"], N * K, P * Q)]

    # ------------------------------------------------------------------ roofline of the dominant kernel: conv_dx_kernel
    b0 = sets5[0]

    def k_dx(i):
        b = sets5[i % 2]
        dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, b["dX"], None, b["ws"],
                            dbp.PATH_MFMA, stream)

    def k_dw(i):
        b = sets5[i % 2]
        dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, None, b["dW"], b["ws"],
                            dbp.PATH_MFMA, stream)

    def k_nsd(i):
        b = sets5[i % 2]
        dbp.nsd_quantize_static(b["d"], N * K, P * Q, p5.step, p5.seed, 0, b["codes"], b["st"], stream)   # codes + statistics, as in the step

    it = max(20, args.steps // 2)
    t_dx, t_dw, t_nsd5 = timed(k_dx, it), timed(k_dw, it), timed(k_nsd, it)
    alg_flops = 2.0 * nnz5 * Cc * R * S                                   # the method's work for dX: 2*nnz*C*R*S
    alg_bytes = float(n_codes + 4 * p5.W.size + 4 * p5.X.size)            # codes + W read, dX written (compulsory)
    exe_flops = 3 * 2.0 * n_codes * Cc * R * S                            # executed: dense product x 3 exact bf16 planes of W
    t_k = t_dx["mean"]
    t_flop_bound, t_byte_bound = alg_flops / (PEAK_F32_VECTOR_TFLOPS * 1e12), alg_bytes / (PEAK_HBM_GBS * 1e9)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "conv_dx_kernel_cfg5_pmc.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline = {
        "bound": "alu", "kernel": "conv_dx_kernel<7, bf16x3> (dX of config 5; the event-timed call includes its 3-5 us weight preparation launch)",
        "achieved": alg_flops / t_k / 1e12, "peak": PEAK_F32_VECTOR_TFLOPS, "unit": "TFLOP/s",
        "frac": alg_flops / t_k / 1e12 / PEAK_F32_VECTOR_TFLOPS, "traffic": traffic,
        "flops_counted": "the method's work, 2*nnz*C*R*S (Sec. 'Computational complexity'), against the fp32 vector peak",
        "us_per_launch": t_k * 1e6, "us_per_launch_median": t_dx["median"] * 1e6,
        "binding_bound": "alu" if t_flop_bound > t_byte_bound else "hbm",
        "hbm": {"bytes_compulsory": alg_bytes, "achieved_GBps": alg_bytes / t_k / 1e9, "frac_of_8TBps": alg_bytes / t_k / 1e9 / PEAK_HBM_GBS},
        "executed_mfma": {"flops": exe_flops, "achieved_TFLOPs": exe_flops / t_k / 1e12, "frac_of_2.5PFLOPs_bf16": exe_flops / t_k / 1e12 / PEAK_BF16_TFLOPS,
                          "note": "what the chosen algorithm executes: dense product x 3 bf16 planes; not the method's work"},
        "dense_equiv_tflops": 2.0 * n_codes * Cc * R * S / t_k / 1e12,
    }
    kernels5 = {"nsd_us": t_nsd5["median"] * 1e6, "dX_us": t_dx["median"] * 1e6, "dW_int8_us": t_dw["median"] * 1e6,
                "nsd_GBps": (5.0 * n_codes) / t_nsd5["median"] / 1e9}

    # the same step with the opt-in two-plane operand split (W in two bf16 planes, 16 significant bits): reported beside the headline
    t_step2 = med(lambda i: conv_call(sets5[i % 2], dims5, xd5, p5, p5.step, path=dbp.PATH_AUTO | dbp.PATH_TWO_PLANES), max(20, args.steps // 2))

    def k_dx2(i):
        b = sets5[i % 2]
        dbp.conv2d_products(b["codes"], None, p5.step, b["W"], b["X"], xd5, N, Cc, H, Wd, K, R, S, p5.stride, p5.pad, b["dX"], None, b["ws"],
                            dbp.PATH_MFMA | dbp.PATH_TWO_PLANES, stream)

    t_dx2 = timed(k_dx2, it)
    two_planes = {
        "ms_per_step": t_step2 * 1e3, "dense_equiv_tflops": dense_flops5 / t_step2 / 1e12, "dX_us": t_dx2["median"] * 1e6,
        "executed_mfma_frac_of_2.5PFLOPs_bf16": 2 * 2.0 * n_codes * Cc * R * S / t_dx2["mean"] / 1e12 / PEAK_BF16_TFLOPS,
        "note": "opt-in flag DBP_PATH_TWO_PLANES: fp32 W in two bf16 planes rounded to nearest (error <= 2^-16 * sum|q||w| per output, inside the "
                "1e-4 tolerance); NOT the headline, which multiplies the exact three-plane split",
    }

    graphs5 = [captured(lambda st_, b=b: conv_call(b, dims5, xd5, p5, p5.step, on=st_)) for b in sets5]
    t_graph5 = med(lambda i: graphs5[i % 2].replay(), max(20, args.steps // 2))

    out_line = {
        "metric": "dithered backward dense-equiv TFLOP/s (NSD + dX + dW, one call on config 5: VGG conv3-shaped layer, 8-bit mode)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "dX: bf16x3 MFMA (exact int8 codes x 3-plane split of fp32 W), fp32 accumulate; dW: int8 MFMA, exact int32",
        "data": "synthetic",
        "config": {"workload": "configs[4] (config 5): conv 3x3, N=32, 256->256, 56x56, int8 X, fp32 W, Delta for %g %% zeros" % (100 * args.sparsity),
                   "sparsity": 1 - nnz5 / n_codes, "path": "AUTO: " + path5},
        "roofline": roofline,
        "cpu_baseline": None,
        "ms_per_step_mean": t_mean * 1e3, "ms_per_step_min": min(per_step) * 1e3, "host_wall_ms_per_step": wall * 1e3,
        "kernels_cfg5_us": kernels5,
        "two_plane_operands": two_planes,
        "hip_graph_replay_ms_per_step": t_graph5 * 1e3,
    }

    if not args.headline_only:
        out_line["configs"] = bench_rows(dbp, workloads, torch, np, med, timed, captured, stream, conv_buffers, conv_call, gate_flag, arm_flag, PATH_NAME,
                                         sets5, dims5, xd5, p5)
        out_line["nsd_2^28"] = bench_nsd(dbp, torch, np, med, stream)

    # ------------------------------------------------------------------ CPU oracle baseline (bounded samples of the headline step)
    if not args.no_cpu:
        from oracle import oracle as O
        threads = O.max_threads()

        def oracle_step(n_img, thr):
            d, X = p5.delta[:n_img], p5.X[:n_img]
            t0 = time.perf_counter()
            k, _ = O.nsd(d, p5.step, p5.seed)
            O.conv2d_backward(p5.W, X.astype(np.float32), codes=k, step=p5.step, stride=1, pad=p5.pad, want_dw=False, threads=thr)
            O.conv2d_dw_i8(k, X, R, S, 1, p5.pad, threads=thr)
            return time.perf_counter() - t0

        t_all = oracle_step(N, threads)
        n1 = 8
        t_one = oracle_step(n1, 1)
        out_line["cpu_baseline"] = {
            "value": dense_flops5 / t_all / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "one whole step (all %d images: NSD + dX in fp64 + exact int32 dW, zero codes skipped) on %d threads: %.2f s" % (N, threads, t_all),
            "single_thread": {"value": dense_flops5 * n1 / N / t_one / 1e12, "unit": "TFLOP/s", "cores": 1,
                              "sample": "the first %d of %d images of the same step on one thread: %.2f s" % (n1, N, t_one)}}
    print(json.dumps(out_line))


def bench_nsd(dbp, torch, np, med, stream):
    """NSD pass on a 2^28-element tensor (1 GiB read): bandwidth against the 8 TB/s peak, 50 timed launches each."""
    dev = torch.device("cuda:0")
    n_big = 1 << 28
    rows_b, cols_b = 1 << 16, 1 << 12
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    big = torch.empty(n_big, dtype=torch.float32, device=dev)
    big.exponential_(1.0 / 1e-3, generator=g)                      # |Laplace(0, 1e-3)|
    sign = torch.empty(n_big, dtype=torch.float32, device=dev).uniform_(-1, 1, generator=g).sign_()
    big.mul_(sign)
    del sign
    step_big = float(np.float32(8 * 1e-3 * np.sqrt(2.0)))
    codes_big = torch.empty(n_big, dtype=torch.int8, device=dev)
    fmt_big = torch.empty(dbp.format_layout(rows_b, cols_b)["total_bytes"], dtype=torch.uint8, device=dev)
    st_big = torch.zeros(32, dtype=torch.uint8, device=dev)
    IT = 50
    t_nsd = med(lambda i: dbp.nsd_quantize(big, rows_b, cols_b, step_big, 1, 0, codes_big, fmt_big, st_big, stream), IT)
    nnz_big = dbp.Stats.from_tensor(st_big).nnz
    nsd_bytes = n_big * (4 + 1 + 0.125 + 2.0 / 256) + 2.0 * nnz_big
    nsd = {"elements": n_big, "iterations": IT, "sparsity": 1 - nnz_big / n_big, "ms": t_nsd * 1e3, "GBps": nsd_bytes / t_nsd / 1e9,
           "frac_of_8TBps": nsd_bytes / t_nsd / 1e9 / PEAK_HBM_GBS, "bytes_per_element": nsd_bytes / n_big,
           "what": "codes + tile-sparse format + statistics (median of %d launches)" % IT}
    t_static = med(lambda i: dbp.nsd_quantize_static(big, rows_b, cols_b, step_big, 1, 0, codes_big, st_big, stream), IT)
    nsd["codes_and_statistics_GBps"] = n_big * 5.0 / t_static / 1e9
    nsd["codes_and_statistics_frac_of_8TBps"] = n_big * 5.0 / t_static / 1e9 / PEAK_HBM_GBS
    t_codes = med(lambda i: dbp.nsd_quantize(big, rows_b, cols_b, step_big, 1, 0, codes_big, None, None, stream), IT)
    nsd["codes_only_GBps"] = n_big * 5.0 / t_codes / 1e9
    # Algorithm 1 on the device and the steps around the quantiser, same tensor: step size (one read of delta),
    # then the quantiser with the rectifier mask on load, the device step and the bias code sums
    pair = torch.zeros(2, dtype=torch.float32, device=dev)
    ws_std = torch.empty(dbp.step_size_workspace_bytes(n_big), dtype=torch.uint8, device=dev)
    t_std = med(lambda i: dbp.step_size(big, None, n_big, 8.0, pair, ws_std, stream), IT)
    act_big = torch.empty(n_big, dtype=torch.float32, device=dev).uniform_(-1, 1, generator=g)
    sums_big = torch.zeros(cols_b, dtype=torch.int64, device=dev)
    grad_big = torch.zeros(cols_b, dtype=torch.float32, device=dev)
    t_ex = med(lambda i: dbp.nsd_quantize_ex(big, rows_b, cols_b, step_big, 1, 0, codes_big, None, None, act=act_big,
                                             step_dev=pair, bias_sums=sums_big, bias_grad=grad_big,
                                             bias_mode=dbp.BIAS_PER_COLUMN, bias_len=cols_b, stream=stream), 20)
    nsd["step_size_ms"] = t_std * 1e3
    nsd["step_size_GBps"] = n_big * 4.0 / t_std / 1e9
    nsd["masked_bias_nsd_ms"] = t_ex * 1e3
    nsd["masked_bias_nsd_GBps"] = n_big * 9.0 / t_ex / 1e9            # delta + activation read, codes written
    return nsd


def bench_rows(dbp, workloads, torch, np, med, timed, captured, stream, conv_buffers, conv_call, gate_flag, arm_flag, PATH_NAME, sets5, dims5, xd5, p5):
    """Rows for every configuration besides the headline step: dithered vs the same library's dense backward, the sweeps
    over the sparsity, the gather kernels, structured gradients."""
    dev = torch.device("cuda:0")
    res = {}

    # ---- config 5: sparsity sweep on the headline layer (same tensors, Delta bisected per target)
    N, Cc, H, Wd, K, R, S = dims5
    P, Q = p5.delta.shape[2:]
    flops5 = 2 * 2.0 * p5.delta.size * Cc * R * S
    b = sets5[0]
    sweep = {}
    for target in (0.5, 0.75, 0.9, 0.95, 0.99, 0.999):
        step = workloads.step_for_sparsity(p5.delta, target)
        arm_flag(b["ws"], N * K, P * Q)
        t = med(lambda i: conv_call(b, dims5, xd5, p5, step), 12, warm=2)
        sp = 1 - dbp.Stats.from_tensor(b["st"]).nnz / p5.delta.size
        row = {"sparsity": sp, "ms_auto": t * 1e3, "dense_equiv_tflops": flops5 / t / 1e12, "path": PATH_NAME[gate_flag(b["ws"], N * K, P * Q)]}
        if target >= 0.99:
            row["ms_gather"] = med(lambda i: conv_call(b, dims5, xd5, p5, step, path=dbp.PATH_GATHER), 5, warm=1) * 1e3
            row["ms_matrix_cores"] = med(lambda i: conv_call(b, dims5, xd5, p5, step, path=dbp.PATH_MFMA), 5, warm=1) * 1e3
        sweep["%g" % target] = row
    res["cfg5_sparsity_sweep"] = sweep
    # full 8-bit backward on the same layer: int8 weights too, both products exact int32
    W8 = torch.randint(-127, 128, p5.W.shape, dtype=torch.int8, device=dev)
    dX32 = torch.empty(p5.X.shape, dtype=torch.int32, device=dev)
    t8 = med(lambda i: dbp.dithered_conv2d_backward_q8(b["d"], W8, b["X"], N, Cc, H, Wd, K, R, S, 1, p5.pad, p5.step, p5.seed, 0, b["codes"],
                                                        dX32, b["dW"], b["ws"], b["st"], stream), 10, warm=2)
    res["cfg5_full_8bit"] = {"ms": t8 * 1e3, "dense_equiv_tops": flops5 / t8 / 1e12}
    del W8, dX32
    # structured gradient: half of the (n, k) planes dead (what ReLU networks without batch normalisation show)
    d_keep = b["d"].clone()
    b["d"].copy_(torch.from_numpy(workloads.structured_planes(p5.delta, 0.5)).to(dev))
    t = med(lambda i: conv_call(b, dims5, xd5, p5, p5.step), 10, warm=2)
    res["cfg5_structured_half_dead_planes"] = {"ms_auto": t * 1e3, "sparsity": 1 - dbp.Stats.from_tensor(b["st"]).nnz / p5.delta.size}
    b["d"].copy_(d_keep)
    del d_keep

    # ---- configs 3, 4a, 4b and the strided ResNet layer
    problems = [("cfg3", workloads.config3()), ("cfg3_c8", workloads.config3(8.0)), ("cfg4a", workloads.config4a()), ("cfg4b", workloads.config4b()),
                ("resnet_3x3_stride2", workloads.resnet_downsample())]
    for name, p in problems:
        bufs, dims, xd = conv_buffers(p)
        bb = bufs[0]
        Nn, Cq, Hq, Wq, Kq, Rq, Sq = dims
        Pq, Qq = p.delta.shape[2:]
        arm_flag(bb["ws"], Nn * Kq, Pq * Qq)
        t = med(lambda i: conv_call(bb, dims, xd, p, p.step), 20)
        flops = 2 * 2.0 * p.delta.size * Cq * Rq * Sq
        nnz = dbp.Stats.from_tensor(bb["st"]).nnz
        row = {"ms": t * 1e3, "dense_equiv_tflops": flops / t / 1e12, "sparsity": 1 - nnz / p.delta.size,
               "path": PATH_NAME[gate_flag(bb["ws"], Nn * Kq, Pq * Qq)]}
        t_x = med(lambda i: dbp.conv2d_products(bb["codes"], None, p.step, bb["W"], bb["X"], xd, Nn, Cq, Hq, Wq, Kq, Rq, Sq, p.stride, p.pad,
                                                bb["dX"], None, bb["ws"], dbp.PATH_MFMA, stream), 20)
        t_w = med(lambda i: dbp.conv2d_products(bb["codes"], None, p.step, bb["W"], bb["X"], xd, Nn, Cq, Hq, Wq, Kq, Rq, Sq, p.stride, p.pad,
                                                None, bb["dW"], bb["ws"], dbp.PATH_MFMA, stream), 20)
        row["dX_us"], row["dW_us"], row["nsd_us"] = t_x * 1e6, t_w * 1e6, max(t - t_x - t_w, 0.0) * 1e6
        row["ms_two_planes"] = med(lambda i: conv_call(bb, dims, xd, p, p.step, path=dbp.PATH_AUTO | dbp.PATH_TWO_PLANES), 20) * 1e3
        t_d = med(lambda i: dbp.dense_conv2d_backward(bb["d"], bb["W"], bb["X"], xd, Nn, Cq, Hq, Wq, Kq, Rq, Sq, p.stride, p.pad, bb["dX"], bb["dW"],
                                                      bb["ws"], stream), 5, warm=1)
        row["same_library_dense_ms"] = t_d * 1e3
        torch.backends.cudnn.allow_tf32 = False
        f = lambda i: torch.ops.aten.convolution_backward(bb["d"], bb["X"], bb["W"], None, [p.stride, p.stride], [p.pad, p.pad], [1, 1], False,
                                                          [0, 0], 1, [True, True, False])
        try:                                                         # context line: never fail the run over it
            row["torch_conv_backward_fp32_ms"] = med(f, 5, warm=2) * 1e3
        except Exception:
            row["torch_conv_backward_fp32_ms"] = None
        if name == "cfg3":
            keep = bb["d"].clone()
            bb["d"].copy_(torch.from_numpy(workloads.structured_planes(p.delta, 0.5)).to(dev))
            ts = med(lambda i: conv_call(bb, dims, xd, p, p.step), 20)
            row["structured_half_dead_planes"] = {"ms": ts * 1e3, "sparsity": 1 - dbp.Stats.from_tensor(bb["st"]).nnz / p.delta.size}
            bb["d"].copy_(keep)
        if name == "cfg4a":
            # the gather kernels on the same layer, at the configuration's step and at steps that leave 1 % and 0.1 % nonzeros
            row["gather"] = {}
            for target in (None, 0.97, 0.99, 0.999):
                step = p.step if target is None else workloads.step_for_sparsity(p.delta, target)
                tg = med(lambda i: conv_call(bb, dims, xd, p, step, path=dbp.PATH_GATHER), 5, warm=1)
                nz = dbp.Stats.from_tensor(bb["st"]).nnz
                tm = med(lambda i: conv_call(bb, dims, xd, p, step, path=dbp.PATH_MFMA), 5, warm=1)
                arm_flag(bb["ws"], Nn * Kq, Pq * Qq)
                ta = med(lambda i: conv_call(bb, dims, xd, p, step), 5, warm=1)
                auto_path = PATH_NAME[gate_flag(bb["ws"], Nn * Kq, Pq * Qq)]
                # the two gather kernels alone (codes and format of the call above): the method's work per product, 2*nnz*C*R*S
                L4 = dbp.format_layout(Nn * Kq, Pq * Qq)
                fmt4 = torch.empty(L4["total_bytes"], dtype=torch.uint8, device=dev)
                dbp.nsd_quantize(bb["d"], Nn * Kq, Pq * Qq, step, p.seed, 0, bb["codes"], fmt4, None, stream)
                per = {}
                for which, a_dx, a_dw in (("dX", bb["dX"], None), ("dW", None, bb["dW"])):
                    for fam, path in (("gather", dbp.PATH_GATHER), ("matrix_core", dbp.PATH_MFMA)):
                        per[fam + "_" + which + "_us"] = med(lambda i: dbp.conv2d_products(
                            bb["codes"], fmt4, step, bb["W"], bb["X"], xd, Nn, Cq, Hq, Wq, Kq, Rq, Sq, p.stride, p.pad, a_dx, a_dw, bb["ws"], path, stream), 10, warm=2) * 1e6
                    per["gather_" + which + "_algorithmic_tflops"] = 2.0 * nz * Cq * Rq * Sq / per["gather_" + which + "_us"] / 1e6
                del fmt4
                row["gather"]["sparsity_%.4f" % (1 - nz / p.delta.size)] = {
                    "gather_ms": tg * 1e3, "matrix_core_ms": tm * 1e3, "auto_ms": ta * 1e3, "auto_path": auto_path,
                    "gather_algorithmic_tflops": 2 * 2.0 * nz * Cq * Rq * Sq / tg / 1e12,
                    "gather_frac_of_fp32_vector_peak": 2 * 2.0 * nz * Cq * Rq * Sq / tg / 1e12 / PEAK_F32_VECTOR_TFLOPS,
                    "kernels": per}
        res[name] = row
        del bufs, bb

    # ---- config 1 (launch bound: microseconds) and the MLP chain of configs[1]
    def linear_buffers(p, perm=None):
        B, in_, out = p.dims
        d = p.delta if perm is None else p.delta[perm]
        X = p.X if perm is None else p.X[perm]
        return dict(p=p, d=torch.from_numpy(d).to(dev), W=torch.from_numpy(p.W).to(dev).clone(), X=torch.from_numpy(X).to(dev),
                    codes=torch.empty((B, out), dtype=torch.int8, device=dev), dX=torch.empty((B, in_), dtype=torch.float32, device=dev),
                    dW=torch.empty((out, in_), dtype=torch.float32, device=dev),
                    ws=torch.zeros(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device=dev), st=torch.zeros(32, dtype=torch.uint8, device=dev))

    def linear_call(b, step=None, path=dbp.PATH_AUTO, dX=True, dW=True, on=None):
        p = b["p"]
        B, in_, out = p.dims
        dbp.dithered_linear_backward(b["d"], b["W"], b["X"], dbp.F32, B, in_, out, p.step if step is None else step, p.seed, 0, b["codes"],
                                     b["dX"] if dX else None, b["dW"] if dW else None, b["ws"], b["st"], path, stream if on is None else on)

    b1 = linear_buffers(workloads.config1())
    t1 = med(lambda i: linear_call(b1), 50)
    g1 = captured(lambda st_: linear_call(b1, on=st_))
    res["cfg1"] = {"us": t1 * 1e6, "us_hip_graph_replay": med(lambda i: g1.replay(), 50) * 1e6,
                   "sparsity": 1 - dbp.Stats.from_tensor(b1["st"]).nnz / b1["d"].numel(), "note": "launch bound: 3 launches"}
    del g1

    NSETS = 3
    mlp = {}
    for c in (2.0, 4.0, 8.0, 16.0, 32.0, 64.0):
        layers = workloads.config2(c)
        sets = []
        for s in range(NSETS):
            perm = np.random.default_rng(4242 + s).permutation(layers[0].dims[0]) if s else None
            sets.append([linear_buffers(p, perm) for p in layers])
        dense_flops = sum(2 * 2 * p.dims[0] * p.dims[1] * p.dims[2] for p in layers)
        row = {}
        for pname, path in (("auto", dbp.PATH_AUTO), ("gather", dbp.PATH_GATHER)):
            def step(i):
                for bq in sets[i % NSETS]:
                    linear_call(bq, path=path)
            t = med(step, 60 if pname == "auto" else 20, warm=5)
            row["ms_" + pname] = t * 1e3
        def step2(i):
            for bq in sets[i % NSETS]:
                linear_call(bq, path=dbp.PATH_AUTO | dbp.PATH_TWO_PLANES)
        row["ms_auto_two_planes"] = med(step2, 60, warm=5) * 1e3
        if c == 8.0:
            def chain(st_, k):
                for bq in sets[k]:
                    linear_call(bq, on=st_)
            gs = [captured(lambda st_, k=k: chain(st_, k)) for k in range(NSETS)]
            row["ms_auto_hip_graph_replay"] = med(lambda i: gs[i % NSETS].replay(), 60, warm=5) * 1e3
            del gs
        row["sparsity_per_layer"] = [round(1 - dbp.Stats.from_tensor(bq["st"]).nnz / bq["d"].numel(), 4) for bq in sets[0]]
        row["dense_equiv_tflops_auto"] = dense_flops / (row["ms_auto"] * 1e-3) / 1e12
        # the gather kernels alone on the 4096x4096 layer: the method's own work, 2*nnz*in per product, against the fp32 vector peak
        g2 = [s_[1] for s_ in sets]
        Bg, ig, og = g2[0]["p"].dims
        for bq in g2:
            dbp.nsd_quantize(bq["d"], Bg, og, bq["p"].step, bq["p"].seed, 0, bq["codes"], None, bq["st"], stream)
        alg_g = 2.0 * dbp.Stats.from_tensor(g2[0]["st"]).nnz * ig
        # (the format argument is only read by the gather kernels that serve odd shapes: a buffer of the right size stands in)
        fmt_g = torch.empty(dbp.format_layout(Bg, og)["total_bytes"], dtype=torch.uint8, device=dev)
        gk = {}
        for nm, wdx, wdw in (("dX", True, False), ("dW", False, True)):
            def gf(i, wdx=wdx, wdw=wdw):
                bq = g2[i % NSETS]
                dbp.linear_products(bq["codes"], fmt_g, bq["p"].step, bq["W"], bq["X"], dbp.F32, Bg, ig, og, bq["dX"] if wdx else None,
                                    bq["dW"] if wdw else None, bq["ws"], dbp.PATH_GATHER, stream)
            tg = med(gf, 20)
            gk[nm + "_us"] = tg * 1e6
            gk[nm + "_algorithmic_tflops"] = alg_g / tg / 1e12
            gk[nm + "_frac_of_fp32_vector_peak"] = alg_g / tg / 1e12 / PEAK_F32_VECTOR_TFLOPS
        row["gather_kernels_4096x4096_layer"] = gk
        if c == 8.0:
            def dense_step(i):
                for bq in sets[i % NSETS]:
                    Bq, iq, oq = bq["p"].dims
                    dbp.dense_linear_backward(bq["d"], bq["W"], bq["X"], dbp.F32, Bq, iq, oq, bq["dX"], bq["dW"], bq["ws"], stream)

            def torch_step(i):
                for bq in sets[i % NSETS]:
                    torch.matmul(bq["d"], bq["W"], out=bq["dX"])
                    torch.matmul(bq["d"].t(), bq["X"], out=bq["dW"])

            torch.backends.cuda.matmul.allow_tf32 = False
            row["same_library_dense_fp32_mfma_ms"] = med(dense_step, 10) * 1e3
            row["torch_matmul_fp32_ms"] = med(torch_step, 10) * 1e3
            # per-kernel times on the 4096x4096 layer and the gather kernels' share of the fp32 vector peak
            b2 = [s[1] for s in sets]
            p2 = b2[0]["p"]
            B, in_, out = p2.dims
            for bq in b2:
                dbp.nsd_quantize(bq["d"], B, out, p2.step, p2.seed, 0, bq["codes"], None, bq["st"], stream)
            nnz2 = dbp.Stats.from_tensor(b2[0]["st"]).nnz

            # (the format argument of linear_products is only read by the gather kernels that serve odd shapes; the workspace stands in)
            ws2 = [torch.empty(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device=dev) for _ in b2]

            def prod2(path, dX, dW):
                def f(i):
                    bq = b2[i % NSETS]
                    dbp.linear_products(bq["codes"], ws2[i % NSETS], p2.step, bq["W"], bq["X"], dbp.F32, B, in_, out, bq["dX"] if dX else None,
                                        bq["dW"] if dW else None, bq["ws"], path, stream)
                return f
            k = {"nsd_1M_elements": med(lambda i: dbp.nsd_quantize(b2[i % NSETS]["d"], B, out, p2.step, p2.seed, 0, b2[i % NSETS]["codes"], None,
                                                                  b2[i % NSETS]["st"], stream), 40) * 1e6}
            for nm, path in (("mfma", dbp.PATH_MFMA), ("gather", dbp.PATH_GATHER)):
                k["dX_" + nm] = med(prod2(path, True, False), 40) * 1e6
                k["dW_" + nm] = med(prod2(path, False, True), 40) * 1e6
                k["dX_and_dW_" + nm] = med(prod2(path, True, True), 40) * 1e6
            alg = 2.0 * nnz2 * in_
            k["gather_dX_algorithmic_tflops"] = alg / k["dX_gather"] / 1e6
            k["gather_dW_algorithmic_tflops"] = alg / k["dW_gather"] / 1e6
            k["gather_dX_frac_of_fp32_vector_peak"] = alg / k["dX_gather"] / 1e6 / PEAK_F32_VECTOR_TFLOPS
            k["gather_dW_frac_of_fp32_vector_peak"] = alg / k["dW_gather"] / 1e6 / PEAK_F32_VECTOR_TFLOPS
            mnk = 2.0 * B * in_ * out
            k["pair_executed_bf16x3_tflops"] = 2 * 3 * mnk / k["dX_and_dW_mfma"] / 1e6
            k["pair_hbm_bytes_compulsory"] = 4.0 * (out * in_ + B * in_) + B * out + 4.0 * (B * in_ + out * in_)
            k["pair_hbm_frac_of_8TBps"] = k["pair_hbm_bytes_compulsory"] / (k["dX_and_dW_mfma"] * 1e-6) / 1e9 / PEAK_HBM_GBS
            row["kernels_4096x4096_layer_us"] = k
            # the same chain through the whole-layer entry point (Algorithm 1 on the device: + std, + mask, + bias gradient)
            lsets = []
            for bufs in sets:
                lrow = []
                for bq in bufs:
                    Bz, iz, oz = bq["p"].dims
                    lrow.append(dict(ws=torch.empty(dbp.linear_layer_workspace_bytes(Bz, iz, oz), dtype=torch.uint8, device=dev),
                                     act=torch.empty((Bz, oz), dtype=torch.float32, device=dev).uniform_(-0.2, 1.0),
                                     db=torch.empty(oz, dtype=torch.float32, device=dev), pair=torch.zeros(2, dtype=torch.float32, device=dev)))
                lsets.append(lrow)

            def layer_step(i):
                for bq, l in zip(sets[i % NSETS], lsets[i % NSETS]):
                    Bz, iz, oz = bq["p"].dims
                    dbp.dithered_linear_layer_backward(bq["d"], l["act"], bq["W"], bq["X"], dbp.F32, Bz, iz, oz, c, bq["p"].seed, 0, bq["codes"],
                                                       bq["dX"], bq["dW"], l["db"], l["pair"], l["ws"], bq["st"], dbp.PATH_AUTO, stream)
            row["whole_layer_entry_ms"] = med(layer_step, 30) * 1e3
            del lsets
            # the same chain in the full 8-bit mode: int8 weights and activations, exact int32 dX and dW
            q8 = []
            for bq in sets[0]:
                Bz, iz, oz = bq["p"].dims
                q8.append(dict(W8=torch.randint(-127, 128, (oz, iz), dtype=torch.int8, device=dev),
                               X8=torch.randint(0, 128, (Bz, iz), dtype=torch.int8, device=dev),
                               dX=torch.empty((Bz, iz), dtype=torch.int32, device=dev), dW=torch.empty((oz, iz), dtype=torch.int32, device=dev)))

            def q8_step(i):
                for bq, q in zip(sets[0], q8):
                    Bz, iz, oz = bq["p"].dims
                    dbp.dithered_linear_backward_q8(bq["d"], q["W8"], q["X8"], Bz, iz, oz, bq["p"].step, bq["p"].seed, 0, bq["codes"], q["dX"],
                                                    q["dW"], bq["ws"], bq["st"], stream)
            row["full_8bit_ms"] = med(q8_step, 30) * 1e3
            del q8
        mlp["c=%g" % c] = row
        del sets
    res["cfg2_mlp_chain"] = mlp

    # ---- a fully connected layer wide enough for the density gate (256 x 4096 x 16384): time against sparsity
    rng = np.random.default_rng(5)
    Bq, iq, oq = 256, 4096, 16384
    X = np.maximum(rng.standard_normal((Bq, iq)), 0).astype(np.float32)
    W = (rng.standard_normal((oq, iq)) / np.sqrt(iq)).astype(np.float32)
    dl = rng.laplace(0, 1e-3, size=(Bq, oq)).astype(np.float32)
    pl = workloads.LinearProblem("fc_wide", dl, W, X, 1.0)
    bl = linear_buffers(pl)
    gated = {}
    for c in (8.0, 32.0, 64.0, 128.0, 512.0):
        step = workloads.step_from_std(dl, c)
        arm_flag(bl["ws"], Bq, oq)
        t = med(lambda i: linear_call(bl, step=step), 20)
        flag = gate_flag(bl["ws"], Bq, oq)
        gated["c=%g" % c] = {"sparsity": 1 - dbp.Stats.from_tensor(bl["st"]).nnz / dl.size, "ms_auto": t * 1e3, "path": PATH_NAME[flag],
                             "ms_matrix_cores": med(lambda i: linear_call(bl, step=step, path=dbp.PATH_MFMA), 10) * 1e3,
                             "ms_gather": med(lambda i: linear_call(bl, step=step, path=dbp.PATH_GATHER), 10) * 1e3}
    res["fc_256x4096x16384_density_gate"] = gated
    del bl

    # ---- top-k sparsifier against the dithered quantiser on identical kernels (Sec. "Comparison to meProp"): the 256 x 4096 x 4096
    # layer, k chosen so that both leave the same share of nonzeros (Delta = 8 std: 8.8 %)
    p2 = workloads.config2(8.0)[1]
    Bq, iq, oq = p2.dims
    dq, Wq, Xq = (torch.from_numpy(a).to(dev) for a in (p2.delta, p2.W, p2.X))
    cq = torch.empty((Bq, oq), dtype=torch.int8, device=dev)
    fq = torch.empty(dbp.format_layout(Bq, oq)["total_bytes"], dtype=torch.uint8, device=dev)
    sq = torch.zeros(32, dtype=torch.uint8, device=dev)
    tq = torch.empty(dbp.topk_workspace_bytes(Bq, 1), dtype=torch.uint8, device=dev)
    dXq = torch.empty((Bq, iq), dtype=torch.float32, device=dev)
    dWq = torch.empty((oq, iq), dtype=torch.float32, device=dev)
    wsq = torch.empty(dbp.linear_workspace_bytes(Bq, iq, oq), dtype=torch.uint8, device=dev)
    ab = {}
    t_nsd = med(lambda i: dbp.nsd_quantize(dq, Bq, oq, p2.step, p2.seed, 0, cq, fq, sq, stream), 30)
    nnz = dbp.Stats.from_tensor(sq).nnz
    k_top = max(1, round(nnz / Bq))
    step_top = float(np.abs(p2.delta).max() / 127)
    for name, quant in (("dithered", lambda i: dbp.nsd_quantize(dq, Bq, oq, p2.step, p2.seed, 0, cq, fq, sq, stream)),
                        ("top_k", lambda i: dbp.topk_quantize(dq, Bq, oq, 1, k_top, step_top, cq, tq, fq, sq, stream))):
        tq_ms = med(quant, 30) * 1e3
        st_now = dbp.Stats.from_tensor(sq)
        step_now = p2.step if name == "dithered" else step_top
        ab[name] = {"quantiser_us": tq_ms * 1e3, "sparsity": 1 - st_now.nnz / p2.delta.size, "max_abs_code": st_now.max_abs_code,
                    "products_matrix_cores_us": med(lambda i: dbp.linear_products(cq, fq, step_now, Wq, Xq, dbp.F32, Bq, iq, oq, dXq, dWq, wsq,
                                                                                  dbp.PATH_MFMA, stream), 30) * 1e6,
                    "products_gather_us": med(lambda i: dbp.linear_products(cq, fq, step_now, Wq, Xq, dbp.F32, Bq, iq, oq, dXq, dWq, wsq,
                                                                            dbp.PATH_GATHER, stream), 30) * 1e6}
    ab["k_per_example"] = k_top
    ab["note"] = ("same kernels after the quantiser; top-k keeps k per example (Delta = max|delta|/127: survivors below Delta/2 round to 0), "
                  "the dithered quantiser the same share in expectation")
    res["fc_256x4096x4096_topk_vs_dithered"] = ab
    del dq, Wq, Xq, cq, fq, dXq, dWq, wsq

    # ---- grouped convolution: N=64, 256 -> 256, 28 x 28, 3 x 3 (a ResNeXt-like block), Delta = 8 std, against the group count
    rng = np.random.default_rng(6)
    Ng, Cg_, Hg, Kg_ = 64, 256, 28, 256
    dg = rng.laplace(0, 5e-4, size=(Ng, Kg_, Hg, Hg)).astype(np.float32)
    step_g = workloads.step_from_std(dg, 8.0)
    Xg = torch.from_numpy(np.maximum(rng.standard_normal((Ng, Cg_, Hg, Hg)), 0).astype(np.float32)).to(dev)
    dgd = torch.from_numpy(dg).to(dev)
    cg = torch.empty(dg.shape, dtype=torch.int8, device=dev)
    dXg = torch.empty_like(Xg)
    grouped = {}
    for groups in (1, 2, 4, 32):
        Wg = torch.from_numpy((rng.standard_normal((Kg_, Cg_ // groups, 3, 3)) * 0.05).astype(np.float32)).to(dev)
        dWg = torch.empty_like(Wg)
        wsg = torch.empty(dbp.conv2d_grouped_workspace_bytes(Ng, Cg_, Hg, Hg, Kg_, 3, 3, 1, 1, groups), dtype=torch.uint8, device=dev)
        t = med(lambda i: dbp.dithered_conv2d_backward_grouped(dgd, Wg, Xg, dbp.F32, Ng, Cg_, Hg, Hg, Kg_, 3, 3, 1, 1, groups, step_g, 1, 0, cg, dXg,
                                                               dWg, wsg, None, dbp.PATH_MFMA, stream), 20)
        flops = 2 * 2.0 * dg.size * (Cg_ // groups) * 9
        grouped["groups=%d" % groups] = {"ms": t * 1e3, "dense_equiv_tflops": flops / t / 1e12}
    res["grouped_conv_n64_256to256_28x28_3x3"] = grouped
    return res


if __name__ == "__main__":
    main()
