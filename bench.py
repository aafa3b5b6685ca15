#!/usr/bin/env python3
"""Benchmark of the dithered-backprop hot path on one MI355X.

One "step" = the whole hot path on the benchmark's configs[1]: the three-layer MLP backward chain
(batch 256, 1024->4096->4096->1000, Delta = 8*std -> ~91% zero codes), i.e. per layer one NSD pass
(Eq. (qdz)) and the two products dX = q.W, dW = q^T.X (Eqs. (qda),(qdw)), through the C ABI entry point
dithered_linear_backward.  Inputs are synthetic (workloads.py), resident in HBM before the timed
region, and three buffer sets are rotated so that the 256 MB Infinity Cache cannot stand in for HBM.

Prints ONE JSON line: whole-job dense-equivalent TFLOP/s, plus `roofline` for the dominant kernel
(timed alone with events on the launch stream), `cpu_baseline` (the CPU oracle on the host cores) and
context numbers (NSD bandwidth on a 2^28-element tensor, the library's own dense fp32 backward and
torch's dense matmul on the same shapes).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_I8_TOPS = 5000.0
PEAK_F32_MFMA_TFLOPS = 157.3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--c", type=float, default=8.0, help="step-size multiple: Delta = c*std(delta)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--all", action="store_true", help="also time the conv / 8-bit configs (slower)")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe: one 1 GiB device copy of known size, then only the dominant kernel "
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
        for _ in range(warm):
            fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e-3          # seconds per call

    # ------------------------------------------------------------------ workload: configs[1]
    layers = workloads.config2(args.c)
    NSETS = 3
    sets = []
    for s in range(NSETS):
        bufs = []
        for p in layers:
            B, in_, out = p.dims
            rng = np.random.default_rng(4242 + s)
            perm = rng.permutation(B) if s else np.arange(B)       # same law, different bytes per set
            d = torch.from_numpy(p.delta[perm]).to(dev)
            W = torch.from_numpy(p.W).to(dev).clone()
            X = torch.from_numpy(p.X[perm]).to(dev)
            bufs.append(dict(p=p, d=d, W=W, X=X,
                             codes=torch.empty((B, out), dtype=torch.int8, device=dev),
                             dX=torch.empty((B, in_), dtype=torch.float32, device=dev),
                             dW=torch.empty((out, in_), dtype=torch.float32, device=dev),
                             ws=torch.empty(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device=dev),
                             stats=torch.zeros(32, dtype=torch.uint8, device=dev)))
        sets.append(bufs)

    if args.probe:
        # counter probe: an elementwise kernel of known traffic (1 GiB read + 1 GiB written), then the dominant kernel
        b = sets[0][1]
        p2 = b["p"]
        B, in_, out = p2.dims
        fmt = torch.empty(dbp.format_layout(B, out)["total_bytes"], dtype=torch.uint8, device=dev)
        dbp.nsd_quantize(b["d"], B, out, p2.step, p2.seed, 0, b["codes"], fmt, None, stream)
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        for i in range(50):
            dbp.linear_products(b["codes"], fmt, p2.step, b["W"], b["X"], dbp.F32, B, in_, out, b["dX"], b["dW"], b["ws"],
                                dbp.PATH_MFMA, stream)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "torch.mul on 2^28 floats (1 GiB read, 1 GiB written) + 50 launches of fc2_pair_kernel "
                                   "and fc2_reduce_kernel on the 256x4096x4096 layer"}))
        return

    def step(i, path=dbp.PATH_AUTO):
        for b in sets[i % NSETS]:
            p = b["p"]
            B, in_, out = p.dims
            dbp.dithered_linear_backward(b["d"], b["W"], b["X"], dbp.F32, B, in_, out, p.step, p.seed, 0,
                                         b["codes"], b["dX"], b["dW"], b["ws"], b["stats"], path, stream)

    dense_flops = sum(2 * 2 * p.dims[0] * p.dims[1] * p.dims[2] for p in layers)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    t_step = max(e0.elapsed_time(e1) * 1e-3 / args.steps, 0.0)
    t_step = max(t_step, 1e-9)
    sparsity = []
    nnz_total = 0
    for b in sets[0]:
        st = dbp.Stats.from_tensor(b["stats"])
        sparsity.append(1 - st.nnz / b["d"].numel())
        nnz_total += st.nnz
    value = dense_flops / t_step / 1e12

    # ------------------------------------------------------------------ per-kernel timings (L2 layer)
    b2 = [s[1] for s in sets]                      # the 4096x4096 layer of each set
    p2 = b2[0]["p"]
    B, in_, out = p2.dims
    fmts = [torch.empty(dbp.format_layout(B, out)["total_bytes"], dtype=torch.uint8, device=dev) for _ in b2]
    for b, f in zip(b2, fmts):
        dbp.nsd_quantize(b["d"], B, out, p2.step, p2.seed, 0, b["codes"], f, b["stats"], stream)

    def k_dx(i, path=dbp.PATH_MFMA):
        b = b2[i % NSETS]
        dbp.linear_products(b["codes"], fmts[i % NSETS], p2.step, b["W"], b["X"], dbp.F32, B, in_, out, b["dX"], None, b["ws"], path, stream)

    def k_dw(i, path=dbp.PATH_MFMA):
        b = b2[i % NSETS]
        dbp.linear_products(b["codes"], fmts[i % NSETS], p2.step, b["W"], b["X"], dbp.F32, B, in_, out, None, b["dW"], b["ws"], path, stream)

    def k_both(i, path=dbp.PATH_MFMA):
        b = b2[i % NSETS]
        dbp.linear_products(b["codes"], fmts[i % NSETS], p2.step, b["W"], b["X"], dbp.F32, B, in_, out, b["dX"], b["dW"], b["ws"], path, stream)

    def k_nsd(i):
        b = b2[i % NSETS]
        dbp.nsd_quantize(b["d"], B, out, p2.step, p2.seed, 0, b["codes"], fmts[i % NSETS], b["stats"], stream)

    iters = max(20, args.steps)
    t_dx, t_dw, t_both, t_nsd_small = timed(k_dx, iters), timed(k_dw, iters), timed(k_both, iters), timed(k_nsd, iters)
    t_dx_g = timed(lambda i: k_dx(i, dbp.PATH_GATHER), max(5, iters // 4))
    t_dw_g = timed(lambda i: k_dw(i, dbp.PATH_GATHER), max(5, iters // 4))
    mnk = 2.0 * B * in_ * out
    # Dominant kernel: fc2_pair_kernel, both products of the 4096x4096 layer in one launch (its split-K
    # reduction launch is included in the time).  Algorithmic work per launch:
    # flops = 2 products x 3 exact bf16 planes x 2*B*in*out; HBM bytes = W + X + codes read, dX + dW written.
    alg_flops = 2 * 3 * mnk
    alg_bytes = 4.0 * (out * in_ + B * in_) + B * out + 4.0 * (B * in_ + out * in_)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "fc2_pair_kernel_cfg2_L2_pmc.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline = {"bound": "mfma", "kernel": "fc2_pair_kernel (dX and dW of the 256x4096x4096 layer, one launch) + fc2_reduce_kernel",
                "achieved": alg_flops / t_both / 1e12, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": alg_flops / t_both / 1e12 / PEAK_BF16_TFLOPS, "traffic": traffic,
                "flops_counted": "2 products x 3 bf16 planes x 2*M*N*K per launch", "us_per_launch": t_both * 1e6,
                "dense_equiv_tflops": 2 * mnk / t_both / 1e12,
                "hbm_bytes_algorithmic": alg_bytes,
                "hbm_frac_of_8TBps": alg_bytes / t_both / 1e9 / PEAK_HBM_GBS}

    # ------------------------------------------------------------------ dense baselines on the same shapes
    def dense_step(i):
        for b in sets[i % NSETS]:
            p = b["p"]
            Bq, iq, oq = p.dims
            dbp.dense_linear_backward(b["d"], b["W"], b["X"], dbp.F32, Bq, iq, oq, b["dX"], b["dW"], b["ws"], stream)

    def torch_step(i):
        for b in sets[i % NSETS]:
            torch.matmul(b["d"], b["W"], out=b["dX"])
            torch.matmul(b["d"].t(), b["X"], out=b["dW"])

    # the same chain through the whole-layer entry point (Algorithm 1 on the device: + std, + mask, + bias gradient)
    lsets = []
    for bufs in sets:
        row = []
        for b in bufs:
            Bq, iq, oq = b["p"].dims
            row.append(dict(ws=torch.empty(dbp.linear_layer_workspace_bytes(Bq, iq, oq), dtype=torch.uint8, device=dev),
                            act=torch.empty((Bq, oq), dtype=torch.float32, device=dev).uniform_(-0.2, 1.0),
                            db=torch.empty(oq, dtype=torch.float32, device=dev), pair=torch.zeros(2, dtype=torch.float32, device=dev)))
        lsets.append(row)

    def layer_step(i):
        for b, l in zip(sets[i % NSETS], lsets[i % NSETS]):
            p = b["p"]
            Bq, iq, oq = p.dims
            dbp.dithered_linear_layer_backward(b["d"], l["act"], b["W"], b["X"], dbp.F32, Bq, iq, oq, args.c, p.seed, 0,
                                               b["codes"], b["dX"], b["dW"], l["db"], l["pair"], l["ws"], b["stats"],
                                               dbp.PATH_AUTO, stream)

    t_layer = timed(layer_step, max(10, args.steps // 2))

    # the same chain in the full 8-bit mode: int8 weights and activations, exact int32 dX and dW
    q8 = []
    for b in sets[0]:
        Bq, iq, oq = b["p"].dims
        q8.append(dict(W8=torch.randint(-127, 128, (oq, iq), dtype=torch.int8, device=dev),
                       X8=torch.randint(0, 128, (Bq, iq), dtype=torch.int8, device=dev),
                       dX=torch.empty((Bq, iq), dtype=torch.int32, device=dev), dW=torch.empty((oq, iq), dtype=torch.int32, device=dev)))

    def q8_step(i):
        for b, q in zip(sets[0], q8):
            p = b["p"]
            Bq, iq, oq = p.dims
            dbp.dithered_linear_backward_q8(b["d"], q["W8"], q["X8"], Bq, iq, oq, p.step, p.seed, 0, b["codes"], q["dX"], q["dW"],
                                            b["ws"], b["stats"], stream)

    t_q8 = timed(q8_step, max(10, args.steps // 2))
    del q8
    del lsets
    t_dense = timed(dense_step, max(5, args.steps // 4))
    torch.backends.cuda.matmul.allow_tf32 = False
    t_torch = timed(torch_step, max(5, args.steps // 4))

    # ------------------------------------------------------------------ NSD bandwidth on a 2^28-element tensor
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
    t_nsd = timed(lambda i: dbp.nsd_quantize(big, rows_b, cols_b, step_big, 1, 0, codes_big, fmt_big, st_big, stream), 10)
    nnz_big = dbp.Stats.from_tensor(st_big).nnz
    nsd_bytes = n_big * (4 + 1 + 0.125 + 2.0 / 256) + 2.0 * nnz_big
    nsd = {"elements": n_big, "sparsity": 1 - nnz_big / n_big, "ms": t_nsd * 1e3, "GBps": nsd_bytes / t_nsd / 1e9,
           "frac_of_8TBps": nsd_bytes / t_nsd / 1e9 / PEAK_HBM_GBS, "bytes_per_element": nsd_bytes / n_big}
    t_nsd_codes = timed(lambda i: dbp.nsd_quantize(big, rows_b, cols_b, step_big, 1, 0, codes_big, None, None, stream), 10)
    nsd["codes_only_GBps"] = n_big * 5.0 / t_nsd_codes / 1e9
    # Algorithm 1 on the device and the steps around the quantiser, same tensor: step size (one read of delta),
    # then the quantiser with the rectifier mask on load, the device step and the bias code sums
    pair = torch.zeros(2, dtype=torch.float32, device=dev)
    ws_std = torch.empty(dbp.step_size_workspace_bytes(n_big), dtype=torch.uint8, device=dev)
    t_std = timed(lambda i: dbp.step_size(big, None, n_big, 8.0, pair, ws_std, stream), 10)
    act_big = torch.empty(n_big, dtype=torch.float32, device=dev).uniform_(-1, 1, generator=g)
    sums_big = torch.zeros(cols_b, dtype=torch.int64, device=dev)
    grad_big = torch.zeros(cols_b, dtype=torch.float32, device=dev)
    t_ex = timed(lambda i: dbp.nsd_quantize_ex(big, rows_b, cols_b, step_big, 1, 0, codes_big, None, None, act=act_big,
                                               step_dev=pair, bias_sums=sums_big, bias_grad=grad_big,
                                               bias_mode=dbp.BIAS_PER_COLUMN, bias_len=cols_b, stream=stream), 10)
    nsd["step_size_ms"] = t_std * 1e3
    nsd["step_size_GBps"] = n_big * 4.0 / t_std / 1e9
    nsd["masked_bias_nsd_ms"] = t_ex * 1e3
    nsd["masked_bias_nsd_GBps"] = n_big * 9.0 / t_ex / 1e9            # delta + activation read, codes written
    del big, codes_big, fmt_big, act_big

    extra = {}
    if args.all:
        extra = bench_conv_configs(dbp, workloads, torch, np, timed, stream)

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu = None
    if not args.no_cpu:
        from oracle import oracle as O
        threads = O.max_threads()
        reps, t_cpu = 0, 0.0
        t0 = time.perf_counter()
        while reps < 3 or (t_cpu < 5.0 and reps < 200):          # bounded sample: a few seconds of whole steps
            for p in layers:
                k, _ = O.nsd(p.delta, p.step, p.seed)
                O.linear_backward(p.W, p.X, codes=k, step=p.step, threads=threads)
            reps += 1
            t_cpu = time.perf_counter() - t0
        t_cpu /= reps
        cpu = {"value": dense_flops / t_cpu / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
               "sample": "%d whole steps (3 layers: NSD + dX + dW, zero codes skipped, fp64 accumulate), %.3f s each" % (reps, t_cpu)}

    out_line = {
        "metric": "dithered backward dense-equiv TFLOP/s (NSD + dX + dW, 3-layer MLP chain)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16x3 MFMA (exact int8 codes x 3-plane split of fp32), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "configs[1]: MLP backward chain, batch 256, 1024-4096-4096-1000, Delta=%g*std" % args.c,
                   "sparsity_per_layer": [round(s, 4) for s in sparsity], "path": "AUTO (matrix cores)"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "host_wall_ms_per_step": wall * 1e3,
        "whole_layer_entry_ms_per_step": t_layer * 1e3,
        "full_8bit_ms_per_step": t_q8 * 1e3,
        "vs_dense": {"same_library_fp32_mfma_ms": t_dense * 1e3, "torch_matmul_fp32_ms": t_torch * 1e3,
                     "speedup_vs_same_library": t_dense / t_step, "speedup_vs_torch": t_torch / t_step},
        "kernels_L2_us": {"nsd_1M_elements": t_nsd_small * 1e6, "dX_mfma": t_dx * 1e6, "dW_mfma": t_dw * 1e6,
                          "dX_and_dW_one_launch": t_both * 1e6,
                          "dX_gather": t_dx_g * 1e6, "dW_gather": t_dw_g * 1e6},
        "nsd_2^28": nsd,
    }
    if extra:
        out_line["other_configs"] = extra
    print(json.dumps(out_line))


def bench_conv_configs(dbp, workloads, torch, np, timed, stream):
    """Context lines for the conv / 8-bit configs: dithered vs the same library's dense backward."""
    dev = torch.device("cuda:0")
    res = {}
    problems = [("cfg3", workloads.config3()), ("cfg4a", workloads.config4a()), ("cfg4b", workloads.config4b())]
    problems += [("cfg5_s%g" % s, workloads.config5(s)) for s in (0.5, 0.9, 0.99)]
    problems += [("resnet_3x3_stride2", workloads.resnet_downsample())]
    for name, p in problems:
        N, Cc, H, Wd = p.X.shape
        K, _, R, S = p.W.shape
        i8 = p.X.dtype == np.int8
        xd = dbp.I8 if i8 else dbp.F32
        d, W, X = (torch.from_numpy(a).to(dev) for a in (p.delta, p.W, p.X))
        codes = torch.empty(p.delta.shape, dtype=torch.int8, device=dev)
        dX = torch.empty(p.X.shape, dtype=torch.float32, device=dev)
        dW = torch.empty(p.W.shape, dtype=torch.int32 if i8 else torch.float32, device=dev)
        ws = torch.empty(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, p.stride, p.pad, xd), dtype=torch.uint8, device=dev)
        st = torch.zeros(32, dtype=torch.uint8, device=dev)
        t = timed(lambda i: dbp.dithered_conv2d_backward(d, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, p.step, p.seed, 0,
                                                         codes, dX, dW, ws, st, dbp.PATH_AUTO, stream), 5, warm=1)
        P, Q = p.delta.shape[2:]
        flops = 2 * 2.0 * N * K * P * Q * Cc * R * S
        row = {"ms": t * 1e3, "dense_equiv_tflops": flops / t / 1e12, "sparsity": 1 - dbp.Stats.from_tensor(st).nnz / p.delta.size}
        t_x = timed(lambda i: dbp.conv2d_products(codes, None, p.step, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, dX, None, ws,
                                                  dbp.PATH_MFMA, stream), 5, warm=1)
        t_w = timed(lambda i: dbp.conv2d_products(codes, None, p.step, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, None, dW, ws,
                                                  dbp.PATH_MFMA, stream), 5, warm=1)
        row["dX_us"], row["dW_us"], row["nsd_us"] = t_x * 1e6, t_w * 1e6, max(t - t_x - t_w, 0.0) * 1e6
        if not i8:
            t_d = timed(lambda i: dbp.dense_conv2d_backward(d, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, dX, dW, ws, stream), 3, warm=1)
            row["same_library_dense_ms"] = t_d * 1e3
            # context only: the vendor library's fp32 convolution backward on the same shapes (dense gradient)
            dt = torch.from_numpy(p.delta).to(dev)
            torch.backends.cudnn.allow_tf32 = False
            f = lambda i: torch.ops.aten.convolution_backward(dt, X, W, None, [p.stride, p.stride], [p.pad, p.pad], [1, 1], False, [0, 0], 1,
                                                              [True, True, False])
            try:
                row["torch_conv_backward_fp32_ms"] = timed(f, 3, warm=2) * 1e3
            except Exception as e:                                   # context line: never fail the run over it
                row["torch_conv_backward_fp32_ms"] = None
            del dt
        if i8 and name == "cfg5_s0.9":
            # full 8-bit backward on the same layer: int8 weights too, both products exact int32
            W8 = torch.randint(-127, 128, p.W.shape, dtype=torch.int8, device=dev)
            dX32 = torch.empty(p.X.shape, dtype=torch.int32, device=dev)
            t8 = timed(lambda i: dbp.dithered_conv2d_backward_q8(d, W8, X, N, Cc, H, Wd, K, R, S, 1, p.pad, p.step, p.seed, 0,
                                                                 codes, dX32, dW, ws, st, stream), 5, warm=1)
            t8x = timed(lambda i: dbp.dithered_conv2d_backward_q8(d, W8, X, N, Cc, H, Wd, K, R, S, 1, p.pad, p.step, p.seed, 0,
                                                                  codes, dX32, None, ws, st, stream), 5, warm=1)
            row["full_8bit"] = {"ms": t8 * 1e3, "dense_equiv_tops": flops / t8 / 1e12, "nsd_plus_dX32_ms": t8x * 1e3}
            Wq = torch.empty(p.W.size, dtype=torch.int8, device=dev)
            sc = torch.empty(2, dtype=torch.float32, device=dev)
            wsq = torch.empty(dbp.quantize_int8_workspace_bytes(p.W.size), dtype=torch.uint8, device=dev)
            tq = timed(lambda i: dbp.quantize_int8(W, p.W.size, Wq, sc, wsq, stream), 5, warm=1)
            row["full_8bit"]["quantize_W_us"] = tq * 1e6
            del W8, dX32, Wq, sc, wsq
        if name == "cfg4a":
            # the gather kernels (walk the nonzero entries of the tile-sparse format) on the same layer, at the step above
            # and at steps that leave 1 % and 0.1 % nonzeros: whole call (NSD with the format + both products)
            row["gather"] = {}
            for target in (None, 0.99, 0.999):
                step = p.step if target is None else workloads.step_for_sparsity(p.delta, target)
                f = lambda i, path: dbp.dithered_conv2d_backward(d, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, step, p.seed, 0,
                                                                 codes, dX, dW, ws, st, path, stream)
                tg = timed(lambda i: f(i, dbp.PATH_GATHER), 3, warm=1)
                sp_ = 1 - dbp.Stats.from_tensor(st).nnz / p.delta.size
                tm = timed(lambda i: f(i, dbp.PATH_MFMA), 3, warm=1)
                row["gather"]["sparsity_%.4f" % sp_] = {"gather_ms": tg * 1e3, "matrix_core_ms": tm * 1e3}
        res[name] = row
        del d, W, X, codes, dX, dW, ws
    return res


if __name__ == "__main__":
    main()
