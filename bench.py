#!/usr/bin/env python3
"""Benchmark of the GCN hot path on one MI355X.

One "step" = one full-graph epoch (forward + loss + backward) of the 3-layer GCN of the
second benchmark configuration: R-MAT scale-20 graph (16 N directed edges, symmetrised,
self-loops, sym-normalised), X = N x 128 ~ N(0,1), Glorot weights 128 -> 256 -> 256 -> 16,
16 classes, fp32.  Inputs are synthetic and resident in HBM before the timed region.

Prints ONE JSON line: whole-job throughput in edges*feat/s (sum over layers of
nnz(A_hat) * d^(l), divided by the step time), the roofline of the dominant kernel (the
aggregation gather at 256 columns) from HIP events recorded around its launches inside the
timed region, and the CPU oracle timed on a bounded, down-scaled sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def measured_traffic(config, width):
    """HBM bytes per launch of the dominant kernel, taken from the committed rocprofv3 --pmc
    summary of this same command (counters cannot be read from inside the run)."""
    files = {("c2", 256): "c2_aggregate_pmc.txt", ("c3", 128): "c3_aggregate_pmc.txt",
             ("c4", 128): "c4_aggregate_pmc.txt"}
    if (config, width) not in files:
        return None
    path = os.path.join(ROOT, "profiles", files[(config, width)])
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split()[1])
    except OSError:
        pass
    return None


def model_dims(name):
    if name == "c2":
        return [128, 256, 256, 16]
    if name == "c1":
        return [64, 32, 8]
    if name == "c5":
        return [100, 256, 256, 47]
    raise ValueError(name)


def make_inputs(name, scale, seed):
    import numpy as np

    import graphgen as gg

    dims = model_dims(name)
    src, dst, n = gg.config_graph(name, seed=seed, scale_override=scale)
    if name in ("c1", "c5"):
        x = gg.uniform(seed, 1, n, dims[0])
    else:
        x = gg.normal(seed, 1, n, dims[0])
    # weights with a leading dimension of whole 16-byte groups (47 columns -> ld 48)
    ws = [gg.glorot(seed, 10 + l, dims[l], dims[l + 1], ld=(dims[l + 1] + 3) // 4 * 4)[:, :dims[l + 1]]
          for l in range(len(dims) - 1)]
    y = gg.labels(seed, 5, n, dims[-1])
    return src, dst, n, x, ws, y, dims


def cpu_baseline(name, scale, seed):
    """The oracle as it stands on the host cores, one forward+backward step of a down-scaled
    instance of the same generator and model."""
    import numpy as np

    import oracle

    src, dst, n, x, ws, y, dims = make_inputs(name, scale, seed)
    g = oracle.transpose(oracle.normalize(oracle.build_csr(src, dst, n)))
    ws = [np.ascontiguousarray(w) for w in ws]
    t0 = time.perf_counter()
    if name == "c5":
        oracle.gcn_step(g, x, ws, y, q=oracle.Q_BF16)
    else:
        oracle.gcn_step(g, x, ws, y)
    dt = time.perf_counter() - t0
    work = sum(g.nnz * d for d in dims[:-1])
    return {
        "value": work / dt, "unit": "edges*feat/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"same generator and model at R-MAT scale {scale} (N={n}, nnz={g.nnz}), "
                  f"one fwd+bwd step, {dt:.1f} s",
    }


def bench_single_layer(args, mg, dev):
    """Configs 3 and 4 (not the default line): one layer forward + backward at the real shape.

    c3: a 128-column slice of a 1024-wide layer, R-MAT scale 24 with 8 N directed edges; H comes
    from the seeded generator, the 68.7 GB upstream gradient G is drawn on the device.
    c4: N = 1.11e8 with 1.6e9 power-law directed edges, one 128 -> 128 layer in the last-layer
    form (no ReLU).  Three N x 128 tensors (56.8 GB each) plus the graph (54 GB) are resident:
    the upstream gradient reuses the layer output's storage and dH is written over H, which the
    backward pass no longer reads.  Tensor values are drawn on the device (they do not matter for
    the timing; parity at this size is covered by the tests)."""
    import numpy as np
    import torch

    import graphgen as gg
    from paper_2501_01951_amd.model import padded_rows

    if args.config == "c3":
        scale = args.scale or 24
        n, k, m, relu = 1 << scale, 128, 1024, True
        src, dst = gg.rmat_edges(args.seed, scale, 8 * n)
        what = f"c3: one GCN layer 128->1024 fwd+bwd, R-MAT scale {scale}"
    else:
        src, dst, n = gg.config_graph("c4", args.seed, args.scale)
        k, m, relu = 128, 128, False
        what = "c4: one GCN layer 128->128 fwd+bwd (no ReLU), power-law graph"
    s_d, d_d = dev(src.view(np.int32)), dev(dst.view(np.int32))
    del src, dst
    g = mg.build_csr(s_d, d_d, n)
    del s_d, d_d
    torch.cuda.empty_cache()
    mg.normalize(g)
    nnz = g.nnz
    hd = padded_rows(n, k, torch.float32, "cuda")
    if args.config == "c3":
        hd.copy_(torch.from_numpy(gg.normal(args.seed, 1, n, k)))
    else:
        hd.normal_()
    wd = dev(gg.glorot(args.seed, 10, k, m))
    zd = padded_rows(n, k, torch.float32, "cuda")
    outd = padded_rows(n, m, torch.float32, "cuda")
    if args.config == "c3":
        gd = padded_rows(n, m, torch.float32, "cuda")
        gd.normal_()
        dhd = padded_rows(n, k, torch.float32, "cuda")
    else:
        gd, dhd = outd, hd
    dwd = torch.empty(k, m, device="cuda")
    pipe = mg.Pipeline()

    def step():
        mg.layer_fwd(g, hd, wd, zd, outd, pipe, relu=relu, n_chunks=args.chunks)
        mg.layer_bwd(g, zd, outd, wd, gd, dwd, dhd, pipe, relu=relu, n_chunks=args.chunks)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    pipe.timing(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    names = ["agg_g4", "agg_g8", "agg_g16", "agg_g32", "agg_g64", "update_fwd", "update_dgrad",
             "update_wgrad"]
    kinds = {}
    for i, nm in enumerate(names):
        ms, cnt = pipe.timing_read(i)
        if cnt:
            kinds[nm] = {"total_ms": ms, "launches": cnt, "avg_ms": ms / cnt}
    agg_ms = kinds["agg_g32"]["avg_ms"]
    algo = 8.0 * nnz + 2.0 * n * k * 4 + 8.0 * n
    traffic = measured_traffic(args.config, k)
    print(json.dumps({
        "metric": "GCN layer fwd+bwd edges*feat/s", "value": nnz * k / dt, "unit": "edges*feat/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{what}, N={n}, nnz(A_hat)={nnz}", "n_nodes": n, "nnz": nnz,
                   "update_arith": args.update_arith},
        "kernels": kinds,
        "roofline": {"bound": "hbm", "achieved": algo / (agg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": algo / (agg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": traffic, "kernel": "aggregate_kernel, 128 fp32 columns",
                     "avg_launch_ms": agg_ms, "algorithmic_bytes_per_launch": algo},
        "gemm_tflops": {kk: 2.0 * n * k * m / (kinds[kk]["avg_ms"] * 1e-3) / 1e12
                        for kk in ("update_fwd", "update_dgrad", "update_wgrad")},
    }))


def bench_variant(args, mg, dev):
    """--model sage | gin (not the default line): the paper's two other architectures, three
    layers with 128 hidden units, on the graph and features of the chosen configuration."""
    import numpy as np
    import torch

    import graphgen as gg

    src, dst, n = gg.config_graph(args.config, seed=args.seed, scale_override=args.scale)
    d0 = model_dims(args.config)[0]
    classes = model_dims(args.config)[-1]
    dims = [d0, 128, 128, classes]
    x = gg.normal(args.seed, 1, n, d0)
    y = gg.labels(args.seed, 5, n, classes)
    sage = args.model == "sage"
    flags = mg.SYMMETRIZE | (0 if sage else mg.ADD_SELF_LOOPS)
    g = mg.build_csr(dev(src.view(np.int32)), dev(dst.view(np.int32)), n, flags)
    mg.normalize(g, mg.NORM_MEAN if sage else mg.NORM_SUM, eps=0.0 if sage else 0.1)
    nnz = g.nnz
    if sage:
        ws = [dev(gg.glorot(args.seed, 20 + l, 2 * dims[l], dims[l + 1])) for l in range(3)]
        step = mg.SAGEStep(g, dev(x), ws, dev(y))
        agg_in, agg_out = step.xc[1][:, :128], step.xc[1][:, 128:256]
    else:
        w1s = [dev(0.02 * gg.glorot(args.seed, 30 + l, dims[l], 128)) for l in range(3)]
        w2s = [dev(gg.glorot(args.seed, 40 + l, 128, dims[l + 1])) for l in range(3)]
        step = mg.GINStep(g, dev(x), w1s, w2s, dev(y))
        agg_in, agg_out = step.h[1], step.z[1]
    for _ in range(args.warmup):
        step.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step.step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    loss = step.loss.item()
    # the aggregation at the hidden width, timed alone with events on the stream it runs on
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * args.steps)]
    for i in range(args.steps):
        ev[2 * i].record()
        mg.aggregate(g, agg_in, agg_out)
        ev[2 * i + 1].record()
    torch.cuda.synchronize()
    agg_ms = sum(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(args.steps)) / args.steps
    per_launch = 8.0 * nnz + 2.0 * n * 128 * 4 + 8.0 * n
    achieved = per_launch / (agg_ms * 1e-3) / 1e9
    name = "GraphSAGE (mean)" if sage else "GIN (eps = 0.1)"
    out = {
        "metric": f"{name} fwd+bwd edges*feat/s", "value": sum(nnz * d for d in dims[:-1]) / dt,
        "unit": "edges*feat/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.config} graph: 3-layer {name} {'-'.join(map(str, dims))}, one "
                               f"fwd+bwd epoch, N={n}, nnz(A_hat)={nnz}",
                   "n_nodes": n, "nnz": nnz, "seed": args.seed, "update_arith": args.update_arith},
        "loss": loss,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "aggregate_kernel<8, 32, 0, false, true> (128 fp32 columns)",
                     "avg_launch_ms": agg_ms, "algorithmic_bytes_per_launch": per_launch},
    }
    if not args.no_cpu_baseline:
        import oracle

        s2, d2, n2 = gg.config_graph(args.config, seed=args.seed, scale_override=args.cpu_scale)
        og = oracle.build_csr(s2, d2, n2, True, not sage)
        og = oracle.transpose(oracle.normalize_mean(og) if sage else oracle.normalize_sum(og, 0.1))
        x2, y2 = gg.normal(args.seed, 1, n2, d0), gg.labels(args.seed, 5, n2, classes)
        t0 = time.perf_counter()
        if sage:
            oracle.sage_step(og, x2, [gg.glorot(args.seed, 20 + l, 2 * dims[l], dims[l + 1])
                                      for l in range(3)], y2)
        else:
            oracle.gin_step(og, x2, [0.02 * gg.glorot(args.seed, 30 + l, dims[l], 128) for l in range(3)],
                            [gg.glorot(args.seed, 40 + l, 128, dims[l + 1]) for l in range(3)], y2)
        t = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": sum(og.nnz * d for d in dims[:-1]) / t, "unit": "edges*feat/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"same generator and model at R-MAT scale {args.cpu_scale} (N={n2}, "
                      f"nnz={og.nnz}), one fwd+bwd step, {t:.1f} s"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--scale", type=int, default=None, help="override the R-MAT scale")
    ap.add_argument("--chunks", type=int, default=1, help="row chunks of the layer pipeline")
    ap.add_argument("--seed", type=int, default=250101951)
    ap.add_argument("--cpu-scale", type=int, default=20, help="R-MAT scale of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-event-timing", action="store_true")
    ap.add_argument("--model", default="gcn", choices=["gcn", "sage", "gin"],
                    help="gcn: the benchmark line; sage / gin: the two other architectures of the "
                         "paper's experiments on the same graph (3 layers, 128 hidden units)")
    ap.add_argument("--hip-graph", action="store_true",
                    help="record the step into a HIP graph and time its replays (one stream, no "
                         "per-kernel events): for small inputs, where launches dominate")
    ap.add_argument("--update-arith", default="fp32", choices=["fp32", "bf16x3"],
                    help="matrix-core arithmetic of the update products of fp32 features: fp32 MFMA "
                         "(the benchmark line) or three bf16 terms per operand, six bf16 MFMAs per "
                         "product (forward and data gradient of wide layers)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives are part of it); "
                 "use --gpus 1")

    import numpy as np
    import torch

    import paper_2501_01951_amd as mg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    mg.load_library()
    torch.cuda.set_device(0)
    mg.set_update_arith(mg.ARITH_BF16X3 if args.update_arith == "bf16x3" else mg.ARITH_FP32)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if args.model != "gcn":
        assert args.config in ("c1", "c2"), "--model sage/gin run on the graphs of c1 and c2"
        return bench_variant(args, mg, dev)
    if args.config in ("c3", "c4"):
        return bench_single_layer(args, mg, dev)
    src, dst, n, x, ws, y, dims = make_inputs(args.config, args.scale, args.seed)

    s_d, d_d = dev(src.view(np.int32)), dev(dst.view(np.int32))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g = mg.build_csr(s_d, d_d, n)
    mg.normalize(g)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t0
    nnz = g.nnz
    del s_d, d_d

    pipe = mg.Pipeline()
    bf16 = args.config == "c5"  # config 5 stores features in bf16
    x_d = torch.from_numpy(x).cuda()
    if bf16:
        x_d = x_d.to(torch.bfloat16)
    w_d = [torch.from_numpy(np.ascontiguousarray(w.base if w.base is not None else w)).cuda()[:, :w.shape[1]]
           for w in ws]
    step = mg.GCNStep(g, x_d, w_d, dev(y), n_chunks=args.chunks, pipe=pipe)

    # A plain copy kernel of known size: its FETCH_SIZE / WRITE_SIZE readings calibrate the
    # counter units when this command runs under rocprofv3 --pmc.
    calib_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)

    run_step = step.step
    if args.hip_graph:
        assert args.chunks == 1, "--hip-graph times the single-stream schedule"
        args.no_event_timing = True
        step.capture()
        run_step = step.replay
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    pipe.timing(not args.no_event_timing)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    loss = step.loss.item()

    work = sum(nnz * d for d in dims[:-1])  # sum over layers of nnz * d^(l)
    value = work / (dt / args.steps)

    kinds = {}
    if not args.no_event_timing:
        names = ["agg_g4", "agg_g8", "agg_g16", "agg_g32", "agg_g64", "update_fwd", "update_dgrad",
                 "update_wgrad"]
        for k, nm in enumerate(names):
            ms, cnt = pipe.timing_read(k)
            if cnt:
                kinds[nm] = {"total_ms": ms, "launches": cnt, "avg_ms": ms / cnt}
    pipe.timing(False)

    roofline = None
    agg = {k: v for k, v in kinds.items() if k.startswith("agg")}
    if agg:
        dom = max(agg, key=lambda k: agg[k]["total_ms"])
        gsz = int(dom.split("g")[-1])
        esz = 2 if bf16 else 4
        f = gsz * 16 // esz  # columns of a pass of that width class (16 bytes per lane)
        # algorithmic minimum per full-graph launch: index + value stream, every feature row
        # read once, every output row written once, one row pointer per row
        full = 8.0 * nnz + 2.0 * n * f * esz + 8.0 * n
        launches_per_layer_call = max(1, args.chunks)
        per_launch = full / launches_per_layer_call
        avg_s = agg[dom]["avg_ms"] * 1e-3
        achieved = per_launch / avg_s / 1e9
        roofline = {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(args.config, f) if args.chunks == 1 else None,
            "kernel": f"aggregate_kernel<8, {gsz}, {1 if bf16 else 0}, false, true> "
                      f"({f} {'bf16' if bf16 else 'fp32'} columns)",
            "avg_launch_ms": agg[dom]["avg_ms"], "launches": agg[dom]["launches"],
            "algorithmic_bytes_per_launch": per_launch,
            "gather_bytes_per_launch": (nnz * (8.0 + f * esz) + n * f * esz) / launches_per_layer_call,
        }

    out = {
        "metric": "GCN layer fwd+bwd edges*feat/s", "value": value, "unit": "edges*feat/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage, f32 accumulate" if bf16 else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{args.config}: {len(dims) - 1}-layer GCN {'-'.join(map(str, dims))}, one "
                        f"fwd+bwd epoch, {'Erdos-Renyi' if args.config == 'c1' else 'R-MAT'} graph "
                        f"N={n}, nnz(A_hat)={nnz}",
            "n_nodes": n, "nnz": nnz, "row_chunks": args.chunks, "seed": args.seed,
            "hip_graph": bool(args.hip_graph), "update_arith": args.update_arith,
        },
        "loss": loss, "build_csr_normalize_ms": t_build * 1e3, "kernels": kinds,
        "roofline": roofline,
    }
    # the same steps with the opt-in update arithmetic (fp32 operands as three bf16 terms on the
    # bf16 matrix cores), after and outside the timed region above: reported beside the result
    if args.update_arith == "fp32" and not bf16 and not args.hip_graph:
        mg.set_update_arith(mg.ARITH_BF16X3)
        try:
            for _ in range(2):
                run_step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                run_step()
            torch.cuda.synchronize()
            dt3 = (time.perf_counter() - t0) / args.steps
            out["with_update_arith_bf16x3"] = {"ms_per_step": dt3 * 1e3, "value": work / dt3,
                                               "loss": step.loss.item()}
        finally:
            mg.set_update_arith(mg.ARITH_FP32)
    # what this device sustains on a plain copy and on register-only MFMA chains (outside the
    # timed region): context for the published peaks the fractions above are quoted against
    del step, calib_src, calib_dst
    torch.cuda.empty_cache()
    try:
        out["measured_peaks"] = mg.measure_peaks()
    except mg.MixGCNError as e:  # needs 8 GiB of free device memory; not part of the result
        out["measured_peaks"] = {"error": str(e)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_scale, args.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
