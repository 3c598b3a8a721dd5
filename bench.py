#!/usr/bin/env python3
"""Benchmark of the FF-INT8 layer-local train step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg2|cfg1] [--no-cpu-baseline]

A "step" is one ff_train_step: one iteration of the paper's Algorithm 1 over one synthetic batch
(positive + negative set, all layers: quantise, int8 forward, goodness/loss, look-ahead, int8 local
gradient, int8 weight gradient, update).  Inputs and weights are resident in HBM before the timed
region starts.  One JSON line is printed.

metric: FF-INT8 train samples/s per layer step = (B_pos + B_neg) * n_layers / step time, i.e. the rate
at which samples pass through one layer's complete step.  `roofline` scores the dominant kernel (the
int8 MFMA contraction, forward and weight-gradient launches together) from HIP events recorded on
the launch stream during the timed steps.  `cpu_baseline` times the CPU oracle on a bounded sample
(a smaller batch of the same network).
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

INT8_MFMA_PEAK_TOPS = 256 * 2.4e9 * 8192 / 1e12   # 256 CUs x 2.4 GHz x 8192 int8 ops/CU/clk = 5033 TOP/s
HBM_PEAK_GBS = 8000.0


def setup(ff, torch, wl, lookahead="coeff"):
    from workloads import make_inputs, make_weights
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    B, k = wl.batch, len(wl.layers)
    d_w = [torch.from_numpy(w.reshape(w.shape[0], -1)).cuda() for w in W]
    d_wq = [torch.zeros((l.N, ff.ff_pitch(l.K)), dtype=torch.int8, device="cuda") for l in wl.layers]
    d_sw = [torch.zeros(1, device="cuda") for _ in wl.layers]
    ws1 = torch.empty(ff.WS_MIN_BYTES, dtype=torch.uint8, device="cuda")
    for i, l in enumerate(wl.layers):
        ff.ff_quantize(d_w[i], l.N, l.K, ff.ROUND_NEAREST, 0, 0, d_wq[i], None, d_sw[i], ws1)
    net = ff.Net(wl.layers, B, d_w, d_wq, d_sw, lookahead=lookahead)
    if net.workspace_bytes() == 0:
        raise SystemExit(f"bench.py: workload {wl.name} is not covered by --lookahead {lookahead}")
    ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    loss = torch.empty((k, 2), device="cuda")
    good = torch.empty((k, 2, B), device="cuda")
    d_xp = torch.from_numpy(xp.reshape(B, -1)).cuda()
    d_xn = torch.from_numpy(xn.reshape(B, -1)).cuda()
    return net, d_xp, d_xn, loss, good, ws


def cpu_baseline(wl, sample_batch: int, lookahead: str = "coeff"):
    """The CPU oracle as it stands, timed on this host, on a smaller batch of the same network."""
    from oracle import ff_oracle as O
    from workloads import make_inputs, make_weights, scaled
    small = scaled(wl, sample_batch)
    W = make_weights(small)
    xp, xn = make_inputs(small)
    O.lib()
    t0 = time.perf_counter()
    step = O.train_step if lookahead == "coeff" else O.train_step_chain
    step(small.layers, W, xp, xn, small.theta, small.lam, small.lr, small.sr_seed, 0, keep=False)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    k = len(small.layers)
    return {"value": 2 * sample_batch * k / dt, "unit": "samples/s per layer step", "cores": cores,
            "kind": "oracle", "seconds": dt,
            "sample": (f"one whole oracle train step of {wl.name} (batch {wl.batch}+{wl.batch})" if sample_batch == wl.batch
                       else f"one oracle train step of {wl.name} at batch {sample_batch}+{sample_batch} "
                            f"(full batch is {wl.batch}+{wl.batch}); rate is per sample, so it carries over")}


def gemm_data_probe(ff, torch, wl, iters: int = 20):
    """The forward contraction of the workload's first layer (one pass), timed on operands that differ only in
    their VALUES: int8 codes of a quantised Gaussian, a constant, zeros.  Same kernel, same instruction stream,
    same memory traffic; what changes is the switching activity in the MFMA pipe, so the spread shows how far
    the launch duration is set by the shader clock under power management rather than by the kernel."""
    l, B = wl.layers[0], wl.batch
    desc = ff.layer_desc(l, B)
    M = B * l.rows_per_sample
    acc = torch.empty((M, ff.ff_pitch32(l.N)), dtype=torch.int32, device="cuda")
    gsum = torch.zeros(B, dtype=torch.int64, device="cuda")
    vmax = torch.zeros(B, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(ff.ff_layer_workspace_bytes(desc), ff.WS_MIN_BYTES), dtype=torch.uint8, device="cuda")
    a_shape = (B, l.K) if l.kind == "dense" else (B * l.H * l.W, l.C_in)
    gen = torch.Generator(device="cuda").manual_seed(1)

    def codes(rows, cols, kind):
        t = torch.zeros((rows, ff.ff_pitch(cols)), dtype=torch.int8, device="cuda")
        if kind == "gaussian":
            t[:, :cols] = (torch.randn((rows, cols), device="cuda", generator=gen) * 23.0).round().clamp(-127, 127).to(torch.int8)
        elif kind == "constant":
            t[:, :cols] = 1
        return t

    res = {}
    gi = ff.KERNEL_CLASSES.index("gemm_fwd")
    for kind in ("gaussian", "constant", "zeros"):
        a_q, w_q = codes(a_shape[0], a_shape[1], kind), codes(l.N, l.K, kind)
        for _ in range(3):
            ff.ff_layer_forward(desc, a_q, w_q, acc, gsum, vmax, ws)
        torch.cuda.synchronize()
        ff.ff_timing_reset()
        ff.ff_timing_enable(True)
        for _ in range(iters):
            ff.ff_layer_forward(desc, a_q, w_q, acc, gsum, vmax, ws)
        torch.cuda.synchronize()
        ff.ff_timing_enable(False)
        ms, n = ff.ff_timing_read(gi)
        ops = 2.0 * M * l.K * l.N
        res[kind] = {"avg_launch_ms": ms / n, "TOPs": ops / (ms / n * 1e-3) / 1e12,
                     "frac_of_peak": ops / (ms / n * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS}
    return {"probe": "forward contraction vs operand values", "workload": wl.name, "M": M, "K": l.K, "N": l.N,
            "launches": iters, "results": res}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB-read / 1 GiB-write elementwise kernel (torch.add) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled against known traffic")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph-replay timing")
    ap.add_argument("--lookahead", choices=("coeff", "chain"), default="coeff",
                    help="chain: the exact-derivative variant of the look-ahead (dense stacks; one more contraction per layer)")
    ap.add_argument("--gemm-data-probe", action="store_true",
                    help="instead of the train step, time the forward contraction of the first layer on Gaussian, "
                         "constant and zero int8 operands (same kernel and traffic; shows the clock/power effect)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2506_22771_amd as ff
    from workloads import workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ff.lib()
    torch.cuda.set_device(0)
    wl = workload(args.workload)
    if args.gemm_data_probe:
        print(json.dumps(gemm_data_probe(ff, torch, wl)))
        return 0
    net, d_xp, d_xn, loss, good, ws = setup(ff, torch, wl, args.lookahead)
    k, B = len(wl.layers), wl.batch

    if args.pmc_calibration:
        cal_in = torch.ones(1 << 28, device="cuda")          # 2^28 fp32 = 1 GiB
        cal_out = torch.empty_like(cal_in)
        torch.add(cal_in, 1.0, out=cal_out)
        torch.cuda.synchronize()
        del cal_in, cal_out

    def run_steps(n, start):
        for i in range(n):
            ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, start + i, loss, good, ws)
        return start + n

    def read_classes(steps):
        out = {}
        for ci, name in enumerate(ff.KERNEL_CLASSES):
            ms, n = ff.ff_timing_read(ci)
            out[name] = {"ms_per_step": ms / steps, "launches_per_step": n / steps}
        return out

    step_no = run_steps(args.warmup, 0)
    torch.cuda.synchronize()
    # ---- the timed region: K steps; HIP events bracket only the launches of the dominant kernel (the two
    # contractions), because an event record after every one of the ~30 launches of a step would itself
    # lengthen the step by 5-10 % (it keeps consecutive launches from overlapping)
    ff.ff_timing_reset()
    ff.ff_timing_enable(True, ("gemm_fwd", "gemm_dw"))
    t0 = time.perf_counter()
    step_no = run_steps(args.steps, step_no)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ff.ff_timing_enable(False)
    ms_per_step = dt / args.steps * 1e3
    samples = 2 * B
    kern = read_classes(args.steps)

    # ---- outside the timed region: the same K steps with every kernel class timed (the per-class breakdown),
    # and as K replays of one captured HIP graph (ff_train_step_at keeps the step number in device memory)
    ff.ff_timing_reset()
    ff.ff_timing_enable(True)
    t0 = time.perf_counter()
    step_no = run_steps(args.steps, step_no)
    torch.cuda.synchronize()
    extra = {"all_classes_timed_ms_per_step": (time.perf_counter() - t0) / args.steps * 1e3}
    ff.ff_timing_enable(False)
    breakdown = read_classes(args.steps)
    if not args.no_graph:
        step_dev = torch.tensor([step_no], dtype=torch.int64, device="cuda")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ff.ff_train_step_at(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, step_dev, 1, loss, good, ws)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) / args.steps * 1e3
        extra["graph_replay_ms_per_step"] = g_ms
        extra["graph_replay_samples_per_s_per_layer_step"] = 2 * B * k / (g_ms * 1e-3)

    # dominant kernel: the int8 contraction (forward + weight-gradient launches; each launch covers both passes)
    gemm_ms = kern["gemm_fwd"]["ms_per_step"] + kern["gemm_dw"]["ms_per_step"]
    gemm_launches = kern["gemm_fwd"]["launches_per_step"] + kern["gemm_dw"]["launches_per_step"]
    # fwd + dW, both passes, of the layers that run on the MFMA contraction kernel (depthwise layers do not)
    ops_per_step = sum(2.0 * 2 * B * l.rows_per_sample * l.K * l.N * 2 for l in wl.layers if l.kind != "dwconv")
    ops_per_launch = ops_per_step / max(gemm_launches, 1)
    avg_launch_ms = gemm_ms / max(gemm_launches, 1)
    achieved = ops_per_launch / (avg_launch_ms * 1e-3) / 1e12 if avg_launch_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("gemm_bytes_per_launch")
        except Exception:
            traffic = None
    roofline = {"bound": "mfma", "kernel": "k_gemm_nt_i8 (forward and weight-gradient launches)",
                "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": achieved / INT8_MFMA_PEAK_TOPS, "traffic": traffic,
                "ops_per_launch": ops_per_launch, "avg_launch_ms": avg_launch_ms,
                "fwd_TOPs": (ops_per_step / 2) / (kern["gemm_fwd"]["ms_per_step"] * 1e-3) / 1e12
                if kern["gemm_fwd"]["ms_per_step"] > 0 else 0.0,
                "dw_TOPs": (ops_per_step / 2) / (kern["gemm_dw"]["ms_per_step"] * 1e-3) / 1e12
                if kern["gemm_dw"]["ms_per_step"] > 0 else 0.0}

    # HBM-bound kernel classes (dense stacks): algorithmic bytes per step / time of the fully instrumented pass
    hbm = None
    if all(l.kind == "dense" for l in wl.layers):
        S = 2 * B   # samples per step, both passes
        byts = {"absmax": 4.0 * wl.layers[0].K * S,
                "quant_act": sum((4.0 * l.K + 2.0 * l.K) * S for l in wl.layers),    # read fp32 / int32, write q and q^T
                "quant_grad": sum((4.0 * l.N + 1.0 * l.N) * S for l in wl.layers),   # read int32, write g^T
                "update": sum(16.0 * l.K * l.N for l in wl.layers),                  # read w, dW+, dW-, write w
                "quant_w": sum(5.0 * l.K * l.N for l in wl.layers)}                  # read w, write w_q
        hbm = {}
        for name, nbytes in byts.items():
            ms = breakdown[name]["ms_per_step"]
            if ms > 0:
                gbs = nbytes / (ms * 1e-3) / 1e9
                hbm[name] = {"algorithmic_MB_per_step": round(nbytes / 1e6, 1), "GBps": round(gbs, 1),
                             "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}

    out = {
        "metric": "FF-INT8 train samples/sec per layer step; int8 MFMA TOPS as % of peak",
        "value": samples * k / (ms_per_step * 1e-3),
        "unit": "samples/s per layer step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 (int32 accumulate; fp32 scales, goodness, master weights)", "data": "synthetic",
        "config": {"workload": wl.name, "layers": [f"{l.K}->{l.N}" for l in wl.layers],
                   "batch_pos": B, "batch_neg": B, "lookahead": args.lookahead, "lambda": wl.lam, "theta": wl.theta, "lr": wl.lr,
                   "layer_steps_per_step": k, "whole_step_samples_per_s": samples / (ms_per_step * 1e-3),
                   "int8_TOPs_whole_step": ops_per_step / (ms_per_step * 1e-3) / 1e12},
        "int8_mfma_pct_of_peak": 100.0 * achieved / INT8_MFMA_PEAK_TOPS,
        "roofline": roofline,
        "kernels_ms_per_step": {n: round(v["ms_per_step"], 5) for n, v in breakdown.items()},
        "hbm_bound_kernels": hbm,
        "other_launch_modes": extra,
        "paper_context": "Jetson Orin Nano, whole training runs: 4.6% faster, 8.3% less energy, 27.0% less memory "
                         "than BP-GDAI8 (Table V); no per-step figure is published",
    }
    if not args.no_cpu_baseline:
        sb = args.cpu_sample_batch or {"cfg5": 8192, "cfg2": 1024, "cfg1": 64, "cfg3": 64, "cfg4_plain": 32}.get(wl.name, min(B, 256))
        out["cpu_baseline"] = cpu_baseline(wl, min(sb, B), args.lookahead)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
