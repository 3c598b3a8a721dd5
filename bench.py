#!/usr/bin/env python3
"""Benchmark of the FF-INT8 layer-local train step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg1|cfg2|cfg3|cfg4|...]
                    [--theta matched|paper] [--no-cpu-baseline] [--no-other-configs]

A "step" is one ff_train_step: one iteration of the paper's Algorithm 1 over one synthetic batch
(positive + negative set, all layers: quantise, int8 forward, goodness/loss, look-ahead, int8 local
gradient, int8 weight gradient, update).  Inputs and weights are resident in HBM before the timed
region starts.  One JSON line is printed.

metric: FF-INT8 train samples/s per layer step = (B_pos + B_neg) * n_layers / step time, i.e. the rate
at which samples pass through one layer's complete step.  `roofline` scores the dominant kernel (the
int8 MFMA contraction, forward and weight-gradient launches together) from HIP events recorded on
the launch stream during the timed steps.

Goodness threshold.  The paper's theta = 2.0 (Section V-A) is far below the goodness of freshly
initialised layers (4000 for cfg5), so at theta = 2.0 the positive-pass coefficient of Eq. (1) is at the
exponent clamp, its int8 local gradient is all zeros and half of every weight-gradient launch multiplies
zeros, which runs faster than live data.  The default (--theta matched) therefore gives every layer its
own threshold, the median of its initial goodness (taken from one untimed step of the library itself), so
that both passes carry live int8 gradients; the theta = 2.0 figures are reported beside it as
`theta_paper`.  `operand_zero_fraction` lists the share of zero codes in every contraction operand.

`cpu_baseline` times the CPU oracle on the same workload (or a bounded sample of it).
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


def setup(ff, torch, wl, lookahead="coeff", theta_layer=None, state=None, launch_mode="auto"):
    """Device state of one workload.  `state` (from an earlier call) re-uses weights, inputs and workspace under a
    new descriptor, e.g. one with per-layer thresholds."""
    from workloads import make_inputs, make_weights
    B, k = wl.batch, len(wl.layers)
    if state is None:
        W = make_weights(wl)
        xp, xn = make_inputs(wl)
        d_w = [torch.from_numpy(w.reshape(w.shape[0], -1)).cuda() for w in W]
        d_wq = [torch.zeros((l.N, ff.ff_pitch(l.K)), dtype=torch.int8, device="cuda") for l in wl.layers]
        d_sw = [torch.zeros(1, device="cuda") for _ in wl.layers]
        ws1 = torch.empty(ff.WS_MIN_BYTES, dtype=torch.uint8, device="cuda")
        for i, l in enumerate(wl.layers):
            ff.ff_quantize(d_w[i], l.N, l.K, ff.ROUND_NEAREST, 0, 0, d_wq[i], None, d_sw[i], ws1)
        d_xp = torch.from_numpy(xp.reshape(B, -1)).cuda()
        d_xn = torch.from_numpy(xn.reshape(B, -1)).cuda()
        loss = torch.empty((k, 2), device="cuda")
        good = torch.empty((k, 2, B), device="cuda")
        ws = None
    else:
        _, d_xp, d_xn, loss, good, ws, d_w, d_wq, d_sw = state
    net = ff.Net(wl.layers, B, d_w, d_wq, d_sw, lookahead=lookahead, theta_layer=theta_layer, launch_mode=launch_mode)
    if net.workspace_bytes() == 0:
        raise SystemExit(f"bench.py: workload {wl.name} is not covered by --lookahead {lookahead} --launch-mode {launch_mode}")
    if ws is None or ws.numel() < net.workspace_bytes():
        ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    return net, d_xp, d_xn, loss, good, ws, d_w, d_wq, d_sw


def matched_thetas(ff, torch, wl, st):
    """One threshold per layer: the median goodness of the layer over both data sets at the initial weights, from
    one untimed step of the library with lr = 0 (the weights are left as they are)."""
    net, d_xp, d_xn, loss, good, ws = st[:6]
    ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, 0.0, wl.sr_seed, 0, loss, good, ws)
    torch.cuda.synchronize()
    k = len(wl.layers)
    med = good.reshape(k, -1).median(dim=1).values.cpu().tolist()
    return [float(m) if l.role != "proj" else 0.0 for m, l in zip(med, wl.layers)]


def cpu_baseline(wl, sample_batch: int, lookahead: str = "coeff", theta=None):
    """The CPU oracle as it stands, timed on this host, on a smaller batch of the same network."""
    from oracle import ff_oracle as O
    from workloads import make_inputs, make_weights, scaled
    small = scaled(wl, sample_batch)
    W = make_weights(small)
    xp, xn = make_inputs(small)
    O.lib()
    t0 = time.perf_counter()
    step = O.train_step if lookahead == "coeff" else O.train_step_chain
    step(small.layers, W, xp, xn, small.theta if theta is None else theta, small.lam, small.lr, small.sr_seed, 0, keep=False)
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
    clk = torch.zeros(16, dtype=torch.int64, device="cuda")
    for kind in ("gaussian", "constant", "zeros"):
        a_q, w_q = codes(a_shape[0], a_shape[1], kind), codes(l.N, l.K, kind)
        for _ in range(3):
            ff.ff_layer_forward(desc, a_q, w_q, acc, gsum, vmax, ws)
        torch.cuda.synchronize()
        clk.zero_()
        ff.ff_timing_clock_probe(clk)
        ff.ff_timing_reset()
        ff.ff_timing_enable(True)
        for _ in range(iters):
            ff.ff_layer_forward(desc, a_q, w_q, acc, gsum, vmax, ws)
        torch.cuda.synchronize()
        ff.ff_timing_enable(False)
        ff.ff_timing_clock_probe(None)
        ms, n = ff.ff_timing_read(gi)
        ops = 2.0 * M * l.K * l.N
        c = clk.cpu().tolist()
        res[kind] = {"avg_launch_ms": ms / n, "TOPs": ops / (ms / n * 1e-3) / 1e12,
                     "frac_of_peak": ops / (ms / n * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
                     "mean_shader_clock_GHz": c[0] / max(c[1], 1) * 0.1}
    return {"probe": "forward contraction vs operand values", "workload": wl.name, "M": M, "K": l.K, "N": l.N,
            "launches": iters, "results": res}


def operand_zero_fractions(ff, torch, wl, theta_layer, theta):
    """Share of zero int8 codes in every operand of the two contractions, per layer and pass, for a dense stack at
    its initial weights: the step taken apart into the single-operation entry points (quantise / hand-off, forward,
    goodness and loss, look-ahead, local gradient)."""
    if any(l.kind != "dense" for l in wl.layers):
        return None
    from workloads import make_inputs, make_weights
    B, k = wl.batch, len(wl.layers)
    W = make_weights(wl)
    xs = make_inputs(wl)
    ws = torch.empty(max([ff.WS_MIN_BYTES] + [ff.ff_layer_workspace_bytes(ff.layer_desc(l, B)) for l in wl.layers]),
                     dtype=torch.uint8, device="cuda")
    f32 = lambda: torch.zeros(1, device="cuda")
    d_w = [torch.from_numpy(w).cuda() for w in W]
    w_q = [torch.zeros((l.N, ff.ff_pitch(l.K)), dtype=torch.int8, device="cuda") for l in wl.layers]
    s_w = [f32() for _ in wl.layers]
    out = {"weights": [], "pos": [], "neg": []}
    for i, l in enumerate(wl.layers):
        ff.ff_quantize(d_w[i], l.N, l.K, ff.ROUND_NEAREST, 0, 0, w_q[i], None, s_w[i], ws)
        out["weights"].append(round(float((w_q[i][:, :l.K] == 0).float().mean()), 4))
    for p, name in enumerate(("pos", "neg")):
        x = torch.from_numpy(xs[p]).cuda()
        coeff = torch.zeros((k, B), device="cuda")
        keep = []
        a_q = a_qt = s_a = None
        for i, l in enumerate(wl.layers):
            desc = ff.layer_desc(l, B)
            nq, nqt, ns = (torch.zeros((B, ff.ff_pitch(l.K)), dtype=torch.int8, device="cuda"),
                           torch.zeros((l.K, ff.ff_pitch(B)), dtype=torch.int8, device="cuda"), f32())
            tag = ff.ff_stream_tag(0, i, p, ff.KIND_ACT)
            if i == 0:
                ff.ff_quantize(x, B, l.K, ff.ROUND_STOCHASTIC, wl.sr_seed, tag, nq, nqt, ns, ws)
            else:
                pd, pacc, psa, pG, pamax = keep[-1][0], keep[-1][1], keep[-1][2], keep[-1][5], keep[-1][6]
                ff.ff_layer_handoff(pd, pacc, psa, s_w[i - 1], pG, pamax, ff.ROUND_STOCHASTIC, wl.sr_seed, tag, nq, nqt, ns)
            a_q, a_qt, s_a = nq, nqt, ns
            acc = torch.empty((B, ff.ff_pitch32(l.N)), dtype=torch.int32, device="cuda")
            gsum = torch.zeros(B, dtype=torch.int64, device="cuda")
            vmax = torch.zeros(B, dtype=torch.int32, device="cuda")
            ff.ff_layer_forward(desc, a_q, w_q[i], acc, gsum, vmax, ws)
            G, lm, amax = torch.empty(B, device="cuda"), f32(), f32()
            th = theta if theta_layer is None else theta_layer[i]
            ff.ff_goodness_loss(desc, gsum, vmax, s_a, s_w[i], ff.PASS_POS if p == 0 else ff.PASS_NEG, th, G, coeff[i], lm, amax)
            keep.append((desc, acc, s_a, vmax, a_qt, G, amax, a_q))
        ct = torch.empty_like(coeff)
        ff.ff_lookahead(coeff, k, B, wl.lam, ct)
        for i, l in enumerate(wl.layers):
            desc, acc, s_a, vmax, a_qt, G, amax, a_q = keep[i]
            gy = torch.zeros((l.N, ff.ff_pitch(B)), dtype=torch.int8, device="cuda")
            dw = torch.empty((l.N, ff.ff_pitch32(l.K)), dtype=torch.int32, device="cuda")
            s_g = f32()
            ff.ff_layer_backward_local(desc, acc, vmax, s_a, s_w[i], ct[i], ff.ROUND_STOCHASTIC, wl.sr_seed,
                                       ff.ff_stream_tag(0, i, p, ff.KIND_GRAD), a_qt, gy, s_g, dw, ws)
            torch.cuda.synchronize()
            out[name].append({"layer_input_codes": round(float((a_q[:, :l.K] == 0).float().mean()), 4),
                              "local_gradient_codes": round(float((gy[:, :B] == 0).float().mean()), 4)})
        del keep
    return out


def mfma_ceiling_probe(ff, torch, iterations=16384, launches=10):
    """Register-resident int8 MFMA loop (ff_probe_mfma_ceiling) by operand kind: TOP/s and the clock it ran at."""
    sink = torch.empty(256 * 512, dtype=torch.int32, device="cuda")
    out = {"probe": "v_mfma_i32_32x32x32_i8 on register-resident operands, 8 wavefronts per compute unit, "
                    f"{iterations} x 8 instructions per wavefront, {launches} launches timed back to back",
           "peak_TOPs": INT8_MFMA_PEAK_TOPS}
    for kind, name in ((0, "zeros"), (1, "all_codes_1"), (2, "pseudo_random_words")):
        for _ in range(3):
            ff.ff_probe_mfma_ceiling(kind, iterations, sink, None)
        torch.cuda.synchronize()
        clk = torch.zeros(2, dtype=torch.int64, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = 0.0
        for _ in range(launches):
            ops += ff.ff_probe_mfma_ceiling(kind, iterations, sink, clk)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        c = clk.cpu().tolist()
        tops = ops / (ms * 1e-3) / 1e12
        out[name] = {"ms_per_launch": round(ms / launches, 4), "TOPs": round(tops, 1),
                     "frac_of_peak": round(tops / INT8_MFMA_PEAK_TOPS, 4),
                     "mean_shader_clock_GHz": round(c[0] / max(c[1], 1) * 0.1, 3)}
    return out


def time_steps(ff, torch, wl, st, theta, steps, start, classes=("gemm_fwd", "gemm_dw")):
    net, d_xp, d_xn, loss, good, ws = st[:6]
    ff.ff_timing_reset()
    ff.ff_timing_enable(True, classes)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ff.ff_train_step(net, d_xp, d_xn, theta, wl.lam, wl.lr, wl.sr_seed, start + i, loss, good, ws)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ff.ff_timing_enable(False)
    out = {}
    for ci, name in enumerate(ff.KERNEL_CLASSES):
        ms, n = ff.ff_timing_read(ci)
        out[name] = {"ms_per_step": ms / steps, "launches_per_step": n / steps}
    return dt / steps * 1e3, out


def contraction_ops_per_step(wl):
    # fwd + dW, both passes, of the layers that run on the MFMA contraction kernel (depthwise layers do not)
    return sum(2.0 * 2 * wl.batch * l.rows_per_sample * l.K * l.N * 2 for l in wl.layers if l.kind != "dwconv")


def gemm_figures(wl, kern):
    gemm_ms = kern["gemm_fwd"]["ms_per_step"] + kern["gemm_dw"]["ms_per_step"]
    launches = kern["gemm_fwd"]["launches_per_step"] + kern["gemm_dw"]["launches_per_step"]
    ops = contraction_ops_per_step(wl)
    avg_ms = gemm_ms / max(launches, 1)
    ach = ops / max(launches, 1) / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
    half = lambda c: (ops / 2) / (kern[c]["ms_per_step"] * 1e-3) / 1e12 if kern[c]["ms_per_step"] > 0 else 0.0
    return {"achieved": ach, "ops_per_launch": ops / max(launches, 1), "avg_launch_ms": avg_ms,
            "fwd_TOPs": half("gemm_fwd"), "dw_TOPs": half("gemm_dw")}


def other_config(ff, torch, name, steps=10, warmup=3):
    """ms per step and the derived rates of another configuration (eager launches; matched thresholds)."""
    from workloads import workload
    wl = workload(name)
    st = setup(ff, torch, wl)
    th = matched_thetas(ff, torch, wl, st)
    st = setup(ff, torch, wl, theta_layer=th, state=st)
    net, d_xp, d_xn, loss, good, ws = st[:6]
    for i in range(warmup):
        ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, i, loss, good, ws)
    ms, kern = time_steps(ff, torch, wl, st, wl.theta, steps, warmup, ("fused",))
    k, B = len(wl.layers), wl.batch
    ops = contraction_ops_per_step(wl)
    fused = kern["fused"]["launches_per_step"] > 0
    # the same step as one kernel per operation on one stream (what FF_LAUNCH_AUTO does not pick for this stack unless
    # the two times are equal), with events around the contraction launches: their share of the int8 peak
    st_k = setup(ff, torch, wl, theta_layer=th, state=st, launch_mode="kernels")
    for i in range(warmup):
        ff.ff_train_step(st_k[0], d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, i, loss, good, st_k[5])
    ms_k, kern_k = time_steps(ff, torch, wl, st_k, wl.theta, steps, warmup)
    g = gemm_figures(wl, kern_k)
    # one captured HIP graph of the default launch mode, replayed
    step_dev = torch.tensor([2 * warmup + 2 * steps], dtype=torch.int64, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ff.ff_train_step_at(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, step_dev, 1, loss, good, ws)
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_g = (time.perf_counter() - t0) / steps * 1e3
    del graph
    out_extra = {"ms_per_step_graph_replay": round(ms_g, 4), "ms_per_step_per_operation_kernels_one_stream": round(ms_k, 4)}
    if not fused:
        out_extra["launch"] = ("one kernel per operation; update chains of different layers on several streams where "
                               "FF_LAUNCH_AUTO chooses so (cfg2, cfg3, cfg4)")
    if fused:
        # phase durations inside the launch (100 MHz stamps of its first workgroup), mean of 20 steps
        stamps = torch.zeros(32, dtype=torch.int64, device="cuda")
        ff.ff_timing_fused_stamps(stamps)
        nph = 2 * k + 4
        acc = None
        for i in range(20):
            ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, 1000 + i, loss, good, ws)
            torch.cuda.synchronize()
            t = stamps[:nph + 1].cpu().numpy().astype("int64")
            d = (t[1:] - t[:-1]) * 0.01   # us
            acc = d if acc is None else acc + d
        ff.ff_timing_fused_stamps(None)
        names = ["absmax_input"] + [n for i in range(k) for n in (f"quantise_{i}", f"forward_{i}")] + \
                ["goodness_lookahead_gradquant", "wgrad_update", "requantise"]
        phases = {n: round(float(v) / 20, 2) for n, v in zip(names, acc)}
        out_extra.update({"launch": "single persistent launch (FF_LAUNCH_FUSED via FF_LAUNCH_AUTO)",
                          "phase_us_inside_the_launch": phases,
                          "phase_note": "each phase but the last ends in a device-wide barrier across the 8 XCDs"})
    return {"layers": k, "batch_per_pass": B, "ms_per_step": round(ms, 4), **out_extra,
            "samples_per_s_per_layer_step": round(2 * B * k / (ms * 1e-3), 1),
            "whole_step_int8_TOPs": round(ops / (ms * 1e-3) / 1e12, 1),
            "whole_step_frac_of_int8_peak": round(ops / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
            "contraction_launches_frac_of_int8_peak": round(g["achieved"] / INT8_MFMA_PEAK_TOPS, 4),
            "contraction_note": "from the one-stream per-operation pass (launch durations are only meaningful unoverlapped)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--settle-seconds", type=float, default=0.4,
                    help="before the W warmup steps, keep the GPU under the same load for this long (untimed), so that "
                         "the timed region starts from the clock/power state of sustained training rather than from "
                         "idle; 0 switches it off (the first ~10 steps after idle run 3-8 %% slower)")
    ap.add_argument("--theta", choices=("matched", "paper"), default="matched",
                    help="matched: one threshold per layer, the median initial goodness (both passes carry live int8 "
                         "gradients); paper: theta = 2.0 for every layer (Section V-A)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the cfg1-cfg4 step times")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB-read / 1 GiB-write elementwise kernel (torch.add) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled against known traffic")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph-replay timing")
    ap.add_argument("--timed-region-only", action="store_true",
                    help="stop after the timed steps and print a short line (for rocprofv3 runs: the trace or the counters "
                         "then cover the threshold set-up step, the warm-up and the timed steps only)")
    ap.add_argument("--launch-mode", choices=("auto", "kernels", "fused", "lanes"), default="auto",
                    help="kernels: one kernel per operation on one stream; lanes: the same, the update chains of "
                         "different layers on up to three streams; fused: the whole step as one persistent launch (small "
                         "dense stacks); auto: fused or lanes where they apply and the layers are small")
    ap.add_argument("--lookahead", choices=("coeff", "chain"), default="coeff",
                    help="chain: the exact-derivative variant of the look-ahead (dense stacks; one more contraction per layer)")
    ap.add_argument("--gemm-data-probe", action="store_true",
                    help="instead of the train step, time the forward contraction of the first layer on Gaussian, "
                         "constant and zero int8 operands (same kernel and traffic; shows the clock/power effect)")
    ap.add_argument("--mfma-ceiling-probe", action="store_true",
                    help="instead of the train step, time a register-resident loop of the contraction kernel's MFMA "
                         "instruction on zero, constant and pseudo-random operands (no operand movement: the rate the "
                         "matrix pipes sustain under the power manager)")
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
    if args.mfma_ceiling_probe:
        print(json.dumps(mfma_ceiling_probe(ff, torch)))
        return 0
    st_paper = setup(ff, torch, wl, args.lookahead, launch_mode=args.launch_mode)
    k, B = len(wl.layers), wl.batch
    theta_layer = matched_thetas(ff, torch, wl, st_paper) if args.theta == "matched" else None
    st = (setup(ff, torch, wl, args.lookahead, theta_layer=theta_layer, state=st_paper, launch_mode=args.launch_mode)
          if theta_layer else st_paper)
    net, d_xp, d_xn, loss, good, ws = st[:6]

    if args.pmc_calibration:
        cal_in = torch.ones(1 << 28, device="cuda")          # 2^28 fp32 = 1 GiB
        cal_out = torch.empty_like(cal_in)
        torch.add(cal_in, 1.0, out=cal_out)
        torch.cuda.synchronize()
        del cal_in, cal_out

    step_no = 0
    settle_steps = 0
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for i in range(10):
            ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, step_no, loss, good, ws)
            step_no += 1
        settle_steps += 10
        torch.cuda.synchronize()
    for i in range(args.warmup):
        ff.ff_train_step(net, d_xp, d_xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, step_no, loss, good, ws)
        step_no += 1
    torch.cuda.synchronize()
    # ---- the timed region: K steps; HIP events bracket only the launches of the dominant kernel (the two
    # contractions), because an event record after every one of the ~30 launches of a step would itself
    # lengthen the step by 5-10 % (it keeps consecutive launches from overlapping)
    ms_per_step, kern = time_steps(ff, torch, wl, st, wl.theta, args.steps, step_no)
    step_no += args.steps
    samples = 2 * B
    if args.timed_region_only:
        # for profiler runs: nothing but the set-up step, the warm-up and the timed steps is launched
        g = gemm_figures(wl, kern)
        print(json.dumps({"workload": wl.name, "ms_per_step": ms_per_step, "steps": args.steps, "warmup": args.warmup,
                          "launch_mode": args.launch_mode, "lookahead": args.lookahead,
                          "contraction_avg_launch_ms": g["avg_launch_ms"], "contraction_TOPs": g["achieved"],
                          "fwd_TOPs": g["fwd_TOPs"], "dw_TOPs": g["dw_TOPs"],
                          "contraction_frac_of_int8_peak": g["achieved"] / INT8_MFMA_PEAK_TOPS}))
        return 0

    # ---- outside the timed region: the same K steps with every kernel class timed (the per-class breakdown) and the
    # shader-clock probe of the contraction launches switched on; then K replays of one captured HIP graph
    # (ff_train_step_at keeps the step number in device memory)
    clk = torch.zeros(16, dtype=torch.int64, device="cuda")
    ff.ff_timing_clock_probe(clk)
    all_ms, breakdown = time_steps(ff, torch, wl, st, wl.theta, args.steps, step_no, None)
    ff.ff_timing_clock_probe(None)
    step_no += args.steps
    clk_v = clk.cpu().tolist()
    mean_clock_ghz = clk_v[0] / max(clk_v[1], 1) * 0.1

    def phases(o):   # shader clocks per tile by phase, as seen by the first thread of each workgroup
        n = max(clk_v[o + 4], 1)
        return {"tiles": clk_v[o + 4], "operand_round_trip": round(clk_v[o] / n), "main_loop": round(clk_v[o + 1] / n),
                "epilogue": round(clk_v[o + 2] / n), "wait_for_other_waves": round(clk_v[o + 3] / n)}
    phase_clocks = {"forward": phases(8), "weight_gradient": phases(2),
                    "note": "shader clocks per 256x256 tile; the MFMA pipe needs 2048 clocks per 128-byte reduction step"}
    extra = {"all_classes_timed_ms_per_step": all_ms}
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
        step_no += args.steps + 3
        extra["graph_replay_ms_per_step"] = g_ms
        extra["graph_replay_samples_per_s_per_layer_step"] = 2 * B * k / (g_ms * 1e-3)

    # dominant kernel: the int8 contraction (forward + weight-gradient launches; each launch covers both passes)
    g = gemm_figures(wl, kern)
    ops_per_step = contraction_ops_per_step(wl)
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            traffic = tj.get("gemm_bytes_per_launch")
            traffic_source = ("not measured in this run: recorded rocprofv3 FETCH_SIZE / WRITE_SIZE figure read from "
                              f"profiles/traffic_{wl.name}.json ({tj.get('source', '')})")
        except Exception:
            traffic = None
    peak_at_clock = 256 * mean_clock_ghz * 1e9 * 8192 / 1e12
    roofline = {"bound": "mfma", "kernel": "k_gemm_nt_i8 (forward and weight-gradient launches)",
                "achieved": g["achieved"], "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": g["achieved"] / INT8_MFMA_PEAK_TOPS, "traffic": traffic, "traffic_source": traffic_source,
                "ops_per_launch": g["ops_per_launch"], "avg_launch_ms": g["avg_launch_ms"],
                "fwd_TOPs": g["fwd_TOPs"], "dw_TOPs": g["dw_TOPs"],
                "fwd_frac": g["fwd_TOPs"] / INT8_MFMA_PEAK_TOPS, "dw_frac": g["dw_TOPs"] / INT8_MFMA_PEAK_TOPS,
                "mean_shader_clock_GHz": round(mean_clock_ghz, 4),
                "peak_measured_clock": round(peak_at_clock, 1),
                "frac_of_peak_measured_clock": round(g["achieved"] / peak_at_clock, 4) if peak_at_clock > 0 else None,
                "phase_clocks_per_tile": phase_clocks,
                "clock_note": "mean shader clock of the contraction launches, read inside the kernels (shader-clock "
                              "cycles over constant-100-MHz ticks) during the fully instrumented pass; "
                              "peak_measured_clock = 256 CU x 8192 op/clk x that clock"}

    # theta = 2.0 (Section V-A) beside the matched thresholds: the positive-pass gradient operand is then all zeros
    theta_paper = None
    if theta_layer is not None:
        p_ms, p_kern = time_steps(ff, torch, wl, st_paper, wl.theta, max(5, args.steps // 2), step_no)
        step_no += max(5, args.steps // 2)
        pg = gemm_figures(wl, p_kern)
        theta_paper = {"theta": wl.theta, "ms_per_step": p_ms, "contraction_frac": pg["achieved"] / INT8_MFMA_PEAK_TOPS,
                       "fwd_TOPs": pg["fwd_TOPs"], "dw_TOPs": pg["dw_TOPs"],
                       "note": "positive-pass local gradient is all zeros at this threshold (see operand_zero_fraction "
                               "for the matched run); not the headline"}

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
        "settle": {"seconds": args.settle_seconds, "untimed_steps_before_warmup": settle_steps,
                   "why": "the timed region starts from the clock state of sustained training, not from idle"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 (int32 accumulate; fp32 scales, goodness, master weights)", "data": "synthetic",
        "config": {"workload": wl.name, "layers": [f"{l.K}->{l.N}" for l in wl.layers],
                   "batch_pos": B, "batch_neg": B, "lookahead": args.lookahead, "launch_mode": args.launch_mode, "lambda": wl.lam,
                   "theta": ("per layer, median initial goodness (both passes live): " + str([round(t, 1) for t in theta_layer]))
                   if theta_layer is not None else wl.theta,
                   "lr": wl.lr,
                   "layer_steps_per_step": k, "whole_step_samples_per_s": samples / (ms_per_step * 1e-3),
                   "int8_TOPs_whole_step": ops_per_step / (ms_per_step * 1e-3) / 1e12,
                   "whole_step_frac_of_int8_peak": ops_per_step / (ms_per_step * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS},
        "int8_mfma_pct_of_peak": 100.0 * g["achieved"] / INT8_MFMA_PEAK_TOPS,
        "roofline": roofline,
        "theta_paper": theta_paper,
        "kernels_ms_per_step": {n: round(v["ms_per_step"], 5) for n, v in breakdown.items()},
        "hbm_bound_kernels": hbm,
        "other_launch_modes": extra,
        "paper_context": "Jetson Orin Nano, whole training runs: 4.6% faster, 8.3% less energy, 27.0% less memory "
                         "than BP-GDAI8 (Table V); no per-step figure is published",
    }
    # free the main workload before the side measurements
    del net, d_xp, d_xn, loss, good, ws, st, st_paper
    torch.cuda.empty_cache()
    try:
        out["operand_zero_fraction"] = operand_zero_fractions(ff, torch, wl, theta_layer, wl.theta)
    except ff.FFError as e:   # a side measurement never takes the headline down
        out["operand_zero_fraction"] = {"error": str(e)}
    torch.cuda.empty_cache()
    # what the matrix pipes sustain with no operand movement at all, by operand values (outside the timed region)
    out["roofline"]["register_loop_ceiling"] = mfma_ceiling_probe(ff, torch, iterations=8192, launches=5)
    if not args.no_other_configs and wl.name == "cfg5":
        oc = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4"):
            oc[name] = other_config(ff, torch, name)
            torch.cuda.empty_cache()
        oc["note"] = ("ms_per_step: eager launches in the default launch mode (FF_LAUNCH_AUTO), 10 steps after 3 warm-up "
                      "steps, thresholds matched per layer; outside the timed region")
        out["other_configs"] = oc
    if not args.no_cpu_baseline:
        sb = args.cpu_sample_batch or {"cfg5": 8192, "cfg2": 1024, "cfg1": 64, "cfg3": 64, "cfg4_plain": 32}.get(wl.name, min(B, 256))
        out["cpu_baseline"] = cpu_baseline(wl, min(sb, B), args.lookahead, theta_layer)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
