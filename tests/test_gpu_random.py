"""Seeded sweeps over random small shapes: the same comparisons as tests/test_gpu_parity.py (HIP library against the
CPU oracle, int8 / int32 bit-exact, fp32 within 1e-5), on shapes nobody picked by hand — odd sizes, single rows and
columns, widths just past a tile or a 16-byte boundary."""
import os
import sys
from dataclasses import replace

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import test_gpu_parity as P  # noqa: E402
from test_gpu_parity import ff  # noqa: E402,F401  (fixture)
from workloads import Workload, bottleneck_stack, conv_stack, mlp, res_stack  # noqa: E402


def _dims(rng, n, lo, hi):
    """n sizes in [lo, hi], biased towards the edges of 16 / 64 / 256 blocks"""
    out = []
    for _ in range(n):
        if rng.random() < 0.4:
            base = int(rng.choice([16, 32, 64, 128, 256]))
            v = base * int(rng.integers(1, max(2, hi // base + 1))) + int(rng.integers(-2, 3))
        else:
            v = int(rng.integers(lo, hi + 1))
        out.append(int(min(max(v, lo), hi)))
    return out


def test_random_quantize_shapes(ff):
    rng = np.random.default_rng(101)
    for _ in range(60):
        rows, cols = _dims(rng, 2, 1, 700)
        P.test_quantize(ff, rows, cols, int(rng.integers(0, 2)))


def test_random_dense_layers(ff):
    rng = np.random.default_rng(202)
    for _ in range(40):
        B, K, N = _dims(rng, 3, 1, 600)
        P.test_layer_forward(ff, B, K, N, int(rng.integers(0, 2)))
        P.test_backward_local_and_update(ff, B, K, N)
        P.test_chain_gradients_and_input_gradient(ff, B, K, N, int(rng.integers(0, 2)))


def test_random_larger_dense_layers(ff):
    """Several tiles of every tile shape with ragged edges, and reductions long enough for a split weight gradient."""
    rng = np.random.default_rng(212)
    for _ in range(6):
        B, K, N = _dims(rng, 3, 200, 1500)
        P.test_layer_forward(ff, B, K, N, 1)
        P.test_backward_local_and_update(ff, B, K, N)
    for (B, K, N) in ((5000, 40, 24), (3000, 272, 130)):     # few outputs, a long reduction: split weight gradient
        P.test_backward_local_and_update(ff, B, K, N)


def test_random_conv_layers(ff):
    rng = np.random.default_rng(303)
    for _ in range(40):
        ks = int(rng.choice([1, 3]))
        stride = int(rng.choice([1, 2]))
        H, W = (int(v) for v in rng.integers(3, 21, 2))
        if rng.random() < 0.4:            # maps the fast transposed-patch paths accept
            H, W = int(rng.choice([4, 8, 16])), int(rng.choice([8, 16, 32]))
        Cin = int(rng.choice([3, 5, 16, 24, 32, 40, 64, 70]))
        Cout = int(rng.choice([4, 8, 20, 32, 64, 72]))
        B = int(rng.integers(1, 7))
        P.test_conv_forward_and_backward(ff, B, H, W, Cin, Cout, ks, stride)


def test_random_depthwise_layers(ff):
    rng = np.random.default_rng(404)
    for _ in range(25):
        H, W = (int(v) for v in rng.integers(3, 25, 2))
        C = int(rng.choice([4, 6, 16, 20, 64, 68, 130]))
        P.test_depthwise_forward_and_backward(ff, int(rng.integers(1, 6)), H, W, C, int(rng.choice([1, 2])))


def test_random_dense_stacks(ff):
    """Whole steps of random dense stacks, both readings of the look-ahead; theta near the goodness of the first
    layer so that both passes carry a live gradient."""
    rng = np.random.default_rng(505)
    for case in range(16):
        depth = int(rng.integers(2, 5))
        widths = [_dims(rng, 1, 12, 300)[0]] + _dims(rng, depth, 1, 300)   # the label overlay needs ten input features
        B = int(rng.integers(1, 90))
        norm = bool(rng.integers(0, 2))
        layers = mlp(widths, norm)
        if case % 3 == 2:      # some stacks mix ReLU and identity activations
            layers = tuple(replace(l, relu=int(rng.integers(0, 2))) for l in layers)
        wl = Workload(f"rand{case}", layers, B, "uniform_onehot", lam=float(rng.choice([0.0, 0.1, 0.7])),
                      theta=float(rng.choice([2.0, 10.0, 40.0])))
        P._run_steps(ff, wl, 2, launch_mode="kernels")
        P._run_steps(ff, wl, 2, launch_mode="fused")
        if not norm:
            P._run_steps(ff, wl, 2, lookahead="chain")


def test_random_conv_stacks(ff):
    rng = np.random.default_rng(606)
    for case in range(10):
        chans = [3] + [int(rng.choice([5, 8, 16, 17, 24, 32])) for _ in range(int(rng.integers(1, 4)))]
        h, w = int(rng.choice([4, 6, 8, 12])), int(rng.choice([10, 11, 16]))   # the label overlay needs ten columns
        wl = Workload(f"randc{case}", conv_stack(chans, h, w), int(rng.integers(2, 9)), "uniform_onehot",
                      lam=float(rng.choice([0.0, 0.25])))
        P._run_steps(ff, wl, 2)


def test_random_residual_and_bottleneck_stacks(ff):
    """Basic residual blocks (identity and projection skips) and inverted bottlenecks (1x1, depthwise 3x3, 1x1) with
    random widths, strides and map sizes."""
    rng = np.random.default_rng(707)
    for case in range(8):
        h, w = int(rng.choice([4, 8, 12])), int(rng.choice([12, 16]))
        stem = int(rng.choice([8, 16]))
        if case % 2 == 0:
            stages = [(stem, 1, 1)] + [(int(rng.choice([16, 24, 32])), int(rng.choice([1, 2])), int(rng.integers(1, 3)))
                                       for _ in range(int(rng.integers(1, 3)))]
            layers = res_stack(stem, stages, h, w)
        else:
            blocks = [(int(rng.integers(1, 5)), int(rng.choice([8, 16, 20, 24])), int(rng.choice([1, 2])))
                      for _ in range(int(rng.integers(1, 3)))]
            layers = bottleneck_stack(stem, blocks, h, w)
        wl = Workload(f"randr{case}", layers, int(rng.integers(2, 7)), "uniform_onehot", lam=float(rng.choice([0.0, 0.05])))
        P._run_steps(ff, wl, 2)
