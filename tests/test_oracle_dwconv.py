"""Pins for the depthwise-convolution functions of the oracle: a depthwise convolution is the full convolution
whose weights are zero off the channel diagonal (exact integer identity, forward and weight gradient), and both
agree with shifted-view sums written with numpy."""
import numpy as np
import pytest

from oracle import ff_oracle as O
from workloads import make_inputs, make_weights, workload


@pytest.mark.parametrize("B,H,W,C,stride", [(2, 5, 7, 3, 1), (3, 8, 6, 8, 2), (1, 4, 4, 20, 1)])
def test_depthwise_is_the_channel_diagonal_of_a_full_convolution(B, H, W, C, stride):
    rng = np.random.default_rng(11)
    a = rng.integers(-127, 128, size=(B, H, W, C)).astype(np.int8)
    w = rng.integers(-127, 128, size=(C, 3, 3)).astype(np.int8)
    full = np.zeros((C, 3, 3, C), np.int8)
    for c in range(C):
        full[c, :, :, c] = w[c]
    acc = O.dwconv_forward(a, w, stride, 1)
    np.testing.assert_array_equal(acc, O.conv_forward(a, full, stride, 1))
    g = rng.integers(-127, 128, size=acc.shape).astype(np.int8)
    dw = O.dwconv_wgrad(g, a, 3, stride, 1, 0, B)
    dfull = O.conv_wgrad(g, a, 3, stride, 1, 0, B)
    for c in range(C):
        np.testing.assert_array_equal(dw[c], dfull[c, :, :, c])
    # sample range: the sum over [0, B) is the sum of the parts
    if B > 1:
        np.testing.assert_array_equal(dw, O.dwconv_wgrad(g, a, 3, stride, 1, 0, 1) + O.dwconv_wgrad(g, a, 3, stride, 1, 1, B))


def test_depthwise_against_shifted_views():
    rng = np.random.default_rng(12)
    B, H, W, C = 2, 6, 9, 5
    a = rng.integers(-127, 128, size=(B, H, W, C)).astype(np.int64)
    w = rng.integers(-127, 128, size=(C, 3, 3)).astype(np.int64)
    ap = np.pad(a, ((0, 0), (1, 1), (1, 1), (0, 0)))
    ref = sum(ap[:, kh:kh + H, kw:kw + W, :] * w[:, kh, kw] for kh in range(3) for kw in range(3))
    np.testing.assert_array_equal(O.dwconv_forward(a.astype(np.int8), w.astype(np.int8), 1, 1), ref)
    g = rng.integers(-127, 128, size=ref.shape).astype(np.int64)
    dref = np.stack([np.stack([(g * ap[:, kh:kh + H, kw:kw + W, :]).sum(axis=(0, 1, 2)) for kw in range(3)]) for kh in range(3)])
    np.testing.assert_array_equal(O.dwconv_wgrad(g.astype(np.int8), a.astype(np.int8), 3, 1, 1, 0, B), dref.transpose(2, 0, 1))


def test_train_step_runs_a_bottleneck_stack_and_stays_layer_local():
    wl = workload("tiny_dw")
    assert [l.kind for l in wl.layers] == ["conv", "conv", "dwconv", "conv", "conv", "dwconv", "conv"]
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    full = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, 1, keep=False)
    part = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, 1, keep=False, train_mask=[0, 0, 1, 0, 0, 0, 0])
    np.testing.assert_array_equal(part["w_master"][2], full["w_master"][2])
    assert part["w_master"][2].shape == (32, 3, 3) and np.any(part["w_master"][2] != W[2])
    for i in (0, 1, 3, 4, 5, 6):
        np.testing.assert_array_equal(part["w_master"][i], W[i])
