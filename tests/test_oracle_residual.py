"""Pins for the residual-block part of the oracle (a reading; Section IV-C names ResNet-style blocks without
mechanics): special cases that reduce to the plain layer, exact values of the order-free goodness, and the
wiring of a block (which tensors are added, which gradient updates the projection) by brute force on a tiny stack."""
import numpy as np

from oracle import ff_oracle as O
from workloads import make_inputs, make_weights, workload


def test_zero_skip_is_the_plain_layer_and_zero_accumulators_give_the_skip():
    rng = np.random.default_rng(3)
    acc = rng.integers(-50000, 50000, size=(5, 37), dtype=np.int32)
    s_a, s_w = np.float32(0.0123), np.float32(0.0077)
    zero = np.zeros(acc.shape, np.float32)
    for relu in (0, 1):
        plain = O.handoff(acc, relu, 0, s_a, s_w, np.zeros(5, np.float32))
        np.testing.assert_array_equal(O.residual_act(acc, zero, relu, s_a, s_w), plain)
    x_q = rng.integers(-127, 128, size=acc.shape).astype(np.int8)
    u = O.skip_identity(x_q, np.float32(0.031))
    np.testing.assert_array_equal(u, O.dequantize(x_q, np.float32(0.031)))
    y = O.residual_act(np.zeros_like(acc), u, 1, s_a, s_w)
    np.testing.assert_array_equal(y, np.maximum(u, 0))
    # the projection skip is the plain (un-rectified) activity of the projection's accumulators
    np.testing.assert_array_equal(O.skip_projection(acc, s_a, s_w), O.handoff(acc, 0, 0, s_a, s_w, np.zeros(5, np.float32)))


def test_order_free_goodness_exact_on_powers_of_two_and_close_to_plain_sum():
    # activities amax * 2^-j: every term floor(2^-2j * 2^40) is exact, so G is the exactly rounded sum of squares
    amax = np.float32(3.0)
    j = np.array([[0, 1, 2, 3, 5, 9], [1, 1, 4, 4, 7, 20]])
    y = (amax * np.exp2(-j.astype(np.float64))).astype(np.float32)
    y[1, 0] = amax          # the tensor maximum may sit in any sample
    gd = O.goodness_fx(y)
    expect = np.sum(y.astype(np.float64) ** 2, axis=1)
    np.testing.assert_array_equal(gd["G"], expect.astype(np.float32))
    np.testing.assert_array_equal(gd["ymax"], np.max(np.abs(y), axis=1))
    # random activities: within 1e-6 of the fp64 sum, independent of the order of the terms, and exactly
    # quadratic under a power-of-two rescale of the tensor
    rng = np.random.default_rng(0)
    y = np.maximum(rng.normal(size=(7, 4096)), 0).astype(np.float32)
    a = O.goodness_fx(y)
    assert np.all(np.abs(a["G"] - a["G_plain"]) <= 1e-6 * a["G_plain"])
    perm = rng.permutation(y.shape[1])
    b = O.goodness_fx(y[:, perm])
    np.testing.assert_array_equal(a["g_int"], b["g_int"])
    np.testing.assert_array_equal(a["G"], b["G"])
    c = O.goodness_fx(y * np.float32(4.0))
    np.testing.assert_array_equal(c["g_int"], a["g_int"])
    np.testing.assert_array_equal(c["G"], a["G"] * np.float32(16.0))
    # a vanishing tensor has zero goodness
    z = O.goodness_fx(np.zeros((2, 8), np.float32))
    assert np.all(z["G"] == 0) and np.all(z["g_int"] == 0)


def test_gradient_from_activities_equals_gradient_from_accumulators():
    rng = np.random.default_rng(5)
    acc = rng.integers(-90000, 90000, size=(4, 50), dtype=np.int32)
    s_a, s_w = np.float32(0.02), np.float32(0.004)
    ct = rng.normal(size=4).astype(np.float32)
    y = O.handoff(acc, 1, 0, s_a, s_w, np.zeros(4, np.float32))
    np.testing.assert_array_equal(O.local_grad_f32(y, ct), O.local_grad(acc, 1, s_a, s_w, ct))


def _run(wl, W, mask=None, lam=None, step=4):
    xp, xn = make_inputs(wl)
    return O.train_step(wl.layers, W, xp, xn, wl.theta, wl.lam if lam is None else lam, wl.lr, wl.sr_seed, step,
                        keep=True, train_mask=mask)


def test_block_wiring_by_brute_force():
    wl = workload("tiny_res")
    L = wl.layers
    assert [l.role for l in L] == ["ff", "ff", "ff", "proj", "ff", "ff"]
    assert [l.skip for l in L] == ["none", "none", "identity", "none", "none", "projection"]
    W = make_weights(wl)
    r = _run(wl, W)
    B = wl.batch
    for p in range(2):
        f = r["fwd"]
        # identity block: output = relu(s*acc2 + dequantised int8 input of conv1), the input of conv1 being the stem output
        t = f[2][p]["acc"].astype(np.float32) * (f[2][p]["s_a"] * r["s_w_in"][2])
        u = f[1][p]["a_q"].astype(np.float32) * f[1][p]["s_a"]
        np.testing.assert_array_equal(f[2][p]["y"], np.maximum(t + u, np.float32(0)))
        # down-sampling block: projection and conv1 quantise the SAME tensor (the output of layer 2) with different
        # rounding streams, so their codes differ by at most one step of either grid
        da = f[3][p]["a_q"].astype(np.float32) * f[3][p]["s_a"] - f[4][p]["a_q"].astype(np.float32) * f[4][p]["s_a"]
        assert np.max(np.abs(da)) <= f[3][p]["s_a"] + f[4][p]["s_a"]
        assert f[3][p]["s_a"] == f[4][p]["s_a"]            # same absmax
        t = f[5][p]["acc"].astype(np.float32) * (f[5][p]["s_a"] * r["s_w_in"][5])
        u = f[3][p]["acc"].astype(np.float32) * (f[3][p]["s_a"] * r["s_w_in"][3])
        np.testing.assert_array_equal(f[5][p]["y"], np.maximum(t + u, np.float32(0)))
        # the projection's accumulators are a strided 1x1 convolution of its int8 input
        xq = f[3][p]["a_q"][:, ::2, ::2, :].astype(np.int64)
        wq = r["w_q_in"][3].reshape(L[3].C_out, L[3].C_in).astype(np.int64)
        np.testing.assert_array_equal(f[3][p]["acc"], np.einsum("bhwc,nc->bhwn", xq, wq))
    # the projection is updated with the block output's quantised gradient and its own int8 input
    dws, sgs, sas = [], [], []
    for p in range(2):
        gq = r["grads"][5][p]["gy_q"].astype(np.int64)
        xq = r["fwd"][3][p]["a_q"][:, ::2, ::2, :].astype(np.int64)
        dws.append(np.einsum("bhwn,bhwc->nc", gq, xq).astype(np.int32).reshape(-1))
        sgs.append(r["grads"][5][p]["s_g"])
        sas.append(r["fwd"][3][p]["s_a"])
    np.testing.assert_array_equal(r["w_master"][3].reshape(-1), O.update(W[3], dws, sgs, sas, wl.lr, 2 * B).reshape(-1))
    # a projection has no loss or goodness of its own and adds nothing to the look-ahead sums
    assert np.all(r["loss"][3] == 0) and np.all(r["goodness"][3] == 0)
    c = np.stack([r["fwd"][i][0]["c"] for i in range(len(L))])
    np.testing.assert_array_equal(r["grads"][2][0]["ctil"], O.lookahead(c, wl.lam)[2])
    assert np.all(c[3] == 0)


def test_zero_second_convolution_passes_the_block_input_through():
    wl = workload("tiny_res")
    W = [w.copy() for w in make_weights(wl)]
    W[2][...] = 0
    r = _run(wl, W)
    for p in range(2):
        f = r["fwd"]
        xhat = O.dequantize(f[1][p]["a_q"], f[1][p]["s_a"])
        np.testing.assert_array_equal(f[2][p]["y"], np.maximum(xhat, 0))
        np.testing.assert_array_equal(f[2][p]["G"], O.goodness_fx(np.maximum(xhat, 0))["G"])


def test_masked_block_output_layer_and_its_projection_are_layer_local():
    wl = workload("tiny_res")
    W = make_weights(wl)
    full = _run(wl, W, lam=0.0)
    part = _run(wl, W, mask=[0, 0, 0, 1, 0, 1], lam=0.0)
    for i in range(6):
        if i in (3, 5):
            np.testing.assert_array_equal(part["w_master"][i], full["w_master"][i])
            assert np.any(part["w_master"][i] != W[i])
        else:
            np.testing.assert_array_equal(part["w_master"][i], W[i])
