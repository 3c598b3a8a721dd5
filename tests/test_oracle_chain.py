"""Pins of the oracle's exact-derivative look-ahead (Eq. (4) taken literally: the later layers' losses are
differentiated through those layers).  CPU only."""
import numpy as np
import pytest

import oracle.ff_oracle as O
from workloads import Layer


def test_input_gradient_brute_force_numpy_and_overflow():
    """e[m][k] = sum_n h[m][n] w[n][k]: python loops on a non-square case (a transposed operand or a swapped
    index cannot pass), the library product in 64-bit integers, the extreme codes, and the overflow report."""
    rng = np.random.default_rng(3)
    M, N, K = 3, 5, 4
    h = rng.integers(-127, 128, (M, N)).astype(np.int8)
    w = rng.integers(-127, 128, (N, K)).astype(np.int8)
    e = O.dense_input_grad(h, w)
    assert e.shape == (M, K) and e.dtype == np.int32
    for m in range(M):
        for k in range(K):
            assert int(e[m, k]) == sum(int(h[m, n]) * int(w[n, k]) for n in range(N))
    M, N, K = 17, 70, 33
    h = rng.integers(-127, 128, (M, N)).astype(np.int8)
    w = rng.integers(-127, 128, (N, K)).astype(np.int8)
    assert np.array_equal(O.dense_input_grad(h, w), h.astype(np.int64) @ w.astype(np.int64))
    h = np.full((2, 1000), 127, np.int8)
    w = np.full((1000, 3), -127, np.int8)
    assert np.all(O.dense_input_grad(h, w) == -127 * 127 * 1000)
    n_over = O.INT32_SAFE_ROWS + 1
    with pytest.raises(O.OracleError):
        O.dense_input_grad(np.full((1, n_over), 127, np.int8), np.full((n_over, 1), 127, np.int8))


def test_combination_hand_example_and_reductions():
    """(2 c y + E) and (2 c y + lambda E) under the ReLU mask, worked by hand with exactly representable
    numbers; lambda = 0 and the top layer (no E) reduce to the local gradient bit for bit."""
    acc = np.array([[8, -4, 0, 2], [1, 3, -5, 16]], np.int32)
    s_a, s_w = np.float32(0.5), np.float32(0.25)          # s_y = 1/8
    c = np.array([0.5, -0.25], np.float32)                # d = 1, -0.5
    e_acc = np.array([[4, 100, -8, -2], [6, 0, 64, -8]], np.int32)
    s_e = np.float32(0.5)                                 # E = 2, 50, -4, -1 | 3, 0, 32, -4
    lam = 0.25
    h, g = O.chain_combine(acc, 1, s_a, s_w, c, e_acc, s_e, lam)
    # y = 1, 0, 0, .25 | .125, .375, 0, 2 ;  t = d*y = 1, 0, 0, .25 | -.0625, -.1875, 0, -1
    assert h.tolist() == [[3.0, 0.0, 0.0, -0.75], [2.9375, -0.1875, 0.0, -5.0]]
    assert g.tolist() == [[1.5, 0.0, 0.0, 0.0], [0.6875, -0.1875, 0.0, -2.0]]
    # identity activation: no mask, negative activities pass
    h2, g2 = O.chain_combine(acc, 0, s_a, s_w, c, e_acc, s_e, lam)
    assert h2[0].tolist() == [3.0, 49.5, -4.0, -0.75] and g2[0].tolist() == [1.5, 12.0, -1.0, 0.0]
    rng = np.random.default_rng(5)
    acc = rng.integers(-30000, 30000, (6, 11)).astype(np.int32)
    c = rng.normal(size=6).astype(np.float32)
    e_acc = rng.integers(-5000, 5000, (6, 11)).astype(np.int32)
    local = O.local_grad(acc, 1, 0.01, 0.02, c)
    h0, g0 = O.chain_combine(acc, 1, 0.01, 0.02, c, e_acc, 0.003, 0.0)
    assert np.array_equal(g0, local) and not np.array_equal(h0, local)
    ht, gt = O.chain_combine(acc, 1, 0.01, 0.02, c, None, 0.0, 0.7)
    assert np.array_equal(ht, local) and np.array_equal(gt, local)


def _softplus(x):
    return np.logaddexp(0.0, x)


def _model_losses(Ws, A, sign, theta):
    """fp64, no quantisation: summed-over-samples loss of every layer of a dense ReLU stack (Eq. (1)/(2))."""
    out, a = [], A
    for W in Ws:
        y = np.maximum(a @ W.T, 0.0)
        G = (y * y).sum(axis=1)
        out.append(_softplus(-sign * (G - theta)).sum())
        a = y
    return out


def _fd(fun, W, h=1e-6):
    g = np.zeros_like(W)
    for idx in np.ndindex(*W.shape):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += h
        Wm[idx] -= h
        g[idx] = (fun(Wp) - fun(Wm)) / (2 * h)
    return g


def _stack():
    """Three dense layers whose goodness is close to theta at every level (live coefficients), inputs exactly
    on the int8 grid (x = q/128 with max |q| = 127 quantises without error)."""
    rng = np.random.default_rng(11)
    B, widths, theta = 24, [12, 10, 9, 8], 2.0
    q = rng.integers(-127, 128, (B, widths[0]))
    q[0, 0] = 127
    x = (q / 128.0).astype(np.float32)
    Ws, a = [], np.maximum(x.astype(np.float64), 0) + 0.0
    a = x.astype(np.float64)
    for i in range(3):
        W = rng.normal(size=(widths[i + 1], widths[i]))
        y = np.maximum(a @ W.T, 0)
        W *= np.sqrt(theta / (y * y).sum(axis=1).mean())
        Ws.append(W.astype(np.float32))
        a = np.maximum(a @ Ws[-1].astype(np.float64).T, 0)
    layers = tuple(Layer("dense", in_features=widths[i], out_features=widths[i + 1]) for i in range(3))
    return layers, Ws, x, theta


@pytest.mark.parametrize("sign", [+1, -1])
def test_chain_gradient_matches_finite_differences_of_l_new(sign):
    """dL_new_i/dW_i with L_new_i = L_i + lambda (L_{i+1} + ... + L_k), by central differences on an fp64 model of
    the stack at the dequantised weights, against the oracle's int8 route s_g s_A dWacc.  What separates the two
    is the int8 quantisation of the activations and of the two gradients (about 1 % each); the look-ahead term
    itself is several times larger than the tolerance, so a dropped, negated, lambda-compounded or unmasked term
    fails, and so does the coefficient reading of the default step (checked below)."""
    layers, Ws, x, theta = _stack()
    lam = 0.8
    p = 0 if sign > 0 else 1
    res = O.train_step_chain(layers, Ws, x, x, theta, lam, 0.01, seed=4, step=0)
    Wd = [res["w_q_in"][i].astype(np.float64) * float(res["s_w_in"][i]) for i in range(3)]
    A = x.astype(np.float64)
    ref = O.train_step(layers, Ws, x, x, theta, lam, 0.01, seed=4, step=0)
    for i in range(3):
        def l_new(Wi, i=i):
            L = _model_losses(Wd[:i] + [Wi] + Wd[i + 1:], A, sign, theta)
            return L[i] + lam * sum(L[i + 1:])

        def l_own(Wi, i=i):
            return _model_losses(Wd[:i] + [Wi] + Wd[i + 1:], A, sign, theta)[i]

        fd = _fd(l_new, Wd[i])
        fd_own = _fd(l_own, Wd[i])
        gr, f = res["grads"][i][p], res["fwd"][i][p]
        got = gr["dw"][0].reshape(fd.shape).astype(np.float64) * float(gr["s_g"]) * float(f["s_a"])
        scale = np.abs(fd).max()
        assert scale > 1e-2
        assert np.abs(got - fd).max() < 0.06 * scale, (i, np.abs(got - fd).max() / scale)
        if i < 2:
            ahead = np.abs(fd - fd_own).max()
            assert ahead > 0.3 * scale                     # the look-ahead term is not a detail of this case
            assert np.abs(got - fd_own).max() > 0.2 * scale  # ... and leaving it out would be seen
            r2 = ref["grads"][i][p]
            got_r2 = r2["dw"][0].reshape(fd.shape).astype(np.float64) * float(r2["s_g"]) * float(ref["fwd"][i][p]["s_a"])
            assert np.abs(got_r2 - fd).max() > 0.2 * scale   # the coefficient reading is a different quantity


def test_chain_step_reductions():
    """lambda = 0: the step equals the default step bit for bit.  Any lambda: the last layer has nothing ahead of
    it and is updated exactly as in the default step.  A frozen layer still hands its gradient down."""
    layers, Ws, x, theta = _stack()
    xn = np.roll(x, 1, axis=0)
    a = O.train_step_chain(layers, Ws, x, xn, theta, 0.0, 0.05, 7, 3)
    b = O.train_step(layers, Ws, x, xn, theta, 0.0, 0.05, 7, 3)
    for i in range(3):
        assert np.array_equal(a["w_master"][i], b["w_master"][i])
        assert np.array_equal(a["w_q"][i], b["w_q"][i])
    a = O.train_step_chain(layers, Ws, x, xn, theta, 0.6, 0.05, 7, 3)
    b = O.train_step(layers, Ws, x, xn, theta, 0.6, 0.05, 7, 3)
    assert np.array_equal(a["w_master"][2], b["w_master"][2])
    assert not np.array_equal(a["w_master"][0], b["w_master"][0])
    assert np.array_equal(a["loss"], b["loss"]) and np.array_equal(a["goodness"], b["goodness"])
    m = O.train_step_chain(layers, Ws, x, xn, theta, 0.6, 0.05, 7, 3, train_mask=[1, 0, 1])
    assert np.array_equal(m["w_master"][1], Ws[1])
    assert np.array_equal(m["w_master"][0], a["w_master"][0]) and np.array_equal(m["w_master"][2], a["w_master"][2])
    with pytest.raises(O.OracleError):
        O.train_step_chain((Layer("dense", in_features=12, out_features=10, l2norm_out=1),), Ws[:1], x, xn, theta, 0.1, 0.05, 7, 3)
