"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test names the passage it pins.  None of them re-types the oracle's own formula
and calls that a check: they use closed forms, invariants, brute force in Python
integers, library routines on special cases and fp64 finite differences.
"""
import math

import numpy as np
import pytest

from oracle import ff_oracle as O


# ----------------------------------------------------------------------------- quantiser
def test_quantize_extremes_and_grid_points():
    """Section IV (symmetric uniform quantiser): |x| = amax -> +-127, 0 -> 0, and values
    already on the grid are unchanged in both rounding modes."""
    codes = np.array([-127, -64, -1, 0, 1, 5, 100, 127], dtype=np.float32)
    x = codes * np.float32(0.5)          # amax = 63.5, scale = 0.5 exactly
    for mode in (O.ROUND_NEAREST, O.ROUND_STOCHASTIC):
        for seed in range(20):
            q, s = O.quantize(x, mode, seed, 7)
            assert s == np.float32(0.5)
            assert q.tolist() == codes.astype(int).tolist()


def test_quantize_all_zero():
    q, s = O.quantize(np.zeros((3, 5), np.float32), O.ROUND_STOCHASTIC, 1, 2)
    assert s == np.float32(1.0) and not q.any()


def test_quantize_vanishing_range():
    """Reading R-Q0: absmax below 2^-100 quantises to zero codes with scale 1; just above it the
    ordinary rule applies and the reciprocal scale is still finite."""
    tiny = np.array([1e-38, -2.7e-37, 0.0, 5e-31], np.float32)
    for mode in (O.ROUND_NEAREST, O.ROUND_STOCHASTIC):
        q, s = O.quantize(tiny, mode, 1, 1)
        assert s == np.float32(1.0) and not q.any()
    ok = np.array([2.0 ** -99, -(2.0 ** -100), 0.0], np.float32)
    q, s = O.quantize(ok, O.ROUND_NEAREST)
    assert q.tolist() == [127, -64, 0] and s == np.float32(2.0 ** -99) / np.float32(127)


def test_quantize_nearest_matches_numpy_rint():
    """Special case that reduces to a library routine: round-to-nearest-even."""
    rng = np.random.default_rng(0)
    x = rng.standard_normal(4099).astype(np.float32) * 3
    q, s = O.quantize(x, O.ROUND_NEAREST)
    amax = np.abs(x).max()
    inv = np.float32(127.0) / amax
    ref = np.clip(np.rint(x * inv), -127, 127).astype(np.int8)
    assert s == amax / np.float32(127.0)
    assert np.array_equal(q, ref)
    # ties go to even
    xt = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 127.0], np.float32)
    qt, st = O.quantize(xt, O.ROUND_NEAREST)
    assert st == 1.0 and qt.tolist() == [0, 2, 2, 0, -2, 127]


def test_quantize_roundtrip_bounds():
    """Round trip: |x - s q| <= s/2 (nearest), < s (stochastic); never -128."""
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(20000) * rng.uniform(0.01, 50)).astype(np.float32)
    qn, s = O.quantize(x, O.ROUND_NEAREST)
    err = np.abs(x.astype(np.float64) - O.dequantize(qn, s).astype(np.float64))
    assert err.max() <= 0.5 * float(s) * (1 + 1e-5)
    qs, s2 = O.quantize(x, O.ROUND_STOCHASTIC, 11, 3)
    assert s2 == s
    err = np.abs(x.astype(np.float64) - O.dequantize(qs, s).astype(np.float64))
    assert err.max() < float(s) * (1 + 1e-5)
    assert qn.min() >= -127 and qs.min() >= -127
    # stochastic result is always one of the two neighbouring codes
    t = x.astype(np.float64) * 127.0 / float(np.abs(x).max())
    assert np.all((qs >= np.floor(t) - 1e-3) & (qs <= np.ceil(t) + 1e-3))


def test_stochastic_rounding_unbiased():
    """Stochastic rounding (cited in Section IV-B) is unbiased: the mean of s*q over many
    seeds approaches x within 4 sigma / sqrt(n)."""
    x = np.array([0.1, -0.37, 0.5, 0.93, -0.999, 0.004, 1.0], np.float32)  # amax 1 -> scale 1/127
    n = 12000
    acc = np.zeros(x.size, np.float64)
    for seed in range(n):
        q, s = O.quantize(x, O.ROUND_STOCHASTIC, seed, 5)
        acc += q.astype(np.float64) * float(s)
    mean = acc / n
    t = x.astype(np.float64) * 127
    frac = t - np.floor(t)
    sigma = np.sqrt(frac * (1 - frac)) / 127
    assert np.all(np.abs(mean - x) <= 4 * sigma / math.sqrt(n) + 1e-7)


def test_uniform_stream_is_uniform_and_streams_differ():
    """chi-square of u over 64 bins for consecutive indices; different tags / seeds differ."""
    n = 1 << 16
    u = np.array([O.uniform(3, 9, i) for i in range(n)])
    assert u.min() >= 0.0 and u.max() < 1.0
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((hist - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 120.0          # 63 dof: P(chi2 > 120) ~ 2e-5
    # lag-1 correlation
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.02
    v = np.array([O.uniform(3, 10, i) for i in range(4096)])
    w = np.array([O.uniform(4, 9, i) for i in range(4096)])
    assert abs(np.corrcoef(u[:4096], v)[0, 1]) < 0.06 and abs(np.corrcoef(u[:4096], w)[0, 1]) < 0.06
    # indices beyond 2^32 do not alias the low ones
    hi = np.array([O.uniform(3, 9, (1 << 32) + i) for i in range(4096)])
    assert abs(np.corrcoef(u[:4096], hi)[0, 1]) < 0.06 and not np.array_equal(u[:4096], hi)


def test_hash_golden_values():
    """Stored words of the generator (tests/golden/hash_words.txt, written by
    tests/golden/make_golden.py from the oracle alone) guard against silent edits."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "hash_words.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        seed, tag, idx, h = (int(t, 0) for t in line.split())
        assert O.hash_u32(seed, tag, idx) == h


# ----------------------------------------------------------------------------- contractions
def test_dense_forward_brute_force():
    """Section IV-B: int8 inputs, int32 accumulation.  Python-integer triple loop."""
    rng = np.random.default_rng(2)
    M, K, N = 5, 7, 6
    a = rng.integers(-127, 128, (M, K)).astype(np.int8)
    w = rng.integers(-127, 128, (N, K)).astype(np.int8)
    acc = O.dense_forward(a, w)
    for m in range(M):
        for n in range(N):
            assert acc[m, n] == sum(int(a[m, k]) * int(w[n, k]) for k in range(K))


def test_dense_forward_extremes_identity_and_numpy():
    K = 300
    a = np.full((2, K), 127, np.int8)
    w = np.stack([np.full(K, 127, np.int8), np.full(K, -127, np.int8)])
    acc = O.dense_forward(a, w)
    assert acc.tolist() == [[K * 16129, -K * 16129]] * 2
    eye = np.eye(16, dtype=np.int8)
    rng = np.random.default_rng(3)
    a = rng.integers(-127, 128, (9, 16)).astype(np.int8)
    assert np.array_equal(O.dense_forward(a, eye), a.astype(np.int32))
    w = rng.integers(-127, 128, (33, 16)).astype(np.int8)
    assert np.array_equal(O.dense_forward(a, w), a.astype(np.int32) @ w.astype(np.int32).T)


def test_dense_wgrad_brute_force_and_numpy():
    """dw[n][k] = sum_m gy[m][n] a[m][k]; a transposed operand would fail here (M != N != K)."""
    rng = np.random.default_rng(4)
    M, K, N = 6, 5, 4
    g = rng.integers(-127, 128, (M, N)).astype(np.int8)
    a = rng.integers(-127, 128, (M, K)).astype(np.int8)
    dw = O.dense_wgrad(g, a)
    assert dw.shape == (N, K)
    for n in range(N):
        for k in range(K):
            assert dw[n, k] == sum(int(g[m, n]) * int(a[m, k]) for m in range(M))
    g = rng.integers(-127, 128, (50, 17)).astype(np.int8)
    a = rng.integers(-127, 128, (50, 23)).astype(np.int8)
    assert np.array_equal(O.dense_wgrad(g, a), g.astype(np.int32).T @ a.astype(np.int32))


def test_int32_overflow_is_reported():
    K = O.INT32_SAFE_ROWS + 1
    a = np.full((1, K), 127, np.int8)
    with pytest.raises(O.OracleError):
        O.dense_forward(a, a.copy())
    ok = np.full((1, O.INT32_SAFE_ROWS), 127, np.int8)
    assert O.dense_forward(ok, ok.copy())[0, 0] == O.INT32_SAFE_ROWS * 16129


def test_batch_chunks_cover_the_batch_and_fit_int32():
    """Section IV-B (INT32 accumulation), reading R-CK: a weight-gradient reduction over more rows than
    floor((2^31 - 1) / 127^2) = 133144 is cut into blocks of samples, each block with its own int32
    accumulator.  Pinned here: the bound itself (worst-case codes of +-127 just fit, one more row does not),
    the exact lists for the conv configurations, and for a sweep of shapes that the blocks are disjoint,
    cover [0, B) in order, stay within the bound and have a power-of-two size (except the last)."""
    assert O.INT32_SAFE_ROWS == 133144
    assert O.INT32_SAFE_ROWS * 127 * 127 <= 2**31 - 1 < (O.INT32_SAFE_ROWS + 1) * 127 * 127
    assert O.batch_chunks(256, 32 * 32) == [(0, 128), (128, 256)]          # cfg3, cfg4 stage 1
    assert O.batch_chunks(140, 32 * 32) == [(0, 128), (128, 140)]          # ragged last block
    assert O.batch_chunks(256, 16 * 16) == [(0, 256)]                      # 65536 rows fit one accumulator
    assert O.batch_chunks(8192, 1) == [(0, 8192)]                          # every dense configuration
    assert O.batch_chunks(0, 1024) == [(0, 0)]
    assert O.batch_chunks(133144, 1) == [(0, 133144)]
    assert O.batch_chunks(133145, 1) == [(0, 131072), (131072, 133145)]
    with pytest.raises(O.OracleError):
        O.batch_chunks(2, O.INT32_SAFE_ROWS + 1)                           # one sample alone is too long
    rng = np.random.default_rng(7)
    for _ in range(300):
        rps = int(rng.integers(1, 70000))
        B = int(rng.integers(1, 5000))
        ch = O.batch_chunks(B, rps)
        assert ch[0][0] == 0 and ch[-1][1] == B
        for (a0, a1), (b0, b1) in zip(ch, ch[1:]):
            assert a1 == b0
        for b0, b1 in ch:
            assert b0 < b1 and (b1 - b0) * rps <= O.INT32_SAFE_ROWS
        if len(ch) > 1:
            per = ch[0][1] - ch[0][0]
            assert per & (per - 1) == 0 and 2 * per * rps > O.INT32_SAFE_ROWS   # the largest power of two that fits
            assert all(b1 - b0 == per for b0, b1 in ch[:-1])


def test_chunked_weight_gradient_sums_to_the_unchunked_one():
    """Blocks of samples are a partition of the reduction: their int32 accumulators add up (in exact
    integer arithmetic) to the accumulator of the whole batch whenever that one exists."""
    rng = np.random.default_rng(11)
    B, H, W, Ci, Co = 5, 4, 6, 3, 4
    a = rng.integers(-127, 128, (B, H, W, Ci)).astype(np.int8)
    g = rng.integers(-127, 128, (B, H, W, Co)).astype(np.int8)
    whole = O.conv_wgrad(g, a, 3, 1, 1, 0, B).astype(np.int64)
    parts = sum(O.conv_wgrad(g, a, 3, 1, 1, b0, b1).astype(np.int64) for b0, b1 in [(0, 2), (2, 4), (4, 5)])
    assert np.array_equal(whole, parts)


def _im2col(a, ks, stride, pad):
    B, H, W, C = a.shape
    Ho = (H + 2 * pad - ks) // stride + 1
    Wo = (W + 2 * pad - ks) // stride + 1
    ap = np.zeros((B, H + 2 * pad, W + 2 * pad, C), a.dtype)
    ap[:, pad:pad + H, pad:pad + W] = a
    cols = np.empty((B, Ho, Wo, ks, ks, C), a.dtype)
    for kh in range(ks):
        for kw in range(ks):
            cols[:, :, :, kh, kw] = ap[:, kh:kh + stride * Ho:stride, kw:kw + stride * Wo:stride]
    return cols.reshape(B * Ho * Wo, ks * ks * C), Ho, Wo


@pytest.mark.parametrize("ks,stride,pad,H,W", [(3, 1, 1, 6, 5), (3, 2, 1, 7, 8), (1, 2, 0, 6, 6), (1, 1, 0, 4, 3)])
def test_conv_forward_equals_im2col_matmul(ks, stride, pad, H, W):
    """Direct convolution == explicit im2col + library integer matmul (stride 1 and 2, 3x3 and 1x1);
    output size ceil(H/stride) with pad = ks//2."""
    rng = np.random.default_rng(5)
    B, Cin, Cout = 3, 5, 7
    a = rng.integers(-127, 128, (B, H, W, Cin)).astype(np.int8)
    w = rng.integers(-127, 128, (Cout, ks, ks, Cin)).astype(np.int8)
    acc = O.conv_forward(a, w, stride, pad)
    cols, Ho, Wo = _im2col(a, ks, stride, pad)
    assert (Ho, Wo) == (-(-H // stride), -(-W // stride))
    ref = cols.astype(np.int32) @ w.reshape(Cout, -1).astype(np.int32).T
    assert np.array_equal(acc.reshape(-1, Cout), ref)


def test_conv_1x1_is_dense_and_padding_counts():
    rng = np.random.default_rng(6)
    a = rng.integers(-127, 128, (2, 4, 4, 8)).astype(np.int8)
    w = rng.integers(-127, 128, (5, 1, 1, 8)).astype(np.int8)
    assert np.array_equal(O.conv_forward(a, w, 1, 0).reshape(-1, 5),
                          O.dense_forward(a.reshape(-1, 8), w.reshape(5, 8)))
    # constant image x all-ones 3x3 kernel: interior 9*Cin*a*w, edges 6, corners 4 taps
    Cin, av, wv = 3, 2, 5
    img = np.full((1, 5, 6, Cin), av, np.int8)
    ker = np.full((1, 3, 3, Cin), wv, np.int8)
    out = O.conv_forward(img, ker, 1, 1)[0, :, :, 0]
    unit = Cin * av * wv
    assert out[2, 3] == 9 * unit and out[0, 2] == 6 * unit and out[3, 0] == 6 * unit
    assert out[0, 0] == out[4, 5] == out[0, 5] == out[4, 0] == 4 * unit


@pytest.mark.parametrize("ks,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 2, 0)])
def test_conv_wgrad_equals_im2col_matmul_and_chunks_add(ks, stride, pad):
    rng = np.random.default_rng(7)
    B, H, W, Cin, Cout = 4, 6, 7, 3, 5
    a = rng.integers(-127, 128, (B, H, W, Cin)).astype(np.int8)
    cols, Ho, Wo = _im2col(a, ks, stride, pad)
    g = rng.integers(-127, 128, (B, Ho, Wo, Cout)).astype(np.int8)
    dw = O.conv_wgrad(g, a, ks, stride, pad, 0, B)
    ref = g.reshape(-1, Cout).astype(np.int32).T @ cols.astype(np.int32)
    assert np.array_equal(dw.reshape(Cout, -1), ref)
    parts = O.conv_wgrad(g, a, ks, stride, pad, 0, 1) + O.conv_wgrad(g, a, ks, stride, pad, 1, B)
    assert np.array_equal(parts, dw)


# ----------------------------------------------------------------------------- goodness / loss
def test_goodness_closed_forms():
    """Section III / Algorithm 1: G = ||y||^2.  (1,2,3) -> 14; ones(n) -> n; ReLU drops negatives."""
    acc = np.array([[1, 2, 3], [1, 1, 1], [-4, 2, -1]], np.int32)
    g = O.goodness(acc, 1, 0, 1.0, 1.0)
    assert g["G"].tolist() == [14.0, 3.0, 4.0] and g["g_int"].tolist() == [14, 3, 4]
    assert g["vmax"].tolist() == [3, 1, 2]
    g = O.goodness(acc, 0, 0, 1.0, 1.0)
    assert g["G"].tolist() == [14.0, 3.0, 21.0] and g["vmax"].tolist() == [3, 1, 4]
    g = O.goodness(acc, 1, 0, 0.5, 0.25)          # s_y = 1/8 -> G / 64
    assert g["G"].tolist() == [14 / 64, 3 / 64, 4 / 64]


def test_goodness_integer_path_matches_plain_sum():
    rng = np.random.default_rng(8)
    K, N = 4096, 4096
    acc = rng.integers(-K * 3000, K * 3000, (4, N)).astype(np.int32)
    for r in (0, 3):
        g = O.goodness(acc, 1, r, 0.0123, 0.00071)
        assert np.all(np.abs(g["G"].astype(np.float64) - g["G_plain"]) <= 1e-6 * g["G_plain"])
    # independent fp64 numpy statement of the definition
    y = np.maximum(acc.astype(np.float64) * float(np.float32(0.0123) * np.float32(0.00071)), 0)
    assert np.allclose(g["G_plain"], (y * y).sum(1), rtol=1e-6)


def test_goodness_shift_bound():
    """r is the smallest shift that keeps the worst-case sum below 2^64 (Python big integers)."""
    for K, terms in [(784, 500), (4096, 4096), (27, 65536), (576, 131072), (1152, 262144), (4608, 8192)]:
        r = O.goodness_shift(K, terms)
        worst = (16129 * K) ** 2 * terms
        assert (worst >> r) < 2 ** 64 and (r == 0 or (worst >> (r - 1)) >= 2 ** 64)
    assert O.goodness_shift(4096, 4096) == 0 and O.goodness_shift(1152, 262144) == 3


def test_loss_closed_forms():
    """Eq. (1)/(2): at G = theta both losses are ln 2 and dL/dG = -+1/2;
    L_neg - L_pos = G - theta;  L_pos(G) = L_neg(2 theta - G);  sigma(x) + sigma(-x) = 1."""
    theta = 2.0
    cp, lp, mp = O.loss_coeff(np.array([theta], np.float32), O.PASS_POS, theta)
    cn, ln, mn = O.loss_coeff(np.array([theta], np.float32), O.PASS_NEG, theta)
    assert abs(mp - math.log(2)) < 1e-12 and abs(mn - math.log(2)) < 1e-12
    assert cp[0] == -0.5 and cn[0] == 0.5
    G = np.array([0.0, 0.3, 1.5, 2.25, 3.0, 7.5, 40.0, 200.0], np.float32)
    cp, lp, _ = O.loss_coeff(G, O.PASS_POS, theta)
    cn, ln, _ = O.loss_coeff(G, O.PASS_NEG, theta)
    assert np.allclose(ln.astype(np.float64) - lp, G - theta, atol=2e-6 * np.maximum(1, G))
    _, lmirror, _ = O.loss_coeff((2 * theta - G).astype(np.float32), O.PASS_NEG, theta)
    assert np.allclose(lp, lmirror, rtol=1e-6, atol=1e-30)
    assert np.all(np.abs((cn - cp) - 1.0) <= 2 * np.finfo(np.float32).eps)
    # signs: more goodness lowers the positive loss and raises the negative one
    assert np.all(cp <= 0) and np.all(cn >= 0)
    # against the textbook sigmoid in fp64
    xd = G.astype(np.float64) - theta
    assert np.allclose(cn, 1 / (1 + np.exp(-xd)), rtol=3e-7, atol=0)
    assert np.allclose(-cp, 1 / (1 + np.exp(xd)), rtol=3e-7, atol=2e-38)   # exp argument clamps at -87
    # large |x| limits
    c, l, _ = O.loss_coeff(np.array([1e4], np.float32), O.PASS_POS, theta)
    assert -1e-37 <= c[0] <= 0 and l[0] == 0
    c, l, _ = O.loss_coeff(np.array([1e4], np.float32), O.PASS_NEG, theta)
    assert c[0] == 1.0 and abs(l[0] - (1e4 - 2)) < 1e-2
    # derivative of the printed loss by fp64 central differences
    for sign, cc in ((O.PASS_POS, cp), (O.PASS_NEG, cn)):
        f = lambda g: math.log1p(math.exp(-sign * (g - theta)))
        for gi, ci in zip(G[:6], cc[:6]):
            fd = (f(float(gi) + 1e-5) - f(float(gi) - 1e-5)) / 2e-5
            assert abs(fd - ci) < 1e-6


def test_exp_spec_against_libm():
    z = -np.concatenate([np.linspace(0, 87, 20001), np.geomspace(1e-8, 87, 5000)]).astype(np.float32)
    mine = np.array([O.exp_spec(v) for v in z], np.float32)
    ref64 = np.exp(z.astype(np.float64))
    ulp = np.spacing(ref64.astype(np.float32)).astype(np.float64)
    assert np.max(np.abs(mine.astype(np.float64) - ref64) / ulp) <= 2.0
    assert O.exp_spec(0.0) == 1.0 and O.exp_spec(-1000.0) == O.exp_spec(-87.0) > 0


# ----------------------------------------------------------------------------- look-ahead
def test_lookahead_hand_example_and_lambda_zero():
    """Eq. (3)/(4): layer i sees its own coefficient plus lambda times the sum of the later
    layers' coefficients.  k = 3, values chosen exactly representable."""
    c = np.array([[0.5, -0.25], [0.125, 0.5], [-0.75, 0.25]], np.float32)   # [k, B]
    out = O.lookahead(c, 0.5)
    assert out.tolist() == [[0.5 + 0.5 * (0.125 - 0.75), -0.25 + 0.5 * (0.5 + 0.25)],
                            [0.125 + 0.5 * -0.75, 0.5 + 0.5 * 0.25],
                            [-0.75, 0.25]]
    rng = np.random.default_rng(9)
    c = rng.standard_normal((5, 33)).astype(np.float32)
    assert np.array_equal(O.lookahead(c, 0.0), c)               # lambda = 0 is the vanilla method, bitwise
    assert np.array_equal(O.lookahead(c, 0.3)[-1], c[-1])       # last layer has nothing ahead


# ----------------------------------------------------------------------------- local gradient
def _loss_fp64(W, A, sign, theta):
    y = np.maximum(A @ W.T, 0.0)
    G = (y * y).sum(1)
    return np.log1p(np.exp(-sign * (G - theta))).sum()


@pytest.mark.parametrize("sign", [O.PASS_POS, O.PASS_NEG])
def test_local_gradient_matches_finite_differences(sign):
    """Section IV-B: g^Y = dL/dY and g^W = g^Y^T A.  Operands sit exactly on the int8 grid so that
    the only approximation left is fp32 rounding: the oracle's fp32 g^Y contracted with A in fp64
    must equal central differences of the printed loss w.r.t. W (sign, factor 2 and ReLU mask)."""
    rng = np.random.default_rng(10)
    B, K, N = 5, 6, 4
    a_q = rng.integers(-127, 128, (B, K)).astype(np.int8)
    w_q = rng.integers(-127, 128, (N, K)).astype(np.int8)
    s_a, s_w = np.float32(1 / 256), np.float32(1 / 512)
    A = a_q.astype(np.float64) * float(s_a)
    W = w_q.astype(np.float64) * float(s_w)
    theta = 2.0
    acc = O.dense_forward(a_q, w_q)
    gd = O.goodness(acc, 1, 0, s_a, s_w)
    c, _, _ = O.loss_coeff(gd["G"], sign, theta)
    g = O.local_grad(acc, 1, s_a, s_w, c)
    dW = g.astype(np.float64).T @ A
    fd = np.zeros_like(W)
    h = 1e-6
    for n in range(N):
        for k in range(K):
            Wp, Wm = W.copy(), W.copy()
            Wp[n, k] += h
            Wm[n, k] -= h
            fd[n, k] = (_loss_fp64(Wp, A, sign, theta) - _loss_fp64(Wm, A, sign, theta)) / (2 * h)
    assert np.allclose(dW, fd, rtol=2e-5, atol=1e-7)
    assert np.abs(fd).max() > 1e-3            # the case is not degenerate


def test_quantized_gradient_within_error_bound_and_step_moves_goodness():
    """The int8 route s_g s_A dWacc stays within the quantisation error bound of the fp64 gradient,
    and one small SGD step raises mean G_pos and lowers mean G_neg (Section III)."""
    from workloads import workload, make_inputs, make_weights
    wl = workload("tiny")
    layers = wl.layers[:1]
    W0 = make_weights(wl)[:1]
    xp, xn = make_inputs(wl)
    theta = 21.0      # close to the initial goodness of this layer, so both passes have a live gradient
    res = O.train_step(layers, W0, xp, xn, theta, 0.0, 0.05, 3, 0)
    for p, (x, sign) in enumerate(((xp, 1), (xn, -1))):
        f, gr = res["fwd"][0][p], res["grads"][0][p]
        A = f["a_q"].astype(np.float64) * float(f["s_a"])
        g = O.local_grad(f["acc"], 1, f["s_a"], res["s_w_in"][0], f["c"]).astype(np.float64)
        exact = g.T @ A
        quant = gr["dw"][0].reshape(exact.shape).astype(np.float64) * float(gr["s_g"]) * float(f["s_a"])
        M = A.shape[0]
        bound = M * float(gr["s_g"]) * (np.abs(A).max() + float(f["s_a"]))
        assert np.abs(exact - quant).max() <= bound
        assert np.abs(exact - quant).max() < 0.2 * np.abs(exact).max()
        # apply this pass's gradient alone and run the layer forward again on the same data
        w1 = O.update(W0[0], [gr["dw"][0]], [gr["s_g"]], [f["s_a"]], lr=0.5, total_samples=2 * M)
        q1, s1 = O.quantize(w1, O.ROUND_NEAREST)
        G1 = O.goodness(O.dense_forward(f["a_q"], q1), 1, 0, f["s_a"], s1)["G"]
        if sign > 0:
            assert G1.mean() > f["G"].mean() * 1.001
        else:
            assert G1.mean() < f["G"].mean() * 0.999


def test_local_grad_absmax_is_rowwise_product():
    """Monotonicity used by the fast path: max |g| == max_b |2 c_b| * fp32(vmax_b) * s_y."""
    rng = np.random.default_rng(11)
    acc = rng.integers(-10 ** 7, 10 ** 7, (9, 40)).astype(np.int32)
    s_a, s_w = np.float32(0.013), np.float32(0.0007)
    c = rng.standard_normal(9).astype(np.float32)
    g = O.local_grad(acc, 1, s_a, s_w, c)
    vmax = O.goodness(acc, 1, 0, s_a, s_w)["vmax"]
    s_y = s_a * s_w
    pred = np.max(np.abs(np.float32(2) * c) * (vmax.astype(np.float32) * s_y))
    assert np.float32(np.abs(g).max()) == np.float32(pred)


# ----------------------------------------------------------------------------- hand-off / update
def test_handoff_l2norm_unit_length_and_zero_row():
    acc = np.array([[3, -5, 4], [0, -1, 0]], np.int32)
    G = O.goodness(acc, 1, 0, 1.0, 1.0)["G"]
    out = O.handoff(acc, 1, 1, 1.0, 1.0, G)
    assert np.allclose(out[0], [0.6, 0.0, 0.8]) and out[1].tolist() == [0, 0, 0]
    assert np.array_equal(O.handoff(acc, 1, 0, 0.5, 1.0, G), np.maximum(acc, 0) * np.float32(0.5))


def test_update_hand_example_and_zero_gradient():
    """Algorithm 1 (weight update), 2x2 example with exactly representable numbers:
    w - lr/B_total * (s_g+ s_a+ dw+ + s_g- s_a- dw-)."""
    w = np.array([[1.0, -2.0], [0.5, 0.25]], np.float32)
    dwp = np.array([4, -8, 16, 0], np.int32)
    dwn = np.array([2, 2, -4, 8], np.int32)
    out = O.update(w, [dwp, dwn], [0.5, 0.25], [0.5, 1.0], lr=0.5, total_samples=4)
    g = 0.25 * dwp + 0.25 * dwn
    assert out.reshape(-1).tolist() == (w.reshape(-1) - 0.125 * g).tolist()
    z = np.zeros(4, np.int32)
    assert np.array_equal(O.update(w, [z, z], [0.3, 0.7], [0.1, 0.2], 0.9, 8), w)


# ----------------------------------------------------------------------------- whole step
def test_train_step_invariants():
    """Algorithm 1: (i) lambda = 0 with look-ahead code path == per-layer vanilla, bitwise;
    (ii) the last layer's update does not depend on lambda; (iii) every layer's update uses
    activations computed with the pre-step weights; (iv) same seeds -> same bytes."""
    from workloads import workload, make_inputs, make_weights
    wl = workload("tiny_l2")
    W0 = make_weights(wl)
    xp, xn = make_inputs(wl)
    a = O.train_step(wl.layers, W0, xp, xn, wl.theta, 0.0, wl.lr, 2, 0)
    b = O.train_step(wl.layers, W0, xp, xn, wl.theta, 0.25, wl.lr, 2, 0)
    c = O.train_step(wl.layers, W0, xp, xn, wl.theta, 0.25, wl.lr, 2, 0)
    k = len(wl.layers)
    assert np.array_equal(a["w_master"][k - 1], b["w_master"][k - 1])
    assert not np.array_equal(a["w_master"][0], b["w_master"][0])
    for i in range(k):
        assert np.array_equal(b["w_master"][i], c["w_master"][i])
        assert np.array_equal(a["fwd"][i][0]["acc"], b["fwd"][i][0]["acc"])     # forward ignores lambda
    # vanilla: layer 0 alone, fed the same input, gives the same layer-0 update as the 4-layer step
    solo = O.train_step(wl.layers[:1], W0[:1], xp, xn, wl.theta, 0.0, wl.lr, 2, 0)
    assert np.array_equal(solo["w_master"][0], a["w_master"][0])
    # l2norm hand-off feeds unit-length rows to the next layer: its int8 input has amax code 127 per
    # tensor and its dequantised rows have length close to one
    f1 = a["fwd"][1][0]
    rows = f1["a_q"].astype(np.float64) * float(f1["s_a"])
    nz = a["fwd"][0][0]["G"] > 0
    assert np.allclose(np.linalg.norm(rows[nz], axis=1), 1.0, atol=0.1)
    assert np.abs(f1["a_q"]).max() == 127
