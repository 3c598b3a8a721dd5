"""Training schedules: the frozen-layer flag of the step, the greedy schedule of Section III and the
look-ahead schedule with the lambda ramp of Section V-A.

CPU part: properties of the oracle step that the paper's method fixes (layer-local updates), and the
sanity signal of a short synthetic run (the goodness of positive data rises above that of negative data).
GPU part: the library's schedules against the same loops written over the oracle, bit for bit."""
import numpy as np
import pytest

from oracle import ff_oracle as O
from workloads import make_inputs, make_weights, workload


def _oracle_greedy(wl, W, xp, xn, epochs_per_layer, step0=0):
    """Section III written over the oracle: layer i is trained on the prefix stack with layers < i frozen."""
    step, W = step0, list(W)
    for i in range(len(wl.layers)):
        mask = [0] * i + [1]
        for _ in range(epochs_per_layer):
            r = O.train_step(wl.layers[:i + 1], W[:i + 1], xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, step,
                             keep=False, train_mask=mask)
            W[:i + 1] = r["w_master"]
            step += 1
    return W


def _oracle_lookahead(wl, W, xp, xn, epochs, lam0, dlam, step0=0):
    step, lam, W = step0, lam0, list(W)
    for _ in range(epochs):
        r = O.train_step(wl.layers, W, xp, xn, wl.theta, lam, wl.lr, wl.sr_seed, step, keep=False)
        W = r["w_master"]
        step += 1
        lam += dlam
    return W, r


# ------------------------------------------------------------------------------------------- CPU: oracle properties
def test_frozen_layers_keep_their_weights_and_updates_are_layer_local():
    """With lambda = 0 the update of layer i depends on nothing but layer i's own goodness (Section III; no
    gradient crosses a layer boundary, Section IV-B): training only layer i must give layer i exactly the weights
    that the all-layers step gives it, and leave the others bit-identical to their inputs."""
    wl = workload("tiny_l2")
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    full = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, 5, keep=False)
    k = len(wl.layers)
    assert k >= 2
    for i in range(k):
        mask = [int(j == i) for j in range(k)]
        part = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, 5, keep=False, train_mask=mask)
        for j in range(k):
            if j == i:
                np.testing.assert_array_equal(part["w_master"][j], full["w_master"][j])
                assert np.any(part["w_master"][j] != W[j])
            else:
                np.testing.assert_array_equal(part["w_master"][j], W[j])
        np.testing.assert_array_equal(part["goodness"], full["goodness"])   # the forward pass is the same


def test_lookahead_reaches_earlier_layers_only():
    """Eq. (3)/(4): with lambda > 0 the coefficient of layer i gains the terms of layers j > i, so the last
    layer's update does not depend on lambda while the first layer's does."""
    wl = workload("tiny_l2")
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    a = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.0, wl.lr, wl.sr_seed, 0, keep=False)
    b = O.train_step(wl.layers, W, xp, xn, wl.theta, 0.3, wl.lr, wl.sr_seed, 0, keep=False)
    np.testing.assert_array_equal(a["w_master"][-1], b["w_master"][-1])
    assert np.any(a["w_master"][0] != b["w_master"][0])


def test_short_greedy_run_separates_positive_from_negative_goodness():
    """Sanity signal of Section III on synthetic label-overlay data: after sixty iterations on one batch the
    first layer's mean goodness of the positive set exceeds that of the negative set by more than at the start,
    and its summed loss has dropped."""
    wl = workload("tiny")
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    r0 = O.train_step(wl.layers[:1], W[:1], xp, xn, wl.theta, 0.0, 0.0, wl.sr_seed, 0, keep=False)
    Wt = W[:1]
    lr = 0.1
    for step in range(60):
        r = O.train_step(wl.layers[:1], Wt, xp, xn, wl.theta, 0.0, lr, wl.sr_seed, step, keep=False)
        Wt = r["w_master"]
    r1 = O.train_step(wl.layers[:1], Wt, xp, xn, wl.theta, 0.0, 0.0, wl.sr_seed, 99, keep=False)
    sep0 = r0["goodness"][0][0].mean() - r0["goodness"][0][1].mean()
    sep1 = r1["goodness"][0][0].mean() - r1["goodness"][0][1].mean()
    assert sep1 > sep0 + 0.5, (sep0, sep1)
    assert r1["loss"][0].sum() < 0.2 * r0["loss"][0].sum()
    # the threshold ends up between the two sets (Eq. (1)/(2) push positive goodness above theta, negative below)
    assert r1["goodness"][0][0].mean() > wl.theta > r1["goodness"][0][1].mean()


# ------------------------------------------------------------------------------------------- GPU: library schedules
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ff():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_22771_amd as m
    m.lib()
    return m


def _state(ff, wl):
    from paper_2506_22771_amd import schedule
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    st = schedule.TrainState.from_weights(wl.layers, wl.batch, W)
    B = wl.batch
    batch = (torch.from_numpy(xp.reshape(B, -1)).cuda(), torch.from_numpy(xn.reshape(B, -1)).cuda())
    return schedule, st, W, xp, xn, batch


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["tiny_l2", "tiny_conv16"])
def test_masked_step_matches_oracle(ff, name):
    wl = workload(name)
    schedule, st, W, xp, xn, batch = _state(ff, wl)
    k = len(wl.layers)
    mask = [int(i == k - 1) for i in range(k)]
    net = st.net(k, mask)
    ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    loss = torch.empty((k, 2), device="cuda")
    good = torch.empty((k, 2, wl.batch), device="cuda")
    ff.ff_train_step(net, batch[0], batch[1], wl.theta, wl.lam, wl.lr, wl.sr_seed, 3, loss, good, ws)
    torch.cuda.synchronize()
    ref = O.train_step(wl.layers, W, xp, xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, 3, keep=False, train_mask=mask)
    for i in range(k):
        np.testing.assert_array_equal(st.w_master[i].cpu().numpy().reshape(-1), ref["w_master"][i].reshape(-1))
        assert st.s_w[i].item() == ref["s_w"][i]
    np.testing.assert_allclose(good.cpu().numpy(), ref["goodness"], rtol=1e-5)


@pytest.mark.gpu
def test_masked_chain_step_and_lambda_ramp_match_oracle(ff):
    """The exact-derivative look-ahead with a frozen middle layer (its gradient still reaches the layer below), then
    the lambda ramp over it, bit for bit against the oracle's loop."""
    from workloads import Workload, mlp
    wl = Workload("tiny3", mlp([60, 44, 36, 28], False), 20, "uniform_onehot", theta=12.0, lam=0.3)
    schedule, st, W, xp, xn, batch = _state(ff, wl)
    k = 3
    mask = [1, 0, 1]
    net = st.net(k, mask, lookahead="chain")
    ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    loss = torch.empty((k, 2), device="cuda")
    good = torch.empty((k, 2, wl.batch), device="cuda")
    ff.ff_train_step(net, batch[0], batch[1], wl.theta, wl.lam, wl.lr, wl.sr_seed, 5, loss, good, ws)
    torch.cuda.synchronize()
    ref = O.train_step_chain(wl.layers, W, xp, xn, wl.theta, wl.lam, wl.lr, wl.sr_seed, 5, keep=False, train_mask=mask)
    for i in range(k):
        np.testing.assert_array_equal(st.w_master[i].cpu().numpy().reshape(-1), ref["w_master"][i].reshape(-1))
        assert st.s_w[i].item() == ref["s_w"][i]
    assert not np.array_equal(ref["w_master"][0], W[0]) and np.array_equal(ref["w_master"][1], W[1])
    Wref = ref["w_master"]
    schedule.train_lookahead(st, [batch], 3, wl.theta, wl.lr, wl.sr_seed, lam0=0.1, dlam=0.2, step0=6, lookahead="chain")
    torch.cuda.synchronize()
    for e in range(3):
        Wref = O.train_step_chain(wl.layers, Wref, xp, xn, wl.theta, 0.1 + 0.2 * e, wl.lr, wl.sr_seed, 6 + e, keep=False)["w_master"]
    for i in range(k):
        np.testing.assert_array_equal(st.w_master[i].cpu().numpy().reshape(-1), Wref[i].reshape(-1))


@pytest.mark.gpu
def test_greedy_schedule_matches_oracle(ff):
    wl = workload("tiny_l2")
    schedule, st, W, xp, xn, batch = _state(ff, wl)
    hist = schedule.train_greedy(st, [batch], 3, wl.theta, wl.lr, wl.sr_seed)
    torch.cuda.synchronize()
    Wref = _oracle_greedy(wl, W, xp, xn, 3)
    for i in range(len(wl.layers)):
        np.testing.assert_array_equal(st.w_master[i].cpu().numpy().reshape(-1), Wref[i].reshape(-1))
    assert len(hist.step) == 3 * len(wl.layers) and hist.step[-1] == 3 * len(wl.layers) - 1


@pytest.mark.gpu
def test_lookahead_schedule_with_lambda_ramp_matches_oracle(ff):
    wl = workload("tiny_l2")
    schedule, st, W, xp, xn, batch = _state(ff, wl)
    hist = schedule.train_lookahead(st, [batch], 4, wl.theta, wl.lr, wl.sr_seed, lam0=0.0, dlam=0.05)
    torch.cuda.synchronize()
    Wref, last = _oracle_lookahead(wl, W, xp, xn, 4, 0.0, 0.05)
    for i in range(len(wl.layers)):
        np.testing.assert_array_equal(st.w_master[i].cpu().numpy().reshape(-1), Wref[i].reshape(-1))
    np.testing.assert_allclose(np.array(hist.loss[-1]), last["loss"], rtol=1e-5)
    assert hist.lam == pytest.approx([0.0, 0.05, 0.10, 0.15])


@pytest.mark.gpu
def test_lookahead_schedule_as_replayed_graphs_equals_eager(ff):
    """Two batches, three epochs with a lambda ramp: one captured graph per epoch, replayed per batch, gives the same
    weights bit for bit and the same logged losses as eagerly launched steps."""
    wl = workload("tiny_l2")
    schedule, st_a, W, xp, xn, batch = _state(ff, wl)
    _, st_b, _, _, _, _ = _state(ff, wl)
    batch2 = (batch[1].clone(), batch[0].clone())
    ha = schedule.train_lookahead(st_a, [batch, batch2], 3, wl.theta, wl.lr, wl.sr_seed, lam0=0.0, dlam=0.1)
    hb = schedule.train_lookahead(st_b, [batch, batch2], 3, wl.theta, wl.lr, wl.sr_seed, lam0=0.0, dlam=0.1, use_graph=True)
    torch.cuda.synchronize()
    for i in range(len(wl.layers)):
        assert torch.equal(st_a.w_master[i], st_b.w_master[i]) and torch.equal(st_a.w_q[i], st_b.w_q[i])
    assert ha.step == hb.step == list(range(6))
    np.testing.assert_allclose(np.array(ha.loss), np.array(hb.loss), rtol=1e-5)
