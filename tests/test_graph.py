"""ff_train_step_at: the step number lives in device memory, so one captured HIP graph serves every iteration.
Checked against eagerly launched ff_train_step on a second copy of the same network: bit-exact weights and
scales, loss and goodness within 1e-5, on every replay, with unrelated eager work and synchronisations between
the replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from workloads import make_inputs, make_weights, workload  # noqa: E402


@pytest.fixture(scope="module")
def ff():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_22771_amd as m
    m.lib()
    return m


def _setup(ff, wl, lookahead="coeff"):
    from paper_2506_22771_amd import schedule
    W = make_weights(wl)
    xp, xn = make_inputs(wl)
    B, k = wl.batch, len(wl.layers)
    st = schedule.TrainState.from_weights(wl.layers, B, W)
    net = st.net(lookahead=lookahead)
    ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    loss = torch.empty((k, 2), device="cuda")
    good = torch.empty((k, 2, B), device="cuda")
    x = (torch.from_numpy(xp.reshape(B, -1)).cuda(), torch.from_numpy(xn.reshape(B, -1)).cuda())
    return st, net, ws, loss, good, x


def _same(a, b, what):
    sa, _, _, la, ga, _ = a
    sb, _, _, lb, gb, _ = b
    for i in range(len(sa.w_master)):
        assert torch.equal(sa.w_master[i], sb.w_master[i]), f"{what}: w_master[{i}]"
        assert torch.equal(sa.w_q[i], sb.w_q[i]), f"{what}: w_q[{i}]"
        assert torch.equal(sa.s_w[i], sb.s_w[i]), f"{what}: s_w[{i}]"
    np.testing.assert_allclose(la.cpu().numpy(), lb.cpu().numpy(), rtol=1e-5, err_msg=what)
    np.testing.assert_allclose(ga.cpu().numpy(), gb.cpu().numpy(), rtol=1e-5, err_msg=what)


@pytest.mark.parametrize("name", ["tiny_l2", "tiny_conv16"])
def test_step_at_equals_step(ff, name):
    wl = workload(name)
    a, b = _setup(ff, wl), _setup(ff, wl)
    step_dev = torch.tensor([5], dtype=torch.int64, device="cuda")
    for s in range(5, 8):
        ff.ff_train_step(a[1], a[5][0], a[5][1], wl.theta, wl.lam, wl.lr, wl.sr_seed, s, a[3], a[4], a[2])
        ff.ff_train_step_at(b[1], b[5][0], b[5][1], wl.theta, wl.lam, wl.lr, wl.sr_seed, step_dev, 1, b[3], b[4], b[2])
        torch.cuda.synchronize()
        _same(a, b, f"{name} step {s}")
    assert int(step_dev.item()) == 8
    # advance = 0 leaves the counter alone
    ff.ff_train_step_at(b[1], b[5][0], b[5][1], wl.theta, wl.lam, wl.lr, wl.sr_seed, step_dev, 0, b[3], b[4], b[2])
    torch.cuda.synchronize()
    assert int(step_dev.item()) == 8


@pytest.mark.parametrize("name", ["tiny_l2", "cfg1", "tiny_conv16", "tiny_res", "tiny/chain"])
def test_captured_graph_replays_match_eager_steps(ff, name):
    name, _, mode = name.partition("/")
    wl = workload(name)
    a, b = _setup(ff, wl, mode or "coeff"), _setup(ff, wl, mode or "coeff")
    step_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ff.ff_train_step_at(b[1], b[5][0], b[5][1], wl.theta, wl.lam, wl.lr, wl.sr_seed, step_dev, 1, b[3], b[4], b[2])
    torch.cuda.synchronize()
    assert int(step_dev.item()) == 0          # capture records, it does not run
    junk = torch.randn(256, 256, device="cuda")
    for s in range(4):
        graph.replay()
        junk = junk @ junk.t() * 1e-3         # the program's own eager work between replays
        ff.ff_train_step(a[1], a[5][0], a[5][1], wl.theta, wl.lam, wl.lr, wl.sr_seed, s, a[3], a[4], a[2])
        torch.cuda.synchronize()
        _same(a, b, f"{name} replay {s}")
    assert int(step_dev.item()) == 4
