"""The entry point that allocates nothing (ff_layer_backward_local_noalloc: scratch in a fixed array inside the
library's device image) against ff_layer_backward_local with a caller-provided workspace: same inputs, outputs
compared bit for bit, on two calls in a row, the second with a smaller layer (the array then still holds the first
call's patch matrix and partial sums)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import ff_oracle as O  # noqa: E402
from workloads import Layer  # noqa: E402


@pytest.fixture(scope="module")
def ff():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_22771_amd as m
    m.lib()
    return m


from gpu_util import dev, empty32, empty8, pad32, pad8, pad_nhwc, scalar, workspace  # noqa: E402


def _case(ff, layer, B, seed):
    """Runs both entry points on the same synthetic accumulators; returns nothing, asserts equality."""
    rng = np.random.default_rng(seed)
    desc = ff.layer_desc(layer, B)
    M, N, K = B * layer.rows_per_sample, layer.N, layer.K
    acc = rng.integers(-30000, 30000, (M, N)).astype(np.int32)
    s_a, s_w = np.float32(0.0041), np.float32(0.0007)
    r = O.goodness_shift(K, layer.terms_per_sample)
    vmax = O.goodness(acc.reshape(B, -1), 1, r, s_a, s_w)["vmax"]
    ct = (rng.standard_normal(B) * 0.3).astype(np.float32)
    if layer.kind == "dense":
        a_q = rng.integers(-127, 128, (B, K)).astype(np.int8)
        d_aqt = dev(pad8(np.ascontiguousarray(a_q.T)))
    else:
        a_q = rng.integers(-127, 128, (B, layer.H, layer.W, layer.C_in)).astype(np.int8)
        d_aqt = dev(pad_nhwc(a_q))
    d_acc, d_vmax, d_sa, d_sw, d_ct = dev(pad32(acc)), dev(vmax), dev(np.array([s_a])), dev(np.array([s_w])), dev(ct)
    need = ff.ff_layer_workspace_bytes(desc)
    assert need <= ff.ff_noalloc_scratch_bytes()
    out = []
    for noalloc in (False, True):
        gy_t, s_g, dw = empty8(N, M), scalar(), empty32(N, K)
        if noalloc:
            ff.ff_layer_backward_local_noalloc(desc, d_acc, d_vmax, d_sa, d_sw, d_ct, 1, 4, 55, d_aqt, gy_t, s_g, dw)
        else:
            ff.ff_layer_backward_local(desc, d_acc, d_vmax, d_sa, d_sw, d_ct, 1, 4, 55, d_aqt, gy_t, s_g, dw,
                                       workspace(need))
        torch.cuda.synchronize()
        out.append((gy_t.cpu().numpy(), s_g.item(), dw.cpu().numpy()[:, :K].copy()))
    (g0, s0, w0), (g1, s1, w1) = out
    assert s0 == s1 and s0 != 1.0
    np.testing.assert_array_equal(g0, g1)
    np.testing.assert_array_equal(w0, w1)
    assert np.count_nonzero(g0) > 0 and np.count_nonzero(w0) > 0


def test_noalloc_backward_local_twice_second_smaller(ff):
    # first call: 3x3 convolution, a reduction long enough to be split (patch planes + partial sums in the scratch)
    _case(ff, Layer("conv", H=16, W=16, C_in=16, C_out=32, ksize=3, stride=1, pad=1), 24, 1)
    # second call, smaller and ragged: generic transposed patch matrix with pad bytes, no split
    _case(ff, Layer("conv", H=9, W=7, C_in=5, C_out=12, ksize=3, stride=1, pad=1), 5, 2)
    # and a dense layer (only the absmax slot of the scratch is used)
    _case(ff, Layer("dense", in_features=200, out_features=72), 130, 3)


def test_noalloc_rejects_layers_beyond_the_fixed_scratch(ff):
    """A layer whose patch matrix does not fit the fixed array is refused on the host (FF_ERR_WORKSPACE, -4)."""
    big = ff.layer_desc(Layer("conv", H=32, W=32, C_in=64, C_out=128, ksize=3, stride=1, pad=1), 256)
    assert ff.ff_layer_workspace_bytes(big) > ff.ff_noalloc_scratch_bytes() == 16 << 20
    P = C.c_void_p
    fake = P(0x1000)   # never dereferenced: the size check fails first
    st = ff.lib().ff_layer_backward_local_noalloc(C.byref(big), fake, fake, fake, fake, fake, 1, 0, 0, fake, fake, fake,
                                                  fake, P(0))
    assert st == -4
