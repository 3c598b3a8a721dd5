"""CPU-side checks of the boundary: the built library loads, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ff():
    import paper_2506_22771_amd as m
    try:
        m.lib()
    except FileNotFoundError:
        import __graft_entry__ as g
        g.build()
        m.lib()
    return m


def test_every_declared_symbol_is_exported(ff):
    text = open(os.path.join(ROOT, "include", "ffint8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(ff_[a-z0-9_]+)\s*\(", text)))
    assert {"ff_quantize", "ff_layer_forward", "ff_goodness_loss", "ff_layer_backward_local", "ff_layer_update",
            "ff_train_step"} <= set(names)
    L = ff.lib()
    for n in names:
        assert hasattr(L, n), n


def test_pitch_and_tags(ff):
    assert [ff.ff_pitch(c) for c in (0, 1, 16, 17, 500, 512, 4096)] == [0, 16, 16, 32, 512, 512, 4096]
    # rows longer than 512 bytes start on 128-byte lines
    assert [ff.ff_pitch(c) for c in (513, 576, 784, 2000, 4097)] == [640, 640, 896, 2048, 4224]
    assert [ff.ff_pitch32(c) for c in (0, 1, 4, 5, 500)] == [0, 4, 4, 8, 500]
    from oracle import ff_oracle as O
    for args in [(0, 0, 0, 0), (3, 2, 1, 1), (1000, 19, 0, 1)]:
        assert ff.ff_stream_tag(*args) == O.stream_tag(*args)
    assert ff.ff_status_string(0) == "ok" and "workspace" in ff.ff_status_string(-4)


def test_goodness_shift_matches_big_integer_bound(ff):
    from workloads import Layer
    for K, N in [(784, 500), (4096, 4096), (100, 72), (133144, 8)]:
        d = ff.layer_desc(Layer("dense", in_features=K, out_features=N), 8)
        r = ff.ff_goodness_shift(d)
        worst = (16129 * K) ** 2 * N
        assert (worst >> r) < 2 ** 64 and (r == 0 or (worst >> (r - 1)) >= 2 ** 64)


def test_argument_errors_are_host_side(ff):
    """Null pointers, bad enums, bad shapes, misalignment and a short workspace are reported as status
    codes before any launch (this runs without a GPU)."""
    L = ff.lib()
    from workloads import Layer
    d = ff.layer_desc(Layer("dense", in_features=32, out_features=16), 8)
    P = C.c_void_p
    fake = P(0x1000)        # never dereferenced: validation fails first
    assert L.ff_quantize(P(0), 4, 4, 1, 0, 0, fake, P(0), P(0), fake, 4096, P(0)) == -1       # scale null
    assert L.ff_quantize(fake, 4, 4, 7, 0, 0, fake, P(0), fake, fake, 4096, P(0)) == -1       # bad rounding mode
    assert L.ff_quantize(fake, 4, 4, 1, 0, 0, fake, P(0), fake, fake, 16, P(0)) == -4         # workspace
    assert L.ff_quantize(fake, 4, 4, 1, 0, 0, P(0x1008), P(0), fake, fake, 4096, P(0)) == -3  # alignment
    assert L.ff_quantize(fake, -1, 4, 1, 0, 0, fake, P(0), fake, fake, 4096, P(0)) == -1
    assert L.ff_layer_forward(C.byref(d), P(0), fake, fake, fake, fake, fake, 4096, P(0)) == -1
    bad = ff.layer_desc(Layer("dense", in_features=0, out_features=16), 8)
    assert L.ff_layer_forward(C.byref(bad), fake, fake, fake, fake, fake, fake, 4096, P(0)) == -2
    long = ff.layer_desc(Layer("dense", in_features=133145, out_features=16), 8)
    assert L.ff_layer_forward(C.byref(long), fake, fake, fake, fake, fake, fake, 4096, P(0)) == -5
    assert L.ff_goodness_loss(C.byref(d), fake, fake, fake, fake, 0, 2.0, fake, fake, fake, P(0), P(0)) == -1
    assert L.ff_lookahead(fake, 0, 8, 0.1, fake, P(0)) == -2
    assert L.ff_lookahead(fake, 33, 8, 0.1, fake, P(0)) == -2
    assert L.ff_layer_update(C.byref(d), fake, fake, fake, fake, fake, fake, fake, 0.1, 0, fake, fake, fake, 4096,
                             P(0)) == -1
    assert L.ff_workspace_bytes(None) == 0


def test_workspace_bytes_and_train_step_validation(ff):
    from workloads import workload
    import ctypes as C
    wl = workload("cfg1")
    descs = (ff.binding.LayerDesc * 2)(*[ff.layer_desc(l, wl.batch) for l in wl.layers])
    net = ff.binding.NetDesc(2, wl.batch, descs)
    n = ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(2, wl.batch, descs, None, 0, None, 1)))   # per-operation kernels
    # the single-launch step (what FF_LAUNCH_AUTO picks for this stack) keeps every layer's int8 local gradient
    extra = 2 * sum(l.N * ff.ff_pitch(wl.batch) for l in wl.layers)
    assert n + extra <= ff.lib().ff_workspace_bytes(C.byref(net)) <= n + extra + 8192
    # at least the retained int32 accumulators and transposed int8 inputs of both layers, both passes
    need = 2 * sum(wl.batch * l.N * 4 + l.K * ff.ff_pitch(wl.batch) for l in wl.layers)
    scratch = 2 * max(l.N * l.K * 4 + wl.batch * ff.ff_pitch(l.K) + l.N * ff.ff_pitch(wl.batch) for l in wl.layers)
    assert need + scratch <= n < 2 * (need + scratch) + (1 << 20)
    mism = (ff.binding.LayerDesc * 2)(ff.layer_desc(wl.layers[0], wl.batch), ff.layer_desc(wl.layers[0], wl.batch))
    assert ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(2, wl.batch, mism))) == 0   # 500 != 784
    assert ff.lib().ff_train_step(C.byref(net), None, None, None, 2.0, 0.0, 0.1, 0, 0, None, None, None, 0, None) == -1


def test_residual_topology_validation(ff):
    """Host-side checks of the residual-block wiring in ff_net_desc: valid stacks get a workspace size, every
    inconsistent wiring is rejected (size 0) before anything could be launched."""
    import ctypes as C
    import dataclasses
    from workloads import workload

    def ws_bytes(layers, batch):
        descs = (ff.binding.LayerDesc * len(layers))(*[ff.layer_desc(l, batch) for l in layers])
        return ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(len(layers), batch, descs)))

    for name in ("tiny_res", "cfg4"):
        wl = workload(name)
        assert ws_bytes(wl.layers, wl.batch) > 0
    wl = workload("tiny_res")
    L = list(wl.layers)   # stem, conv1, conv2(identity), proj, conv1(input_back=1), conv2(projection)
    rep = dataclasses.replace

    def bad(i, **kw):
        layers = list(L)
        layers[i] = rep(layers[i], **kw)
        return ws_bytes(layers, wl.batch)

    assert bad(2, skip="projection") == 0          # no projection two layers back
    assert bad(2, C_out=24) == 0                   # identity skip with a different channel count
    assert bad(5, skip="identity") == 0            # block input 16 channels at 8x16, output 32 channels at 4x8
    assert bad(5, skip="none") == 0                # a projection nobody adds
    assert bad(4, input_back=0) == 0               # conv1 after a projection must read the block input
    assert bad(3, relu=1) == 0                     # a projection has no activation of its own
    assert bad(1, input_back=2) == 0               # only the previous layer or the one before it
    assert bad(2, l2norm_out=1) == 0               # no normalised hand-off from a block output
    assert ws_bytes(L[:4], wl.batch) == 0          # stack ends in a projection


def test_chain_lookahead_validation(ff):
    """FF_LOOKAHEAD_CHAIN: plain dense stacks only; it needs more workspace than the default reading; an unknown mode
    is an argument error (workspace 0)."""
    import ctypes as C
    from workloads import workload

    def nbytes(name, mode):
        wl = workload(name)
        descs = (ff.binding.LayerDesc * len(wl.layers))(*[ff.layer_desc(l, wl.batch) for l in wl.layers])
        # (per-operation kernels on both sides: the single-launch step has workspace needs of its own)
        return ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(len(wl.layers), wl.batch, descs, None, mode, None, 1)))

    assert nbytes("tiny", 1) > nbytes("tiny", 0) > 0
    assert nbytes("cfg5", 1) > nbytes("cfg5", 0)
    assert nbytes("tiny_l2", 1) == 0 and nbytes("tiny_conv", 1) == 0 and nbytes("tiny_res", 1) == 0
    assert nbytes("tiny", 2) == 0 and nbytes("tiny", -1) == 0


def test_int32_reduction_limits(ff):
    """The longest weight-gradient reduction that cannot overflow int32 is 133 144 rows (127^2 * 133144 < 2^31): one
    accumulator up to there, power-of-two sample blocks beyond, and the step refuses more than two blocks per pass."""
    import ctypes as C
    from workloads import Layer
    assert 127 * 127 * 133144 < 2**31 <= 127 * 127 * 133145

    def chunks_and_ws(B):
        d = ff.layer_desc(Layer("dense", in_features=32, out_features=16), B)
        descs = (ff.binding.LayerDesc * 1)(d)
        return ff.ff_layer_dw_chunks(d), ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(1, B, descs)))

    assert chunks_and_ws(133144)[0] == 1 and chunks_and_ws(133144)[1] > 0
    assert chunks_and_ws(133145)[0] == 2 and chunks_and_ws(133145)[1] > 0       # blocks of 131072 samples
    assert chunks_and_ws(262144)[0] == 2 and chunks_and_ws(262144)[1] > 0
    assert chunks_and_ws(262145) == (3, 0)                                       # a third block: not in ff_train_step
    conv = Layer("conv", H=32, W=32, C_in=16, C_out=16, ksize=3, stride=1, pad=1)   # 1024 rows per sample
    assert ff.ff_layer_dw_chunks(ff.layer_desc(conv, 130)) == 1                  # 133120 rows
    assert ff.ff_layer_dw_chunks(ff.layer_desc(conv, 131)) == 2                  # blocks of 128 samples
    assert ff.ff_layer_dw_chunks(ff.layer_desc(conv, 256)) == 2
    assert ff.ff_layer_dw_chunks(ff.layer_desc(conv, 257)) == 3
    # a reduction over the input features longer than the limit cannot be chunked: the forward pass refuses it
    long = ff.layer_desc(Layer("dense", in_features=133145, out_features=16), 8)
    assert ff.ff_goodness_shift(long) >= 0 and ff.ff_layer_workspace_bytes(long) >= 0


def test_launch_limits_are_host_side(ff):
    """Sizes beyond what the kernels' grids and 32-bit element indices cover are refused on the host with
    FF_ERR_UNSUPPORTED (-6) before anything is enqueued: tensors of 2^32 elements or more, more than 65535 row
    blocks of 128 rows in a quantised matrix, more than 65535 output features."""
    L = ff.lib()
    from workloads import Layer
    P = C.c_void_p
    fake = P(0x1000)        # never dereferenced: validation fails first
    assert L.ff_quantize(fake, 1 << 16, 1 << 16, 1, 0, 0, fake, P(0), fake, fake, 4096, P(0)) == -6   # 2^32 elements
    assert L.ff_quantize(fake, 65535 * 128 + 1, 4, 1, 0, 0, fake, P(0), fake, fake, 4096, P(0)) == -6   # grid rows

    def status(layer, B):
        d = ff.layer_desc(layer, B)
        return L.ff_layer_forward(C.byref(d), fake, fake, fake, fake, fake, fake, 4096, P(0))

    assert status(Layer("dense", in_features=1 << 15, out_features=1 << 15), 1 << 17) == -6   # B*K = 2^32
    assert status(Layer("dense", in_features=16, out_features=65536), 8) == -6                # weight rows on grid.y
    assert status(Layer("dense", in_features=16, out_features=16), 65535 * 128 + 1) == -6     # batch rows on grid.y
    assert ff.ff_layer_workspace_bytes(ff.layer_desc(Layer("dense", in_features=16, out_features=65535), 8)) > 0
    assert ff.ff_layer_workspace_bytes(ff.layer_desc(Layer("dense", in_features=16, out_features=16), 65535 * 128)) > 0
    many = Layer("conv", H=32, W=32, C_in=16, C_out=16, ksize=3, stride=1, pad=1, skip="identity")
    descs = (ff.binding.LayerDesc * 2)(ff.layer_desc(Layer("conv", H=32, W=32, C_in=16, C_out=16, ksize=3, stride=1, pad=1), 70000),
                                       ff.layer_desc(many, 70000))
    assert L.ff_workspace_bytes(C.byref(ff.binding.NetDesc(2, 70000, descs))) == 0            # block-output kernels: B on grid.y


def test_launch_mode_validation(ff):
    """ff_net_desc.launch_mode: unknown values are argument errors; the single launch is refused (workspace 0) for
    stacks it does not cover; where it applies it needs more workspace than the per-operation kernels."""
    import ctypes as C
    from workloads import workload

    def nbytes(name, mode):
        wl = workload(name)
        descs = (ff.binding.LayerDesc * len(wl.layers))(*[ff.layer_desc(l, wl.batch) for l in wl.layers])
        return ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(len(wl.layers), wl.batch, descs, None, 0, None, mode)))

    assert nbytes("cfg1", 4) == 0 and nbytes("cfg1", -1) == 0
    assert nbytes("cfg1", 2) == nbytes("cfg1", 0) > nbytes("cfg1", 1) > 0        # auto picks the single launch for cfg1
    assert nbytes("cfg5", 2) == 0 and nbytes("cfg5", 0) == nbytes("cfg5", 1) > 0  # 8192 samples per pass: too many
    assert nbytes("cfg3", 2) == 0 and nbytes("tiny_res", 2) == 0                  # convolutions, residual wiring
    # update chains on several streams: every lane has its own chain scratch; auto picks lanes for stacks of small
    # layers (three for cfg4 and cfg2, two for cfg3) and none for cfg5
    assert nbytes("cfg4", 3) == nbytes("cfg4", 0) > nbytes("cfg4", 1) > 0
    assert nbytes("cfg2", 3) == nbytes("cfg2", 0) > nbytes("cfg2", 1) > 0
    assert nbytes("cfg3", 3) > nbytes("cfg3", 0) > nbytes("cfg3", 1) > 0
    assert nbytes("cfg5", 3) > nbytes("cfg5", 1)
    wl = workload("tiny")
    descs = (ff.binding.LayerDesc * 2)(*[ff.layer_desc(l, wl.batch) for l in wl.layers])
    assert ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(2, wl.batch, descs, None, 1, None, 2))) == 0   # chain + fused
    assert ff.lib().ff_workspace_bytes(C.byref(ff.binding.NetDesc(2, wl.batch, descs, None, 1, None, 3))) == 0   # chain + lanes
