"""ctypes face of oracle/ff_oracle.c plus the step orchestration of Algorithm 1.

TEST INFRASTRUCTURE ONLY (see the C file's header).  Nothing here imports the
HIP package; the HIP package imports nothing from here.

`train_step` strings the C functions together exactly in the order of
Algorithm 1: one full int8 forward pass per data set (positive, negative) that
records the goodness of every layer, then, for every layer, the look-ahead loss
coefficient, the int8 local gradient, the int8 weight-gradient contraction and
one SGD update of the fp32 master weights.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Sequence

import numpy as np

from . import build as _build

ROUND_NEAREST = 0
ROUND_STOCHASTIC = 1
PASS_POS = +1
PASS_NEG = -1
KIND_ACT = 0   # stochastic-rounding stream of an activation tensor
KIND_GRAD = 1  # stochastic-rounding stream of a local-gradient tensor
KIND_CHAIN = 2  # stochastic-rounding stream of the gradient handed down the chain (exact-derivative variant)
INT32_SAFE_ROWS = (2**31 - 1) // (127 * 127)   # longest reduction that cannot overflow int32

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        i64, u64, f32, f64, i32 = C.c_int64, C.c_uint64, C.c_float, C.c_double, C.c_int
        P = C.c_void_p
        L.ffo_key.restype = u64
        L.ffo_key.argtypes = [u64, u64]
        L.ffo_hash.restype = C.c_uint32
        L.ffo_hash.argtypes = [u64, u64, u64]
        L.ffo_uniform.restype = f32
        L.ffo_uniform.argtypes = [u64, u64, u64]
        L.ffo_quantize.argtypes = [P, i64, i32, u64, u64, P, P]
        L.ffo_dequantize.argtypes = [P, i64, f32, P]
        L.ffo_dequantize.restype = None
        L.ffo_dense_forward.argtypes = [P, P, i64, i64, i64, P]
        L.ffo_conv_forward.argtypes = [P, P, i64, i64, i64, i64, i64, i64, i64, i64, P]
        L.ffo_goodness_shift.argtypes = [i64, i64]
        L.ffo_goodness.argtypes = [P, i64, i64, i32, i32, f32, f32, P, P, P, P]
        L.ffo_exp_spec.restype = f32
        L.ffo_exp_spec.argtypes = [f32]
        L.ffo_loss_coeff.argtypes = [P, i64, i32, f32, P, P, P]
        L.ffo_handoff.argtypes = [P, i64, i64, i32, i32, f32, f32, P, P]
        L.ffo_lookahead.argtypes = [P, i32, i64, f32, P]
        L.ffo_local_grad.argtypes = [P, i64, i64, i32, f32, f32, P, P]
        L.ffo_dense_wgrad.argtypes = [P, P, i64, i64, i64, P]
        L.ffo_dwconv_forward.argtypes = [P, P, i64, i64, i64, i64, i64, i64, i64, P]
        L.ffo_dwconv_wgrad.argtypes = [P, P, i64, i64, i64, i64, i64, i64, i64, i64, P]
        L.ffo_skip_identity.argtypes = [P, i64, f32, P]
        L.ffo_skip_projection.argtypes = [P, i64, f32, f32, P]
        L.ffo_residual_act.argtypes = [P, P, i64, i32, f32, f32, P]
        L.ffo_goodness_fx.argtypes = [P, i64, i64, f32, P, P, P, P]
        L.ffo_local_grad_f32.argtypes = [P, i64, i64, P, P]
        L.ffo_conv_wgrad.argtypes = [P, P, i64, i64, i64, i64, i64, i64, i64, i64, i64, P]
        L.ffo_update.argtypes = [P, i64, P, P, P, i32, f32, i32]
        L.ffo_dense_input_grad.argtypes = [P, P, i64, i64, i64, P]
        L.ffo_chain_combine.argtypes = [P, i64, i64, i32, f32, f32, P, P, f32, f32, P, P]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    pass


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise OracleError(f"{what}: status {rc}")


def _p(a: np.ndarray) -> C.c_void_p:
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def stream_tag(step: int, layer: int, pass_idx: int, kind: int) -> int:
    """Unique stochastic-rounding stream per (step, layer, pass, tensor kind)."""
    return (int(step) << 20) | (int(layer) << 4) | (int(pass_idx) << 2) | int(kind)


def hash_u32(seed: int, tag: int, idx: int) -> int:
    return int(lib().ffo_hash(seed, tag, idx))


def uniform(seed: int, tag: int, idx: int) -> float:
    return float(lib().ffo_uniform(seed, tag, idx))


def quantize(x: np.ndarray, mode: int, seed: int = 0, tag: int = 0):
    """Per-tensor symmetric int8 quantisation.  Returns (q with x's shape, scale)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.int8)
    s = np.zeros(1, dtype=np.float32)
    _chk(lib().ffo_quantize(_p(x), x.size, mode, seed, tag, _p(q), _p(s)), "quantize")
    return q, np.float32(s[0])


def dequantize(q: np.ndarray, scale) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    x = np.empty(q.shape, dtype=np.float32)
    lib().ffo_dequantize(_p(q), q.size, np.float32(scale), _p(x))
    return x


def exp_spec(z: float) -> np.float32:
    return np.float32(lib().ffo_exp_spec(np.float32(z)))


def dense_forward(a_q: np.ndarray, w_q: np.ndarray) -> np.ndarray:
    M, K = a_q.shape
    N, K2 = w_q.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    _chk(lib().ffo_dense_forward(_p(a_q), _p(w_q), M, K, N, _p(acc)), "dense_forward")
    return acc


def conv_forward(a_q: np.ndarray, w_q: np.ndarray, stride: int, pad: int) -> np.ndarray:
    B, H, W, Cin = a_q.shape
    Cout, ks, ks2, Cin2 = w_q.shape
    assert ks == ks2 and Cin == Cin2
    Ho = (H + 2 * pad - ks) // stride + 1
    Wo = (W + 2 * pad - ks) // stride + 1
    acc = np.empty((B, Ho, Wo, Cout), dtype=np.int32)
    _chk(lib().ffo_conv_forward(_p(a_q), _p(w_q), B, H, W, Cin, Cout, ks, stride, pad, _p(acc)),
         "conv_forward")
    return acc


def dwconv_forward(a_q: np.ndarray, w_q: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Depthwise convolution: a_q [B, H, W, C] int8, w_q [C, ks, ks] int8 -> int32 [B, Ho, Wo, C]."""
    B, H, W, Cc = a_q.shape
    C2, ks, ks2 = w_q.shape
    assert ks == ks2 and Cc == C2
    Ho = (H + 2 * pad - ks) // stride + 1
    Wo = (W + 2 * pad - ks) // stride + 1
    acc = np.empty((B, Ho, Wo, Cc), dtype=np.int32)
    _chk(lib().ffo_dwconv_forward(_p(a_q), _p(w_q), B, H, W, Cc, ks, stride, pad, _p(acc)), "dwconv_forward")
    return acc


def dwconv_wgrad(gy_q: np.ndarray, a_q: np.ndarray, ks: int, stride: int, pad: int, b0: int, b1: int) -> np.ndarray:
    B, H, W, Cc = a_q.shape
    dw = np.empty((Cc, ks, ks), dtype=np.int32)
    _chk(lib().ffo_dwconv_wgrad(_p(gy_q), _p(a_q), b0, b1, H, W, Cc, ks, stride, pad, _p(dw)), "dwconv_wgrad")
    return dw


def goodness_shift(K: int, terms: int) -> int:
    return int(lib().ffo_goodness_shift(K, terms))


def goodness(acc: np.ndarray, relu: int, r: int, s_a, s_w):
    """acc: [B, ...]; everything after the first axis is one sample's activities.
    Returns dict(g_int uint64[B], vmax int32[B], G float32[B], G_plain float64[B])."""
    B = acc.shape[0]
    terms = acc.size // B if B else 0
    g_int = np.empty(B, dtype=np.uint64)
    vmax = np.empty(B, dtype=np.int32)
    G = np.empty(B, dtype=np.float32)
    Gp = np.empty(B, dtype=np.float64)
    _chk(lib().ffo_goodness(_p(acc), B, terms, relu, r, np.float32(s_a), np.float32(s_w),
                            _p(g_int), _p(vmax), _p(G), _p(Gp)), "goodness")
    return dict(g_int=g_int, vmax=vmax, G=G, G_plain=Gp)


def loss_coeff(G: np.ndarray, pass_sign: int, theta: float):
    G = np.ascontiguousarray(G, dtype=np.float32)
    B = G.size
    c = np.empty(B, dtype=np.float32)
    loss = np.empty(B, dtype=np.float32)
    mean = np.zeros(1, dtype=np.float64)
    _chk(lib().ffo_loss_coeff(_p(G), B, pass_sign, np.float32(theta), _p(c), _p(loss), _p(mean)),
         "loss_coeff")
    return c, loss, float(mean[0])


def handoff(acc: np.ndarray, relu: int, l2norm: int, s_a, s_w, G: np.ndarray) -> np.ndarray:
    B = acc.shape[0]
    terms = acc.size // B if B else 0
    out = np.empty(acc.shape, dtype=np.float32)
    G = np.ascontiguousarray(G, dtype=np.float32)
    _chk(lib().ffo_handoff(_p(acc), B, terms, relu, l2norm, np.float32(s_a), np.float32(s_w),
                           _p(G), _p(out)), "handoff")
    return out


def lookahead(c: np.ndarray, lam: float) -> np.ndarray:
    """c: float32 [k, B] of dL_j/dG_j.  Returns ctil [k, B]."""
    c = np.ascontiguousarray(c, dtype=np.float32)
    k, B = c.shape
    out = np.empty_like(c)
    _chk(lib().ffo_lookahead(_p(c), k, B, np.float32(lam), _p(out)), "lookahead")
    return out


def local_grad(acc: np.ndarray, relu: int, s_a, s_w, ctil: np.ndarray) -> np.ndarray:
    B = acc.shape[0]
    terms = acc.size // B if B else 0
    ctil = np.ascontiguousarray(ctil, dtype=np.float32)
    g = np.empty(acc.shape, dtype=np.float32)
    _chk(lib().ffo_local_grad(_p(acc), B, terms, relu, np.float32(s_a), np.float32(s_w),
                              _p(ctil), _p(g)), "local_grad")
    return g


# ---- residual blocks (a reading: the paper names ResNet-style blocks in Section IV-C without mechanics) ----
def skip_identity(x_q: np.ndarray, s_x) -> np.ndarray:
    x_q = np.ascontiguousarray(x_q, dtype=np.int8)
    u = np.empty(x_q.shape, dtype=np.float32)
    _chk(lib().ffo_skip_identity(_p(x_q), x_q.size, np.float32(s_x), _p(u)), "skip_identity")
    return u


def skip_projection(acc_p: np.ndarray, s_a, s_w) -> np.ndarray:
    acc_p = np.ascontiguousarray(acc_p, dtype=np.int32)
    u = np.empty(acc_p.shape, dtype=np.float32)
    _chk(lib().ffo_skip_projection(_p(acc_p), acc_p.size, np.float32(s_a), np.float32(s_w), _p(u)), "skip_projection")
    return u


def residual_act(acc: np.ndarray, u: np.ndarray, relu: int, s_a, s_w) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    assert acc.shape == u.shape
    y = np.empty(acc.shape, dtype=np.float32)
    _chk(lib().ffo_residual_act(_p(acc), _p(u), acc.size, relu, np.float32(s_a), np.float32(s_w), _p(y)), "residual_act")
    return y


def goodness_fx(y: np.ndarray) -> Dict[str, np.ndarray]:
    """Order-free goodness of an fp32 activity tensor [B, ...] (one pass): see ffo_goodness_fx."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    B = y.shape[0]
    terms = y.size // B if B else 0
    amax = np.float32(np.max(np.abs(y))) if y.size else np.float32(0)
    g_int = np.empty(B, dtype=np.uint64)
    ymax = np.empty(B, dtype=np.float32)
    G = np.empty(B, dtype=np.float32)
    G_plain = np.empty(B, dtype=np.float64)
    _chk(lib().ffo_goodness_fx(_p(y), B, terms, amax, _p(g_int), _p(ymax), _p(G), _p(G_plain)), "goodness_fx")
    return dict(g_int=g_int, ymax=ymax, G=G, G_plain=G_plain, amax=amax)


def local_grad_f32(y: np.ndarray, ctil: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float32)
    B = y.shape[0]
    terms = y.size // B if B else 0
    ctil = np.ascontiguousarray(ctil, dtype=np.float32)
    g = np.empty(y.shape, dtype=np.float32)
    _chk(lib().ffo_local_grad_f32(_p(y), B, terms, _p(ctil), _p(g)), "local_grad_f32")
    return g


def dense_wgrad(gy_q: np.ndarray, a_q: np.ndarray) -> np.ndarray:
    M, N = gy_q.shape
    M2, K = a_q.shape
    assert M == M2
    dw = np.empty((N, K), dtype=np.int32)
    _chk(lib().ffo_dense_wgrad(_p(gy_q), _p(a_q), M, K, N, _p(dw)), "dense_wgrad")
    return dw


def conv_wgrad(gy_q: np.ndarray, a_q: np.ndarray, ks: int, stride: int, pad: int,
               b0: int, b1: int) -> np.ndarray:
    B, H, W, Cin = a_q.shape
    Cout = gy_q.shape[-1]
    dw = np.empty((Cout, ks, ks, Cin), dtype=np.int32)
    _chk(lib().ffo_conv_wgrad(_p(gy_q), _p(a_q), b0, b1, H, W, Cin, Cout, ks, stride, pad, _p(dw)),
         "conv_wgrad")
    return dw


def dense_input_grad(h_q: np.ndarray, w_q: np.ndarray) -> np.ndarray:
    """e[m][k] = sum_n h_q[m][n] * w_q[n][k] (int32): the gradient handed to the layer below."""
    M, N = h_q.shape
    N2, K = w_q.shape
    assert N == N2
    e = np.empty((M, K), dtype=np.int32)
    _chk(lib().ffo_dense_input_grad(_p(h_q), _p(w_q), M, K, N, _p(e)), "dense_input_grad")
    return e


def chain_combine(acc: np.ndarray, relu: int, s_a, s_w, c: np.ndarray, e_acc, s_e, lam: float):
    """(h, g) of ffo_chain_combine; e_acc None = the top layer (no later losses)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    B = acc.shape[0]
    terms = acc.size // B if B else 0
    c = np.ascontiguousarray(c, dtype=np.float32)
    h = np.empty(acc.shape, dtype=np.float32)
    g = np.empty(acc.shape, dtype=np.float32)
    ep = None
    if e_acc is not None:
        e_acc = np.ascontiguousarray(e_acc, dtype=np.int32)
        assert e_acc.shape == acc.shape
        ep = _p(e_acc)
    _chk(lib().ffo_chain_combine(_p(acc), B, terms, relu, np.float32(s_a), np.float32(s_w), _p(c), ep,
                                 np.float32(s_e), np.float32(lam), _p(h), _p(g)), "chain_combine")
    return h, g


def update(w: np.ndarray, dws: Sequence[np.ndarray], s_g: Sequence[float], s_a: Sequence[float],
           lr: float, total_samples: int) -> np.ndarray:
    """Returns the updated fp32 master weights (w itself is left untouched)."""
    w = np.array(w, dtype=np.float32, copy=True, order="C")
    n = len(dws)
    ptrs = (C.c_void_p * n)(*[d.ctypes.data for d in dws])
    sg = np.asarray(s_g, dtype=np.float32)
    sa = np.asarray(s_a, dtype=np.float32)
    for d in dws:
        assert d.dtype == np.int32 and d.size == w.size and d.flags["C_CONTIGUOUS"]
    _chk(lib().ffo_update(_p(w), w.size, ptrs, _p(sg), _p(sa), n, np.float32(lr), total_samples),
         "update")
    return w


def batch_chunks(B: int, rows_per_sample: int) -> List[tuple]:
    """Sample ranges whose reduction length (rows) cannot overflow an int32 accumulator: the whole batch
    if it fits, else equal blocks of `per` samples, per = the largest power of two whose rows still fit."""
    if B * rows_per_sample <= INT32_SAFE_ROWS:
        return [(0, B)]
    if rows_per_sample > INT32_SAFE_ROWS:
        raise OracleError("one sample alone exceeds the int32-safe reduction length")
    per = 1
    while per * 2 * rows_per_sample <= INT32_SAFE_ROWS:
        per *= 2
    return [(b0, min(B, b0 + per)) for b0 in range(0, B, per)]


# --------------------------------------------------------------------------------------
# Algorithm 1, one iteration.
# --------------------------------------------------------------------------------------
def _theta_of(theta, i: int) -> float:
    """The goodness threshold of layer i: Section V-A uses one value (2.0) for every layer; a sequence
    gives each layer its own (a generalisation the tests use to keep both passes' gradients live at
    initialisation, where the goodness differs from layer to layer by orders of magnitude)."""
    return float(theta[i]) if hasattr(theta, "__len__") else float(theta)


def forward_layer(layer, a_f32: np.ndarray, w_q: np.ndarray, s_w, pass_sign: int, theta: float,
                  seed: int, tag_act: int) -> Dict:
    """Quantise the layer input (stochastic rounding), contract, goodness, loss coefficient,
    and the fp32 input of the next layer."""
    a_q, s_a = quantize(a_f32, ROUND_STOCHASTIC, seed, tag_act)
    if layer.kind == "dense":
        acc = dense_forward(a_q, w_q)
    elif layer.kind == "dwconv":
        acc = dwconv_forward(a_q, w_q, layer.stride, layer.pad)
    else:
        acc = conv_forward(a_q, w_q, layer.stride, layer.pad)
    r = goodness_shift(layer.K, layer.terms_per_sample)
    gd = goodness(acc, layer.relu, r, s_a, s_w)
    c, loss, loss_mean = loss_coeff(gd["G"], pass_sign, theta)
    a_next = handoff(acc, layer.relu, layer.l2norm_out, s_a, s_w, gd["G"])
    return dict(a_q=a_q, s_a=s_a, acc=acc, r=r, c=c, loss=loss, loss_mean=loss_mean,
                a_next=a_next, **gd)


def _layer_attr(layer, name, default):
    return getattr(layer, name, default)


def train_step(layers, w_master: List[np.ndarray], x_pos: np.ndarray, x_neg: np.ndarray,
               theta: float, lam: float, lr: float, seed: int, step: int,
               keep: bool = True, train_mask=None) -> Dict:
    """One iteration of Algorithm 1 over both data sets.  Returns the new master weights,
    the new int8 weights and (keep=True) every intermediate, per layer and pass.
    train_mask: optional per-layer flags; a layer whose flag is false is frozen (forward only,
    its coefficients still enter the look-ahead sums of earlier layers): the greedy
    layer-by-layer schedule of Section III.

    Basic residual blocks (a reading, see ffo_residual_act): a layer may carry
      input_back = n : its input is the output of layer i-1-n (0 = the previous layer),
      role = 'proj'  : a 1x1 projection branch: contraction only, no activity, goodness or
                       hand-off of its own; its accumulators are the skip of layer i+2,
      skip = 'identity'   : block output y = act(s*acc + dequantised input of layer i-1),
      skip = 'projection' : block output y = act(s*acc + s_p*acc of layer i-2).
    A projection layer is updated with the quantised local gradient of the block output."""
    k = len(layers)
    wq = [quantize(w, ROUND_NEAREST) for w in w_master]
    B = x_pos.shape[0]
    role = [_layer_attr(l, "role", "ff") for l in layers]
    skip = [_layer_attr(l, "skip", "none") for l in layers]
    fwd: List[List[Dict]] = [[None, None] for _ in range(k)]
    for p, (x, sign) in enumerate(((x_pos, PASS_POS), (x_neg, PASS_NEG))):
        outs: List[np.ndarray] = [None] * k
        for i, layer in enumerate(layers):
            src = i - 1 - _layer_attr(layer, "input_back", 0)
            a = np.ascontiguousarray(x if src < 0 else outs[src], dtype=np.float32)
            if layer.kind == "dense" and a.ndim > 2:
                a = a.reshape(B, -1)     # flatten: NHWC order, the element order of the tensor itself
            tag = stream_tag(step, i, p, KIND_ACT)
            if role[i] == "proj":
                a_q, s_a = quantize(a, ROUND_STOCHASTIC, seed, tag)
                acc = conv_forward(a_q, wq[i][0], layer.stride, layer.pad)
                fwd[i][p] = dict(a_q=a_q, s_a=s_a, acc=acc, c=np.zeros(B, np.float32), loss_mean=0.0,
                                 G=np.zeros(B, np.float32))
            elif skip[i] == "none":
                f = forward_layer(layer, a, wq[i][0], wq[i][1], sign, _theta_of(theta, i), seed, tag)
                outs[i] = f.pop("a_next")
                fwd[i][p] = f
            else:
                a_q, s_a = quantize(a, ROUND_STOCHASTIC, seed, tag)
                acc = conv_forward(a_q, wq[i][0], layer.stride, layer.pad)
                if skip[i] == "identity":
                    u = skip_identity(fwd[i - 1][p]["a_q"], fwd[i - 1][p]["s_a"])
                else:
                    u = skip_projection(fwd[i - 2][p]["acc"], fwd[i - 2][p]["s_a"], wq[i - 2][1])
                y = residual_act(acc, u.reshape(acc.shape), layer.relu, s_a, wq[i][1])
                gd = goodness_fx(y)
                c, loss, loss_mean = loss_coeff(gd["G"], sign, _theta_of(theta, i))
                outs[i] = y
                fwd[i][p] = dict(a_q=a_q, s_a=s_a, acc=acc, y=y, c=c, loss=loss, loss_mean=loss_mean, **gd)
    ctil = [lookahead(np.stack([fwd[i][p]["c"] for i in range(k)]), lam) for p in range(2)]
    new_w = [None] * k
    new_wq = [None] * k
    new_sw = [None] * k
    grads = [None] * k

    def frozen(i):
        return train_mask is not None and not train_mask[i]

    def finish(i, dws, sgs, sas):
        if frozen(i):
            new_w[i], new_wq[i], new_sw[i] = w_master[i], wq[i][0], wq[i][1]
            return
        w_new = update(w_master[i], dws, sgs, sas, lr, 2 * B)
        q_new, s_new = quantize(w_new, ROUND_NEAREST)
        new_w[i], new_wq[i], new_sw[i] = w_new, q_new, s_new

    for i, layer in enumerate(layers):
        if role[i] == "proj":
            continue          # updated together with the block-output layer i+2
        dws, sgs, sas = [], [], []
        pdws, psas = [], []
        per_pass = []
        for p in range(2):
            f = fwd[i][p]
            if skip[i] == "none":
                g = local_grad(f["acc"], layer.relu, f["s_a"], wq[i][1], ctil[p][i])
            else:
                g = local_grad_f32(f["y"], ctil[p][i])
            gy_q, s_g = quantize(g, ROUND_STOCHASTIC, seed, stream_tag(step, i, p, KIND_GRAD))
            chunks = batch_chunks(B, layer.rows_per_sample)
            dw_chunks = []
            for (b0, b1) in chunks:
                if layer.kind == "dense":
                    dw = dense_wgrad(gy_q[b0:b1], f["a_q"][b0:b1])
                elif layer.kind == "dwconv":
                    dw = dwconv_wgrad(gy_q, f["a_q"], layer.ksize, layer.stride, layer.pad, b0, b1)
                else:
                    dw = conv_wgrad(gy_q, f["a_q"], layer.ksize, layer.stride, layer.pad, b0, b1)
                dw_chunks.append(dw.reshape(-1))
                dws.append(dw.reshape(-1))
                sgs.append(s_g)
                sas.append(f["s_a"])
                if skip[i] == "projection":
                    lp, fp = layers[i - 2], fwd[i - 2][p]
                    pdws.append(conv_wgrad(gy_q, fp["a_q"], lp.ksize, lp.stride, lp.pad, b0, b1).reshape(-1))
                    psas.append(fp["s_a"])
            per_pass.append(dict(gy_q=gy_q, s_g=s_g, dw=dw_chunks, ctil=ctil[p][i]))
        finish(i, dws, sgs, sas)
        if skip[i] == "projection":
            finish(i - 2, pdws, sgs, psas)
        grads[i] = per_pass
    out = dict(w_master=new_w, w_q=new_wq, s_w=new_sw,
               loss=np.array([[fwd[i][p]["loss_mean"] for p in range(2)] for i in range(k)]),
               goodness=np.stack([np.stack([fwd[i][p]["G"] for p in range(2)]) for i in range(k)]))
    if keep:
        out.update(fwd=fwd, grads=grads, w_q_in=[q for q, _ in wq], s_w_in=[s for _, s in wq])
    return out


def train_step_chain(layers, w_master: List[np.ndarray], x_pos: np.ndarray, x_neg: np.ndarray,
                     theta: float, lam: float, lr: float, seed: int, step: int, keep: bool = True,
                     train_mask=None) -> Dict:
    """One iteration with Eq. (4) read as an exact derivative (see ffo_dense_input_grad): the same
    forward pass as train_step, then per pass a sweep from the last layer to the first that hands
    the int8 gradient H_i down through the pre-step weights.  Dense layers without normalisation."""
    k = len(layers)
    for l in layers:
        if l.kind != "dense" or l.l2norm_out or _layer_attr(l, "skip", "none") != "none" \
                or _layer_attr(l, "role", "ff") != "ff" or _layer_attr(l, "input_back", 0):
            raise OracleError("the exact-derivative look-ahead is defined for plain dense stacks only")
    wq = [quantize(w, ROUND_NEAREST) for w in w_master]
    B = x_pos.shape[0]
    fwd: List[List[Dict]] = [[None, None] for _ in range(k)]
    for p, (x, sign) in enumerate(((x_pos, PASS_POS), (x_neg, PASS_NEG))):
        a = np.ascontiguousarray(x, dtype=np.float32)
        for i, layer in enumerate(layers):
            f = forward_layer(layer, a, wq[i][0], wq[i][1], sign, _theta_of(theta, i), seed, stream_tag(step, i, p, KIND_ACT))
            a = f.pop("a_next")
            fwd[i][p] = f
    grads: List[List[Dict]] = [[None, None] for _ in range(k)]
    for p in range(2):
        e_acc, s_e = None, np.float32(0)
        for i in range(k - 1, -1, -1):
            f, layer = fwd[i][p], layers[i]
            h, g = chain_combine(f["acc"], layer.relu, f["s_a"], wq[i][1], f["c"], e_acc, s_e, lam)
            gy_q, s_g = quantize(g, ROUND_STOCHASTIC, seed, stream_tag(step, i, p, KIND_GRAD))
            rec = dict(gy_q=gy_q, s_g=s_g, dw=[dense_wgrad(gy_q, f["a_q"]).reshape(-1)], h=h, g=g, e_acc=e_acc, s_e=s_e)
            if i > 0:
                h_q, s_h = quantize(h, ROUND_STOCHASTIC, seed, stream_tag(step, i, p, KIND_CHAIN))
                e_acc = dense_input_grad(h_q, wq[i][0])
                s_e = np.float32(s_h) * np.float32(wq[i][1])
                rec.update(h_q=h_q, s_h=s_h)
            grads[i][p] = rec
    new_w, new_wq, new_sw = [None] * k, [None] * k, [None] * k
    for i in range(k):
        if train_mask is not None and not train_mask[i]:
            new_w[i], new_wq[i], new_sw[i] = w_master[i], wq[i][0], wq[i][1]
            continue
        w_new = update(w_master[i], [grads[i][p]["dw"][0] for p in range(2)], [grads[i][p]["s_g"] for p in range(2)],
                       [fwd[i][p]["s_a"] for p in range(2)], lr, 2 * B)
        new_w[i] = w_new
        new_wq[i], new_sw[i] = quantize(w_new, ROUND_NEAREST)
    out = dict(w_master=new_w, w_q=new_wq, s_w=new_sw,
               loss=np.array([[fwd[i][p]["loss_mean"] for p in range(2)] for i in range(k)]),
               goodness=np.stack([np.stack([fwd[i][p]["G"] for p in range(2)]) for i in range(k)]))
    if keep:
        out.update(fwd=fwd, grads=grads, w_q_in=[q for q, _ in wq], s_w_in=[s for _, s in wq])
    return out
