"""ctypes binding of include/ffint8.h.  Argument marshalling only.

Functions mirror the C-ABI names.  Tensor arguments are torch CUDA tensors (or None where the
header allows NULL); their data_ptr() is handed to the library together with the current
torch stream.  Nothing here computes."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
PASS_POS, PASS_NEG = 1, -1
KIND_ACT, KIND_GRAD, KIND_CHAIN = 0, 1, 2
WS_MIN_BYTES = 1024

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libffint8.so")
_lib = None


class FFError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {ff_status_string(status)} ({status})")


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "batch", "in_features", "out_features", "H", "W", "C_in", "C_out",
                                         "ksize", "stride", "pad", "relu", "l2norm_out", "input_back", "role", "skip")]


class NetDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("layers", C.POINTER(LayerDesc)),
                ("train_layer", C.POINTER(C.c_int32)), ("lookahead", C.c_int32),
                ("theta_layer", C.POINTER(C.c_float)), ("launch_mode", C.c_int32)]


class NetState(C.Structure):
    _fields_ = [("w_master", C.POINTER(C.c_void_p)), ("w_q", C.POINTER(C.c_void_p)), ("s_w", C.POINTER(C.c_void_p))]


def lib() -> C.CDLL:
    """Loads the built HIP library; raises if it has not been built (python -m paper_2506_22771_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with `python -m paper_2506_22771_amd.build`")
        L = C.CDLL(_LIB_PATH)
        P, i32, i64, u64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
        LD = C.POINTER(LayerDesc)
        L.ff_pitch.restype = i64
        L.ff_pitch.argtypes = [i64]
        L.ff_pitch32.restype = i64
        L.ff_pitch32.argtypes = [i64]
        L.ff_stream_tag.restype = u64
        L.ff_stream_tag.argtypes = [u64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.ff_status_string.restype = C.c_char_p
        L.ff_status_string.argtypes = [i32]
        L.ff_version.restype = C.c_char_p
        L.ff_goodness_shift.restype = i32
        L.ff_goodness_shift.argtypes = [LD]
        L.ff_layer_dw_chunks.restype = i32
        L.ff_layer_dw_chunks.argtypes = [LD]
        L.ff_layer_workspace_bytes.restype = sz
        L.ff_layer_workspace_bytes.argtypes = [LD]
        L.ff_quantize.restype = i32
        L.ff_quantize.argtypes = [P, i64, i64, i32, u64, u64, P, P, P, P, sz, P]
        L.ff_layer_forward.restype = i32
        L.ff_layer_forward.argtypes = [LD, P, P, P, P, P, P, sz, P]
        L.ff_goodness_loss.restype = i32
        L.ff_goodness_loss.argtypes = [LD, P, P, P, P, i32, f32, P, P, P, P, P]
        L.ff_layer_handoff.restype = i32
        L.ff_layer_handoff.argtypes = [LD, P, P, P, P, P, i32, u64, u64, P, P, P, P]
        L.ff_lookahead.restype = i32
        L.ff_lookahead.argtypes = [P, i32, i64, f32, P, P]
        L.ff_layer_backward_local.restype = i32
        L.ff_layer_backward_local.argtypes = [LD, P, P, P, P, P, i32, u64, u64, P, P, P, P, P, sz, P]
        L.ff_layer_backward_local_noalloc.restype = i32
        L.ff_layer_backward_local_noalloc.argtypes = [LD, P, P, P, P, P, i32, u64, u64, P, P, P, P, P]
        L.ff_noalloc_scratch_bytes.restype = sz
        L.ff_chain_gradients.restype = i32
        L.ff_chain_gradients.argtypes = [LD, P, P, P, P, P, P, P, f32, P, P, P, P, P]
        L.ff_layer_input_grad.restype = i32
        L.ff_layer_input_grad.argtypes = [LD, P, P, P, P, sz, P]
        L.ff_layer_update.restype = i32
        L.ff_layer_update.argtypes = [LD, P, P, P, P, P, P, P, f32, i32, P, P, P, sz, P]
        L.ff_train_step.restype = i32
        L.ff_train_step.argtypes = [C.POINTER(NetDesc), C.POINTER(NetState), P, P, f32, f32, f32, u64, u64, P, P, P,
                                    sz, P]
        L.ff_train_step_at.restype = i32
        L.ff_train_step_at.argtypes = [C.POINTER(NetDesc), C.POINTER(NetState), P, P, f32, f32, f32, u64, P, i32, P, P,
                                       P, sz, P]
        L.ff_workspace_bytes.restype = sz
        L.ff_workspace_bytes.argtypes = [C.POINTER(NetDesc)]
        L.ff_timing_enable.restype = i32
        L.ff_timing_enable.argtypes = [i32]
        L.ff_timing_clock_probe.restype = i32
        L.ff_timing_clock_probe.argtypes = [P]
        L.ff_probe_mfma_ceiling.restype = i32
        L.ff_probe_mfma_ceiling.argtypes = [i32, i32, P, sz, P, C.POINTER(C.c_double), P]
        L.ff_timing_fused_stamps.restype = i32
        L.ff_timing_fused_stamps.argtypes = [P]
        L.ff_timing_reset.restype = i32
        L.ff_timing_read.restype = i32
        L.ff_timing_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _chk(st: int, what: str) -> None:
    if st != 0:
        raise FFError(st, what)


def layer_desc(layer, batch: int) -> LayerDesc:
    """From a workloads.Layer (or any object with the same attributes)."""
    kind = {"dense": 0, "conv": 1, "dwconv": 2}[layer.kind]
    return LayerDesc(kind, batch, layer.in_features, layer.out_features, layer.H, layer.W, layer.C_in, layer.C_out,
                     layer.ksize, layer.stride, layer.pad, layer.relu, layer.l2norm_out,
                     getattr(layer, "input_back", 0), {"ff": 0, "proj": 1}[getattr(layer, "role", "ff")],
                     {"none": 0, "identity": 1, "projection": 2}[getattr(layer, "skip", "none")])


def ff_pitch(cols: int) -> int:
    return int(lib().ff_pitch(cols))


def ff_pitch32(cols: int) -> int:
    return int(lib().ff_pitch32(cols))


def ff_stream_tag(step: int, layer: int, pass_idx: int, kind: int) -> int:
    return int(lib().ff_stream_tag(step, layer, pass_idx, kind))


def ff_status_string(st: int) -> str:
    return lib().ff_status_string(st).decode()


def ff_version() -> str:
    return lib().ff_version().decode()


def ff_goodness_shift(desc: LayerDesc) -> int:
    return int(lib().ff_goodness_shift(C.byref(desc)))


def ff_layer_dw_chunks(desc: LayerDesc) -> int:
    return int(lib().ff_layer_dw_chunks(C.byref(desc)))


def ff_layer_workspace_bytes(desc: LayerDesc) -> int:
    return int(lib().ff_layer_workspace_bytes(C.byref(desc)))


def ff_quantize(x, rows, cols, round_mode, seed, stream_tag, q, q_t, scale, ws) -> None:
    _chk(lib().ff_quantize(_ptr(x), rows, cols, round_mode, seed, stream_tag, _ptr(q), _ptr(q_t), _ptr(scale),
                           _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream()), "ff_quantize")


def ff_layer_forward(desc, a_q, w_q, acc, gsum_int, vmax, ws) -> None:
    _chk(lib().ff_layer_forward(C.byref(desc), _ptr(a_q), _ptr(w_q), _ptr(acc), _ptr(gsum_int), _ptr(vmax), _ptr(ws),
                                ws.numel() * ws.element_size() if ws is not None else 0, _stream()), "ff_layer_forward")


def ff_goodness_loss(desc, gsum_int, vmax, s_a, s_w, pass_sign, theta, goodness, coeff, loss_mean, next_amax) -> None:
    _chk(lib().ff_goodness_loss(C.byref(desc), _ptr(gsum_int), _ptr(vmax), _ptr(s_a), _ptr(s_w), pass_sign, theta,
                                _ptr(goodness), _ptr(coeff), _ptr(loss_mean), _ptr(next_amax), _stream()),
         "ff_goodness_loss")


def ff_layer_handoff(desc, acc, s_a, s_w, goodness, amax, round_mode, seed, stream_tag, q, q_t, scale) -> None:
    _chk(lib().ff_layer_handoff(C.byref(desc), _ptr(acc), _ptr(s_a), _ptr(s_w), _ptr(goodness), _ptr(amax), round_mode,
                                seed, stream_tag, _ptr(q), _ptr(q_t), _ptr(scale), _stream()), "ff_layer_handoff")


def ff_lookahead(coeff, n_layers, batch, lam, coeff_total) -> None:
    _chk(lib().ff_lookahead(_ptr(coeff), n_layers, batch, lam, _ptr(coeff_total), _stream()), "ff_lookahead")


def ff_layer_backward_local(desc, acc, vmax, s_a, s_w, coeff_total, round_mode, seed, stream_tag, a_q_t, gy_q_t, s_g,
                            dw_acc, ws) -> None:
    _chk(lib().ff_layer_backward_local(C.byref(desc), _ptr(acc), _ptr(vmax), _ptr(s_a), _ptr(s_w), _ptr(coeff_total),
                                       round_mode, seed, stream_tag, _ptr(a_q_t), _ptr(gy_q_t), _ptr(s_g), _ptr(dw_acc),
                                       _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
         "ff_layer_backward_local")


def ff_layer_backward_local_noalloc(desc, acc, vmax, s_a, s_w, coeff_total, round_mode, seed, stream_tag, a_q_t,
                                    gy_q_t, s_g, dw_acc) -> None:
    _chk(lib().ff_layer_backward_local_noalloc(C.byref(desc), _ptr(acc), _ptr(vmax), _ptr(s_a), _ptr(s_w),
                                               _ptr(coeff_total), round_mode, seed, stream_tag, _ptr(a_q_t),
                                               _ptr(gy_q_t), _ptr(s_g), _ptr(dw_acc), _stream()),
         "ff_layer_backward_local_noalloc")


def ff_noalloc_scratch_bytes() -> int:
    return int(lib().ff_noalloc_scratch_bytes())


def ff_chain_gradients(desc, acc, s_a, s_w, coeff, e_acc, s_h, s_w_up, lam, h, g, h_amax, g_amax) -> None:
    _chk(lib().ff_chain_gradients(C.byref(desc), _ptr(acc), _ptr(s_a), _ptr(s_w), _ptr(coeff), _ptr(e_acc), _ptr(s_h),
                                  _ptr(s_w_up), lam, _ptr(h), _ptr(g), _ptr(h_amax), _ptr(g_amax), _stream()),
         "ff_chain_gradients")


def ff_layer_input_grad(desc, h_q, w_q_t, e_acc, ws) -> None:
    _chk(lib().ff_layer_input_grad(C.byref(desc), _ptr(h_q), _ptr(w_q_t), _ptr(e_acc), _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
         "ff_layer_input_grad")


def ff_layer_update(desc, w_master, dw_pos, s_g_pos, s_a_pos, dw_neg, s_g_neg, s_a_neg, lr, total_samples, w_q, s_w,
                    ws) -> None:
    _chk(lib().ff_layer_update(C.byref(desc), _ptr(w_master), _ptr(dw_pos), _ptr(s_g_pos), _ptr(s_a_pos), _ptr(dw_neg),
                               _ptr(s_g_neg), _ptr(s_a_neg), lr, total_samples, _ptr(w_q), _ptr(s_w), _ptr(ws),
                               ws.numel() * ws.element_size() if ws is not None else 0, _stream()), "ff_layer_update")


class Net:
    """Host-side descriptors of a layer stack plus the device pointers of its trainable state.
    Holds references to the tensors so that the pointer arrays stay valid."""

    def __init__(self, layers: Sequence, batch: int, w_master: List[torch.Tensor], w_q: List[torch.Tensor],
                 s_w: List[torch.Tensor], train_layer: Optional[Sequence[int]] = None, lookahead: str = "coeff",
                 theta_layer: Optional[Sequence[float]] = None, launch_mode: str = "auto"):
        self.k = len(layers)
        self.batch = batch
        self._descs = (LayerDesc * self.k)(*[layer_desc(l, batch) for l in layers])
        self._mask = (C.c_int32 * self.k)(*[int(bool(f)) for f in train_layer]) if train_layer is not None else None
        self._theta = (C.c_float * self.k)(*[float(t) for t in theta_layer]) if theta_layer is not None else None
        if theta_layer is not None and len(theta_layer) != self.k:
            raise ValueError("theta_layer needs one threshold per layer")
        self.desc = NetDesc(self.k, batch, self._descs, self._mask, {"coeff": 0, "chain": 1}[lookahead], self._theta,
                            {"auto": 0, "kernels": 1, "fused": 2, "lanes": 3}[launch_mode])
        self.w_master, self.w_q, self.s_w = list(w_master), list(w_q), list(s_w)
        self._pm = (C.c_void_p * self.k)(*[t.data_ptr() for t in self.w_master])
        self._pq = (C.c_void_p * self.k)(*[t.data_ptr() for t in self.w_q])
        self._ps = (C.c_void_p * self.k)(*[t.data_ptr() for t in self.s_w])
        self.state = NetState(self._pm, self._pq, self._ps)

    def workspace_bytes(self) -> int:
        return ff_workspace_bytes(self)


def ff_workspace_bytes(net: Net) -> int:
    return int(lib().ff_workspace_bytes(C.byref(net.desc)))


def ff_train_step(net: Net, x_pos, x_neg, theta, lam, lr, seed, step, loss, goodness, ws) -> None:
    _chk(lib().ff_train_step(C.byref(net.desc), C.byref(net.state), _ptr(x_pos), _ptr(x_neg), theta, lam, lr, seed,
                             step, _ptr(loss), _ptr(goodness), _ptr(ws),
                             ws.numel() * ws.element_size() if ws is not None else 0, _stream()), "ff_train_step")


def ff_train_step_at(net: Net, x_pos, x_neg, theta, lam, lr, seed, step_dev, advance, loss, goodness, ws) -> None:
    _chk(lib().ff_train_step_at(C.byref(net.desc), C.byref(net.state), _ptr(x_pos), _ptr(x_neg), theta, lam, lr, seed,
                                _ptr(step_dev), int(advance), _ptr(loss), _ptr(goodness), _ptr(ws),
                                ws.numel() * ws.element_size() if ws is not None else 0, _stream()), "ff_train_step_at")


KERNEL_CLASSES = ("gemm_fwd", "gemm_dw", "quant_act", "quant_grad", "quant_w", "update", "absmax", "small", "im2col",
                  "residual", "dwconv", "chain", "fused")


def ff_timing_enable(on, classes: Optional[Sequence[str]] = None) -> None:
    """on: False = off, True = every kernel class, or restrict to the named `classes` (see KERNEL_CLASSES)."""
    mask = 0
    if on:
        mask = -1 if classes is None else sum(1 << KERNEL_CLASSES.index(c) for c in classes)
    _chk(lib().ff_timing_enable(mask), "ff_timing_enable")


def ff_timing_clock_probe(counters: Optional[torch.Tensor]) -> None:
    """counters: a zeroed int64 CUDA tensor of 16 elements (kept alive by the caller), or None to switch off."""
    _chk(lib().ff_timing_clock_probe(_ptr(counters)), "ff_timing_clock_probe")


def ff_probe_mfma_ceiling(operand_kind: int, iterations: int, sink: torch.Tensor, counters: Optional[torch.Tensor]) -> float:
    """Launches the register-resident MFMA loop on the current stream; returns the int8 operations of the launch."""
    ops = C.c_double(0.0)
    _chk(lib().ff_probe_mfma_ceiling(operand_kind, iterations, _ptr(sink), sink.numel() * sink.element_size(),
                                     _ptr(counters), C.byref(ops), _stream()), "ff_probe_mfma_ceiling")
    return ops.value


def ff_timing_fused_stamps(stamps: Optional[torch.Tensor]) -> None:
    """stamps: an int64 CUDA tensor of 32 elements (kept alive by the caller), or None to switch off."""
    _chk(lib().ff_timing_fused_stamps(_ptr(stamps)), "ff_timing_fused_stamps")


def ff_timing_reset() -> None:
    _chk(lib().ff_timing_reset(), "ff_timing_reset")


def ff_timing_read(kernel_class: int):
    """(total device milliseconds, launches) of one kernel class since the last reset."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _chk(lib().ff_timing_read(kernel_class, C.byref(ms), C.byref(n)), "ff_timing_read")
    return ms.value, n.value
