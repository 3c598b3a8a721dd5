"""Helpers shared by the GPU parity tests: padded layouts <-> numpy, oracle-side reference data."""
import numpy as np
import torch

import paper_2506_22771_amd as ff


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pad8(q: np.ndarray) -> np.ndarray:
    """int8 [rows, cols] -> [rows, ff_pitch(cols)] with zero pad bytes."""
    rows, cols = q.shape
    out = np.zeros((rows, ff.ff_pitch(cols)), np.int8)
    out[:, :cols] = q
    return out


def pad32(a: np.ndarray) -> np.ndarray:
    rows, cols = a.shape
    out = np.zeros((rows, ff.ff_pitch32(cols)), np.int32)
    out[:, :cols] = a
    return out


def empty8(rows: int, cols: int, fill: int = 0x5A) -> torch.Tensor:
    """Device int8 buffer [rows, pitch(cols)] pre-filled with junk so that unwritten bytes show up."""
    return torch.full((rows, ff.ff_pitch(cols)), fill, dtype=torch.int8, device="cuda")


def empty32(rows: int, cols: int) -> torch.Tensor:
    return torch.full((rows, ff.ff_pitch32(cols)), 0x5A5A5A5A, dtype=torch.int32, device="cuda")


def scalar() -> torch.Tensor:
    return torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")


def workspace(nbytes: int = ff.WS_MIN_BYTES) -> torch.Tensor:
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def check_q(t: torch.Tensor, ref: np.ndarray, what: str) -> None:
    """Device padded int8 matrix equals the reference in the logical region and is zero in the pad."""
    got = t.cpu().numpy()
    rows, cols = ref.shape
    assert got.shape[0] == rows, what
    np.testing.assert_array_equal(got[:, :cols], ref, err_msg=what)
    assert not got[:, cols:].any(), f"{what}: pad bytes not zero"


def rel_close(got, ref, tol=1e-5):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return np.all(np.abs(got - ref) <= tol * np.abs(ref) + 1e-38)


def pad_nhwc(a: np.ndarray) -> np.ndarray:
    """int8 [B, H, W, C] -> [B, H, W, ff_pitch(C)] with zero pad channels."""
    B, H, W, C = a.shape
    out = np.zeros((B, H, W, ff.ff_pitch(C)), np.int8)
    out[..., :C] = a
    return out
