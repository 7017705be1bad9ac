"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np

TOL_F32 = 2e-5   # max |y_gpu - y_oracle| / sum|x*w| per output


def normalised_error(y_gpu: np.ndarray, y_ref: np.ndarray, d: np.ndarray) -> float:
    """max over outputs of |y_gpu - y_ref| / D; outputs with D == 0 must be exactly 0."""
    y = y_gpu.astype(np.float64)
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    assert np.all(np.isfinite(y)), "non-finite output"
    zero = d == 0
    if zero.any():
        assert np.all(y[zero] == 0.0), "output with an empty/zero window is not exactly 0"
    if zero.all():
        return 0.0
    return float(np.max(np.abs(y - y_ref)[~zero] / d[~zero]))


def assert_f32_parity(y_gpu, y_ref, d, what=""):
    err = normalised_error(y_gpu, y_ref, d)
    assert err <= TOL_F32, f"{what}: normalised error {err:.3e} > {TOL_F32}"
    return err


def guarded_empty(torch, shape, dtype, guard=64, fill=None):
    """Output tensor carved out of a larger buffer whose margins hold a sentinel."""
    n = int(np.prod(shape))
    # keep the payload 256-byte aligned like a fresh allocation
    front = 256 // torch.empty((), dtype=dtype).element_size()
    buf = torch.empty(front + n + guard, dtype=dtype, device="cuda")
    sentinel = 12345 if fill is None else fill
    buf.fill_(sentinel)
    view = buf[front:front + n].view(shape)
    return buf, view, front, n, sentinel


def assert_guards_intact(buf, front, n, sentinel):
    assert bool((buf[:front] == sentinel).all()), "write before the output buffer"
    assert bool((buf[front + n:] == sentinel).all()), "write past the output buffer"
