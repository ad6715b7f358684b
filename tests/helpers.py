"""Shared test helpers: moving tensors between torch (device) and numpy (oracle)."""
import numpy as np
import torch


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> numpy with the oracle's dtypes (bf16 -> uint16 bits, int64 -> uint64...)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype == torch.int64:
        return t.numpy().view(np.uint64).copy()
    if t.dtype == torch.int16:
        return t.numpy().view(np.uint16).copy()
    return t.numpy().copy()


def bits32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_f32_equal(got: np.ndarray, want: np.ndarray, what: str, rel: float = 1e-6):
    """fp32 state must agree within max relative error ``rel``; report bit-exactness too.

    The arithmetic is the same sequence of individually rounded fp32 operations
    on both sides, so the values are expected to be bit-identical; the stated
    bar is 1e-6 relative.  NaNs must sit in the same places.
    """
    got = np.asarray(got, dtype=np.float32)
    want = np.asarray(want, dtype=np.float32)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN pattern differs"
    ok = ~nan_g
    g64, w64 = got[ok].astype(np.float64), want[ok].astype(np.float64)
    fin = np.isfinite(w64)
    assert np.array_equal(g64[~fin], w64[~fin]), f"{what}: infinities differ"
    diff = np.abs(g64[fin] - w64[fin])
    denom = np.maximum(np.abs(w64[fin]), np.finfo(np.float32).tiny)
    worst = float((diff / denom).max()) if diff.size else 0.0
    assert worst <= rel, f"{what}: max relative error {worst:.3e} > {rel:.1e}"
    return bool(np.array_equal(bits32(got)[ok], bits32(want)[ok]))


def strided_rows(N: int, d: int, stride: int, dtype, device, fill=None) -> torch.Tensor:
    """``[N, d]`` view into a ``[N, stride]`` buffer (padding poisoned so stray writes show)."""
    buf = torch.empty((N, stride), dtype=dtype, device=device)
    if dtype in (torch.float32, torch.bfloat16):
        buf.fill_(float("nan") if fill is None else fill)
    else:
        buf.fill_(-1 if fill is None else fill)
    return buf[:, :d]
