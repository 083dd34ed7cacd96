"""Helpers shared by the GPU parity tests."""
import numpy as np

TOL = 1e-3          # |gpu - oracle| <= TOL * max(1, |oracle|), per element


def up(bits, device="cuda:0"):
    """fp16 bit patterns (numpy uint16) -> torch fp16 CUDA tensor with the same bits."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).to(device)


def scaled_err(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    return np.abs(gpu - ref) / np.maximum(1.0, np.abs(ref))


def assert_close(gpu, ref, what=""):
    assert gpu.shape == ref.shape, f"{what}: shape {gpu.shape} vs {ref.shape}"
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output"
    e = scaled_err(gpu, ref)
    i = np.unravel_index(np.argmax(e), e.shape)
    assert e[i] <= TOL, f"{what}: max scaled error {e[i]:.3e} at {i}: gpu {gpu[i]} oracle {ref[i]}"
    return float(e[i])


def padded(t, pitch):
    """A (H, W) view with row pitch `pitch` over a fresh canary-filled buffer holding t."""
    import torch
    H, W = t.shape
    buf = torch.full((H, pitch), 7.0 if t.dtype.is_floating_point else 7, dtype=t.dtype, device=t.device)
    buf[:, :W] = t
    return buf, buf[:, :W]
