"""Shared plumbing for the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch


def to_np32(t: torch.Tensor) -> np.ndarray:
    """Exact float32 copy on the host of a f32/bf16 tensor (bf16 widens without rounding)."""
    return t.detach().to("cpu").to(torch.float32).contiguous().numpy()


def bits_equal(gpu_w: torch.Tensor, oracle_w32: np.ndarray) -> bool:
    """Bit-for-bit comparison of a GPU f32/bf16 matrix with the oracle's float32 result."""
    got = to_np32(gpu_w)
    return np.array_equal(got.view(np.uint32), oracle_w32.view(np.uint32))


def first_mismatch(gpu_w: torch.Tensor, oracle_w32: np.ndarray) -> str:
    got = to_np32(gpu_w)
    bad = np.argwhere(got.view(np.uint32) != oracle_w32.view(np.uint32))
    if bad.size == 0:
        return "none"
    r, c = bad[0]
    return f"{len(bad)} mismatches, first at ({r},{c}): gpu={got[r, c]!r} oracle={oracle_w32[r, c]!r}"


def padded(t: torch.Tensor, pad_cols: int) -> torch.Tensor:
    """A view of shape t.shape inside a wider allocation (leading dimension > cols), canary filled."""
    rows, cols = t.shape
    big = torch.full((rows, cols + pad_cols), 7.0, dtype=t.dtype, device=t.device)
    big[:, :cols] = t
    return big[:, :cols]
