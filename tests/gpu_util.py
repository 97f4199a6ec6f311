"""Helpers shared by the GPU parity tests (test infrastructure)."""
import numpy as np
import torch

from oracle import fp6_oracle as O


def to_np16(t: torch.Tensor) -> np.ndarray:
    """GPU/CPU fp16 tensor -> numpy uint16 bit patterns (same bits)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def from_np16(a: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.float16).to(device)


def y_error(Y: torch.Tensor, Yref: np.ndarray):
    """(max abs err / max |Yref|, worst element-wise excess over 2e-3*|Yref| + 2e-3*rms)"""
    y = Y.detach().cpu().to(torch.float64).numpy()
    err = np.abs(y - Yref)
    scale = np.abs(Yref).max()
    rms = np.sqrt(np.mean(Yref ** 2))
    rel = err.max() / scale if scale > 0 else err.max()
    excess = (err - (2e-3 * np.abs(Yref) + 2e-3 * rms)).max()
    return rel, excess


def assert_y_close(Y: torch.Tensor, Yref: np.ndarray, what=""):
    assert torch.isfinite(Y).all(), what
    rel, excess = y_error(Y, Yref)
    # max relative error 2e-3 (fp32 accumulate, fp16 output): |Y - Yref| against the
    # largest |Yref| of the matrix, and element-wise against 2e-3*|Yref| + 2e-3*rms(Yref)
    assert rel <= 2e-3, (what, rel)
    assert excess <= 0, (what, excess)


def oracle_reference(W: torch.Tensor, X: torch.Tensor):
    """codes, scale bits, Y (float64) from the oracle for fp16 tensors W [N,K], X [M,K]."""
    codes, scales = O.quantize(to_np16(W))
    Y = O.linear(to_np16(X), codes, scales)
    return codes, scales, Y
