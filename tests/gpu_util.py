"""Helpers for the GPU parity tests: move seeded bf16-grid NumPy data to the device and back."""
import numpy as np
import torch


def dev_bf16(x: np.ndarray) -> torch.Tensor:
    """fp32 array whose values lie on the bf16 grid -> bf16 device tensor (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).cuda()


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def empty_bf16(*shape) -> torch.Tensor:
    return torch.empty(*shape, dtype=torch.bfloat16, device="cuda")


def scratch(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def nmax_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref|: the normalised-max error the tolerances are stated in."""
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref))) / max(denom, 1e-30)
