"""Helpers shared by the GPU parity tests: host arrays <-> device tensors."""
import numpy as np
import torch

import oracle

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}     # max|err| <= TOL * ||out||_inf


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Stored host array (bf16 = uint16 bit patterns) -> GPU tensor, bits unchanged."""
    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda()
        return t.view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def to_host64(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> float64 host array, exactly."""
    return t.detach().to(torch.float64).cpu().numpy()


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


def assert_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max()
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err <= TOL[dtype] * scale, f"{what}: max|err|={err:.3e} > {TOL[dtype]:g}*{scale:.3e}"
    return err / scale
