"""Helpers shared by the GPU parity tests: tensors in, numpy out."""
import numpy as np
import torch

import paper_2409_12517_amd as ssg

DEV = "cuda:0"


def has_gpu() -> bool:
    return torch.cuda.is_available()


def dev(t: torch.Tensor) -> torch.Tensor:
    return t.to(DEV).contiguous()


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).numpy()


def u8(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def scalar(t: torch.Tensor) -> np.float32:
    return np.float32(t.detach().cpu().numpy().reshape(-1)[0])


def empty_u8(*shape):
    return torch.empty(*shape, dtype=torch.uint8, device=DEV)


def empty_f32(*shape):
    return torch.empty(*shape, dtype=torch.float32, device=DEV)


def bf16_ulp(ref: np.ndarray) -> np.ndarray:
    """Spacing of bf16 at the magnitude of ref (8 significant bits)."""
    a = np.maximum(np.abs(ref), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def assert_close_gemm(got: np.ndarray, ref: np.ndarray, bf16_out: bool, what: str = ""):
    """The stated bar: max|err| <= 2e-3 * max|ref| for fp32 outputs, plus one bf16 ulp for bf16 outputs."""
    tol = 2e-3 * np.abs(ref).max()
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = tol + (bf16_ulp(ref) if bf16_out else 0.0)
    worst = (err - bound).max()
    assert worst <= 0, f"{what}: max err {err.max():.4g}, tol {tol:.4g}, max|ref| {np.abs(ref).max():.4g}"
