"""Helpers for the GPU parity tests: moving bit patterns between numpy (oracle side) and torch
(HIP side).  No codec arithmetic here."""
import numpy as np
import torch

DEV = "cuda:0"


def u16_to_dev(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> bf16 device tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def dev_to_u16(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f32_to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def announce(*what):
    """Name the case before the GPU runs it, so that a lost box still tells which case it was."""
    print("[gpu-case]", *what, flush=True)
