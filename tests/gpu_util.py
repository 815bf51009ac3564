"""Helpers for the GPU parity tests: move generated numpy tensors to the device and back."""
import numpy as np
import torch

import workloads as wl


def to_dev(x: np.ndarray):
    if x.dtype == np.uint16:     # bf16 bit patterns
        return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x).cuda()


def to_f64_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def attn_to_dev(t):
    return {k: to_dev(v) for k, v in t.items()}


def attn_to_f64(t):
    return {k: (wl.to_f64(v) if k != "keep_idx" else v) for k, v in t.items()}
