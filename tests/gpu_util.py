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


def attention_error_ratio(got, want, want_abs):
    """Largest |got - want| over the element-wise bound that follows from the kernel's bf16 arithmetic.

    bf16 keeps 8 significant bits: rounding to nearest has unit roundoff u = 2^-8.  The probabilities enter the
    P V product rounded to bf16 (relative error <= u each) and the result is rounded to bf16 once more, everything
    else is fp32: for output element (row, d)
        |err| <= u * (A + 2 |o|),   A = sum_j p_j |v_jd| / sum_j p_j,
    (A: the attention output over |V|, `want_abs`: the oracle run on the absolute values of V), plus the fp32
    accumulation, which the 5 % margin and the 1e-6 floor cover.  A key that is dropped or counted twice moves an
    element by p_j |v_jd|, which exceeds this bound wherever |v_jd| is large against the row's effective key count
    times u.  Returns the worst ratio (<= 1 passes; rounding errors of random sign stay well below the bound)."""
    bound = 2.0 ** -8 * (want_abs + 2.0 * np.abs(want)) * 1.05 + 1e-6
    return float((np.abs(got - want) / bound).max())
