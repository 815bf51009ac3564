"""Oracle: the step on the other side of Eq. 4 -- the logits themselves.

Eq. 3 (section 3.1) writes a denoising step as z = f_theta(x); the last map inside f_theta is the
vocabulary projection of the final hidden state, z_i = W h_i (W [V, Hd], one row per token id;
the paper's models use no bias there), and Eq. 4 consumes z_i for the masked positions of the
active block only.  This module is that projection written out in float64, followed by the unmask
oracle on the resulting logits; nothing is rounded in between (a fused kernel never stores z).

Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np

from .unmask import confidence_unmask


def lm_head_logits(hidden, weight, rows_per_chunk: int = 8192):
    """hidden [..., Hd], weight [V, Hd] (any float dtype, widened exactly) -> logits [..., V] float64,
    logits[..., v] = sum_k hidden[..., k] * weight[v, k].

    The vocabulary is walked in slices only to bound the float64 copy of `weight`; every logit is
    one dot product over the whole of Hd, whichever slice it falls in.
    """
    h = np.asarray(hidden, dtype=np.float64)
    V, Hd = weight.shape
    assert h.shape[-1] == Hd, (h.shape, weight.shape)
    h2 = h.reshape(-1, Hd)
    z = np.empty((h2.shape[0], V), dtype=np.float64)
    for v0 in range(0, V, rows_per_chunk):
        Wc = np.asarray(weight[v0:v0 + rows_per_chunk], dtype=np.float64)
        z[:, v0:v0 + Wc.shape[0]] = h2 @ Wc.T
    return z.reshape(h.shape[:-1] + (V,))


def lm_head_unmask(hidden, weight, tokens, masked, tau0, alpha, **kw):
    """hidden [B,K,Hd], weight [V,Hd]: Eq. 3's last map for the masked positions, then Eq. 4, 10, 9, 5 and
    the exit tests exactly as oracle.unmask.confidence_unmask (same keyword arguments, same result dict).
    Rows of unmasked positions are never projected (their logits are left at zero and never looked at).
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    B, K, Hd = hidden.shape
    V = weight.shape[0]
    m = np.asarray(masked) != 0
    logits = np.zeros((B, K, V), dtype=np.float64)
    if m.any():
        logits[m] = lm_head_logits(hidden[m], weight)
    return confidence_unmask(logits, tokens, masked, tau0, alpha, **kw)
