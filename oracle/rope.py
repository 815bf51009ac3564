"""Oracle: rotary position embedding of the pruned query / key rows with their ORIGINAL position ids
(paper section 3.3, the sentence that introduces Eq. 7: the kept suffix tokens keep the logical
order of the full sequence through their RoPE position ids; the trailing-position ablation,
Table "Impact of trailing positional information", is about exactly this id).

The paper cites RoPE (Su et al., RoFormer) without restating it.  Definition used, in fp64:
for a row x of head dim D at position p, and frequencies theta_i = base^(-2i/D), i = 0..D/2-1,
every pair (x_a, x_b) is rotated by the angle p * theta_i:
        x_a' = x_a cos(p theta_i) - x_b sin(p theta_i)
        x_b' = x_b cos(p theta_i) + x_a sin(p theta_i)
with the pair (a, b) = (i, i + D/2) ("half" layout, the one the paper's models use: reading) or
(a, b) = (2i, 2i + 1) ("interleaved" layout, RoFormer's own).

Positions of the pruned rows: block row r sits at pos0 + r; kept suffix row j sits at
pos0 + K + keep_idx[j] -- NOT at pos0 + K + j: pruning must not shift the ids.
Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np


def rope_rotate(x: np.ndarray, positions: np.ndarray, base: float, interleaved: bool = False) -> np.ndarray:
    """x [..., T, D] float64, positions [T] integers -> rotated copy."""
    x = np.asarray(x, dtype=np.float64)
    T, D = x.shape[-2], x.shape[-1]
    assert D % 2 == 0 and len(positions) == T
    out = np.empty_like(x)
    for t in range(T):
        p = float(int(positions[t]))
        for i in range(D // 2):
            theta = float(base) ** (-2.0 * i / D)
            c, s = np.cos(p * theta), np.sin(p * theta)
            a, b = (2 * i, 2 * i + 1) if interleaved else (i, i + D // 2)
            out[..., t, a] = x[..., t, a] * c - x[..., t, b] * s
            out[..., t, b] = x[..., t, b] * c + x[..., t, a] * s
    return out


def pruned_positions(pos0: int, K: int, keep_idx) -> np.ndarray:
    """Position ids of the K block rows followed by the kept suffix rows."""
    keep_idx = np.asarray(keep_idx, dtype=np.int64).reshape(-1)
    return np.concatenate([pos0 + np.arange(K, dtype=np.int64), pos0 + K + keep_idx])


def rope_gathered(x_block: np.ndarray, x_suffix: np.ndarray, keep_idx, pos0: int, base: float,
                  interleaved: bool = False):
    """x_block [B,H,K,D], x_suffix [B,H,S,D] -> (rotated block [B,H,K,D], rotated kept rows [B,H,s,D]
    in keep_idx order).  Rows of the suffix that are not kept are not part of the result."""
    keep_idx = np.asarray(keep_idx, dtype=np.int64).reshape(-1)
    K = x_block.shape[-2]
    pos = pruned_positions(pos0, K, keep_idx)
    ob = rope_rotate(x_block, pos[:K], base, interleaved)
    if keep_idx.size:
        os_ = rope_rotate(np.asarray(x_suffix, dtype=np.float64)[..., keep_idx, :], pos[K:], base, interleaved)
    else:
        os_ = np.zeros(x_block.shape[:-2] + (0, x_block.shape[-1]))
    return ob, os_
