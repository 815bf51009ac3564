"""Oracle: bidirectional attention of (active block + kept suffix) queries over
(prefix cache + active block + kept suffix) keys/values.

Follows the paper's section 3.3: the pruned input is prefix U current U kept
suffix (Eq. 8); the queries are the current block together with the kept suffix
and they attend to the K/V of that whole pruned sequence, with no mask
(bidirectional attention, sections 1 and 3.2).  Given the operands this is
exactly dense softmax attention, so the oracle is that definition in float64.
Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np


def compose_rows(cache, block, suffix, keep_idx, P):
    """Rows of the pruned sequence for one head: cache[0:P] ++ block ++ suffix[keep_idx]  (Eq. 8)."""
    parts = []
    if cache is not None:
        parts.append(cache[:P])
    parts.append(block)
    parts.append(suffix[keep_idx])
    return np.concatenate(parts, axis=0)


def block_attention(q_block, q_suffix, k_cache, v_cache, k_block, v_block, k_suffix, v_suffix,
                    keep_idx, P, scale=None, return_probs=False):
    """All arguments float64 arrays in [B,H,T,D] layout (see workloads.py); keep_idx int array.

    Returns out[B,Hq,K+s,D] float64: block rows first, then kept-suffix rows in
    keep_idx order.  Query head hq reads KV head hq // (Hq // Hkv).
    """
    q_block = np.asarray(q_block, dtype=np.float64)
    B, Hq, K, D = q_block.shape
    Hkv = k_block.shape[1]
    assert Hq % Hkv == 0
    g = Hq // Hkv
    keep_idx = np.asarray(keep_idx, dtype=np.int64).reshape(-1)
    s = keep_idx.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty((B, Hq, K + s, D), dtype=np.float64)
    probs = [] if return_probs else None
    for b in range(B):
        for hq in range(Hq):
            kvh = hq // g
            Q = compose_rows(None, q_block[b, hq], q_suffix[b, hq], keep_idx, 0)           # [Nq, D]
            Kr = compose_rows(k_cache[b, kvh], k_block[b, kvh], k_suffix[b, kvh], keep_idx, P)  # [Nkv, D]
            Vr = compose_rows(v_cache[b, kvh], v_block[b, kvh], v_suffix[b, kvh], keep_idx, P)
            Sc = scale * (Q.astype(np.float64) @ Kr.astype(np.float64).T)                   # [Nq, Nkv]
            Sc = Sc - Sc.max(axis=1, keepdims=True)
            E = np.exp(Sc)
            Pm = E / E.sum(axis=1, keepdims=True)
            out[b, hq] = Pm @ Vr.astype(np.float64)
            if return_probs:
                probs.append(Pm)
    if return_probs:
        return out, probs
    return out
