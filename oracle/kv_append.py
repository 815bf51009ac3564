"""Oracle: append the finished block's K/V to the prefix cache.

The prefix K/V is kept and reused across steps instead of being recomputed
(paper section 3.3, first paragraph of the dynamic-decoding part); when a block is
complete its K/V rows become rows P..P+K-1 of every layer's cache.  This is a
slice assignment; everything else in the caches stays bit-identical.
Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np


def kv_append(k_caches, v_caches, k_blocks, v_blocks, P, do_append=None):
    """caches [L,B,Hkv,cap,D], blocks [L,B,Hkv,K,D] (any dtype, copied bit-for-bit).
    do_append: optional [B] flags; sequences with 0 are left untouched.  Returns new caches."""
    k_out = np.array(k_caches, copy=True)
    v_out = np.array(v_caches, copy=True)
    L, B, Hkv, K, D = k_blocks.shape
    for b in range(B):
        if do_append is not None and do_append[b] == 0:
            continue
        k_out[:, b, :, P:P + K, :] = k_blocks[:, b]
        v_out[:, b, :, P:P + K, :] = v_blocks[:, b]
    return k_out, v_out
