"""Pins for oracle.kv_append (paper section 3.3: prefix K/V is kept and reused)."""
import numpy as np

import workloads as wl
from oracle import kv_append


def test_append_rows_and_nothing_else():
    t = wl.make_append_inputs("bf16", 3, 2, 2, 8, 4, 16, seed=0)
    P = 5
    k, v = kv_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], P)
    for L in range(3):
        for b in range(2):
            for h in range(2):
                for r in range(16):
                    if P <= r < P + 4:
                        assert (k[L, b, h, r] == t["k_blocks"][L, b, h, r - P]).all()
                        assert (v[L, b, h, r] == t["v_blocks"][L, b, h, r - P]).all()
                    else:
                        assert (k[L, b, h, r] == t["k_caches"][L, b, h, r]).all()
                        assert (v[L, b, h, r] == t["v_caches"][L, b, h, r]).all()
    assert k.dtype == t["k_caches"].dtype


def test_do_append_flags():
    t = wl.make_append_inputs("fp32", 2, 3, 1, 4, 2, 6, seed=1)
    k, v = kv_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], 4, do_append=np.array([1, 0, 1], np.uint8))
    assert (k[:, 1] == t["k_caches"][:, 1]).all() and (v[:, 1] == t["v_caches"][:, 1]).all()
    assert (k[:, 0, :, 4:6] == t["k_blocks"][:, 0]).all()
    assert (v[:, 2, :, 4:6] == t["v_blocks"][:, 2]).all()


def test_inputs_not_modified():
    t = wl.make_append_inputs("fp32", 1, 1, 1, 4, 2, 4, seed=2)
    before = t["k_caches"].copy()
    kv_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], 0)
    assert (t["k_caches"] == before).all()


def test_appended_rows_compose_like_the_block_operand():
    """Rows P..P+K-1 read back from the appended cache equal the block operand, so the next
    block's prefix is [old prefix | finished block] (consistency with the attention operands)."""
    B, Hq, Hkv, D, P, cap, K, S = 1, 2, 2, 4, 3, 8, 2, 3
    t = wl.make_custom_attention_inputs("fp32", B, Hq, Hkv, D, P, cap, K, S, (0, 2), seed=4)
    kc, vc = kv_append(t["k_cache"][None], t["v_cache"][None], t["k_block"][None], t["v_block"][None], P)
    for h in range(Hkv):
        want_k = np.concatenate([t["k_cache"][0, h, :P], t["k_block"][0, h]])
        want_v = np.concatenate([t["v_cache"][0, h, :P], t["v_block"][0, h]])
        assert (kc[0, 0, h, :P + K] == want_k).all()
        assert (vc[0, 0, h, :P + K] == want_v).all()
