"""Pins for oracle.block_attention that do not re-use its own formula
(paper section 3.3, Eq. 8 and the paragraph on query / KV composition)."""
import math

import numpy as np
import pytest
import scipy.special

import workloads as wl
from oracle import block_attention


def _tiny(seed=0, B=2, Hq=2, Hkv=2, D=4, P=5, cap=7, K=3, S=6, keep=(0, 2, 5)):
    t = wl.make_custom_attention_inputs("fp32", B, Hq, Hkv, D, P, cap, K, S, keep, seed=seed)
    return {k: (wl.to_f64(v) if k != "keep_idx" else v) for k, v in t.items()}


def _brute(t, P, scale):
    """Scalar definition: no max subtraction, math.exp, nested loops, explicit row lists."""
    qb = t["q_block"]
    B, Hq, K, D = qb.shape
    Hkv = t["k_block"].shape[1]
    g = Hq // Hkv
    keep = [int(i) for i in t["keep_idx"]]
    out = np.zeros((B, Hq, K + len(keep), D))
    for b in range(B):
        for h in range(Hq):
            kv = h // g
            qrows = [qb[b, h, i] for i in range(K)] + [t["q_suffix"][b, h, j] for j in keep]
            krows = [t["k_cache"][b, kv, r] for r in range(P)] + [t["k_block"][b, kv, i] for i in range(K)] \
                + [t["k_suffix"][b, kv, j] for j in keep]
            vrows = [t["v_cache"][b, kv, r] for r in range(P)] + [t["v_block"][b, kv, i] for i in range(K)] \
                + [t["v_suffix"][b, kv, j] for j in keep]
            for qi, q in enumerate(qrows):
                w = []
                for k in krows:
                    dot = 0.0
                    for d in range(D):
                        dot += float(q[d]) * float(k[d])
                    w.append(math.exp(scale * dot))
                tot = sum(w)
                for d in range(D):
                    acc = 0.0
                    for wi, v in zip(w, vrows):
                        acc += wi * float(v[d])
                    out[b, h, qi, d] = acc / tot
    return out


def _call(t, P, scale=None, **kw):
    return block_attention(t["q_block"], t["q_suffix"], t["k_cache"], t["v_cache"], t["k_block"], t["v_block"],
                           t["k_suffix"], t["v_suffix"], t["keep_idx"], P, scale, **kw)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_tiny(seed):
    t = _tiny(seed)
    got = _call(t, 5, 0.37)
    want = _brute(t, 5, 0.37)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_brute_force_gqa_and_default_scale():
    t = _tiny(3, B=1, Hq=4, Hkv=2, D=8, P=4, cap=4, K=2, S=5, keep=(1, 4))
    got = _call(t, 4)
    want = _brute(t, 4, 1.0 / math.sqrt(8))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_keep_all_equals_full_context():
    """Keeping every suffix position reproduces dense attention over the physically
    concatenated [prefix | block | suffix] sequence (the paper's no-window case)."""
    B, Hq, Hkv, D, P, cap, K, S = 2, 4, 2, 16, 9, 12, 4, 11
    t = _tiny(5, B, Hq, Hkv, D, P, cap, K, S, keep=tuple(range(S)))
    got = _call(t, P)
    g = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            kv = h // g
            Q = np.concatenate([t["q_block"][b, h], t["q_suffix"][b, h]])
            Kf = np.concatenate([t["k_cache"][b, kv, :P], t["k_block"][b, kv], t["k_suffix"][b, kv]])
            Vf = np.concatenate([t["v_cache"][b, kv, :P], t["v_block"][b, kv], t["v_suffix"][b, kv]])
            A = scipy.special.softmax(Q @ Kf.T / math.sqrt(D), axis=1)   # library softmax
            np.testing.assert_allclose(got[b, h], A @ Vf, rtol=0, atol=1e-12)


def test_rows_sum_to_one():
    t = _tiny(7)
    _, probs = _call(t, 5, return_probs=True)
    for Pm in probs:
        assert Pm.shape == (3 + 3, 5 + 3 + 3)
        np.testing.assert_allclose(Pm.sum(axis=1), 1.0, rtol=0, atol=1e-12)
        assert (Pm >= 0).all()


def test_scale_zero_gives_mean_of_values():
    t = _tiny(8)
    got = _call(t, 5, 0.0)
    keep = t["keep_idx"]
    for b in range(2):
        for h in range(2):
            Vr = np.concatenate([t["v_cache"][b, h, :5], t["v_block"][b, h], t["v_suffix"][b, h][keep]])
            want = Vr.mean(axis=0)
            np.testing.assert_allclose(got[b, h], np.broadcast_to(want, got[b, h].shape), atol=1e-12)


def test_equal_values_pass_through():
    t = _tiny(9)
    v = np.arange(4, dtype=np.float64) - 1.5
    for k in ("v_cache", "v_block", "v_suffix"):
        t[k] = np.broadcast_to(v, t[k].shape).copy()
    got = _call(t, 5)
    np.testing.assert_allclose(got, np.broadcast_to(v, got.shape), atol=1e-12)


def test_single_key():
    t = _tiny(10, B=1, Hq=1, Hkv=1, D=4, P=0, cap=2, K=1, S=3, keep=())
    got = _call(t, 0)
    np.testing.assert_allclose(got[0, 0, 0], t["v_block"][0, 0, 0], atol=1e-15)
    assert got.shape == (1, 1, 1, 4)


def test_cache_rows_beyond_P_are_ignored():
    t = _tiny(11)
    a = _call(t, 5)
    t["k_cache"][:, :, 5:] = 1e6
    t["v_cache"][:, :, 5:] = -1e6
    b = _call(t, 5)
    np.testing.assert_array_equal(a, b)


def test_unkept_suffix_rows_are_ignored():
    t = _tiny(12)
    a = _call(t, 5)
    for k in ("q_suffix", "k_suffix", "v_suffix"):
        t[k][:, :, [1, 3, 4]] = 123.0
    b = _call(t, 5)
    np.testing.assert_array_equal(a, b)


def test_keep_order_permutes_suffix_rows_only():
    """Attention over keys is order-invariant: permuting keep_idx leaves the block rows
    unchanged and permutes the suffix output rows."""
    t = _tiny(13)
    a = _call(t, 5)
    t2 = dict(t)
    t2["keep_idx"] = np.array([5, 0, 2], dtype=np.int32)
    b = _call(t2, 5)
    np.testing.assert_allclose(a[:, :, :3], b[:, :, :3], atol=1e-13)
    np.testing.assert_allclose(a[:, :, 3 + 0], b[:, :, 3 + 1], atol=1e-13)
    np.testing.assert_allclose(a[:, :, 3 + 1], b[:, :, 3 + 2], atol=1e-13)
    np.testing.assert_allclose(a[:, :, 3 + 2], b[:, :, 3 + 0], atol=1e-13)


def test_gqa_equals_mha_on_repeated_kv():
    t = _tiny(14, B=1, Hq=6, Hkv=2, D=4, P=3, cap=3, K=2, S=4, keep=(0, 3))
    a = _call(t, 3)
    t2 = dict(t)
    for k in ("k_cache", "v_cache", "k_block", "v_block", "k_suffix", "v_suffix"):
        t2[k] = np.repeat(t[k], 3, axis=1)
    b = _call(t2, 3)
    np.testing.assert_allclose(a, b, atol=1e-14)


def test_value_of_one_hot_attention():
    """A query aligned with exactly one key and a huge scale selects that key's value row."""
    t = _tiny(15, B=1, Hq=1, Hkv=1, D=4, P=2, cap=2, K=2, S=2, keep=(1,))
    eye = np.eye(4)
    t["k_cache"][0, 0, :2] = eye[:2]
    t["k_block"][0, 0] = eye[2:4]
    t["k_suffix"][0, 0] = -eye[:2]
    t["q_block"][0, 0] = eye[[2, 0]]
    t["q_suffix"][0, 0, 1] = eye[3]
    got = _call(t, 2, 200.0)
    np.testing.assert_allclose(got[0, 0, 0], t["v_block"][0, 0, 0], atol=1e-12)   # q=e2 -> key row P+0
    np.testing.assert_allclose(got[0, 0, 1], t["v_cache"][0, 0, 0], atol=1e-12)   # q=e0 -> cache row 0
    np.testing.assert_allclose(got[0, 0, 2], t["v_block"][0, 0, 1], atol=1e-12)   # q=e3 -> key row P+1


def test_shift_invariance_of_scores():
    """Adding a constant vector to every key shifts each score row by a constant: output unchanged."""
    t = _tiny(16)
    a = _call(t, 5)
    # keys k -> k + u changes score(q,k) by q.u, constant over keys for a fixed query
    u = np.array([0.3, -0.2, 0.5, 0.1])
    t2 = dict(t)
    for k in ("k_cache", "k_block", "k_suffix"):
        t2[k] = t[k] + u
    b = _call(t2, 5)
    np.testing.assert_allclose(a, b, atol=1e-12)
