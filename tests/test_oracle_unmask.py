"""Pins for oracle.confidence_unmask (paper Eq. 4, 5, 9, 10, block termination, early exit)
that do not re-use its own formulas: golden closed forms, scalar brute force, invariants."""
import math
import os

import numpy as np
import pytest
import scipy.special

import workloads as wl
from oracle import confidence_unmask, dynamic_threshold, row_confidence

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_threshold_golden_eq10():
    for tau0, alpha, m, K, em, et, tau in _rows("eq10_threshold.txt"):
        got = dynamic_threshold(float(tau0), float(alpha), int(m), int(K), int(em), int(et))
        assert abs(got - float(tau)) < 1e-12, (tau0, alpha, m, K, got, tau)


def test_alpha_zero_is_static_threshold():
    for m in range(1, 33):
        assert dynamic_threshold(0.9, 0.0, m, 32) == 0.9


def test_threshold_monotone_in_mask_ratio():
    vals = [dynamic_threshold(0.9, 0.3, m, 32) for m in range(1, 33)]
    assert all(a < b for a, b in zip(vals, vals[1:]))
    assert vals[-1] == pytest.approx(0.9, abs=1e-15)


def test_confidence_golden_eq4():
    for case, a, V, j, c, xhat in _rows("eq4_confidence.txt"):
        a, V, j, c, xhat = float(a), int(V), int(j), float(c), int(xhat)
        z = np.zeros(V) if case == "one_hot" else np.full(V, a)
        if case == "one_hot":
            z[j] = a
        gc, gx, _ = row_confidence(z)
        assert gx == xhat
        assert abs(gc - c) < 1e-12 * max(1.0, c)


def test_row_confidence_brute_force():
    g = np.random.default_rng(0)
    for _ in range(50):
        V = int(g.integers(1, 17))
        z = g.normal(0, 3, size=V)
        e = [math.exp(float(v)) for v in z]
        p = [v / sum(e) for v in e]
        best = 0
        for j in range(V):
            if p[j] > p[best]:
                best = j
        c, xh, gap = row_confidence(z)
        assert xh == best
        assert abs(c - p[best]) < 1e-13
        if V > 1:
            second = sorted(p)[-2]
            assert abs(gap - (p[best] - second)) < 1e-13


def test_row_confidence_matches_library_softmax():
    g = np.random.default_rng(1)
    z = g.normal(0, 4, size=5000)
    c, xh, _ = row_confidence(z)
    p = scipy.special.softmax(z)
    assert xh == int(np.argmax(p))
    assert abs(c - p.max()) < 1e-14


def test_argmax_tie_takes_lowest_id():
    z = np.zeros(10)
    z[[7, 3, 9]] = 5.0
    c, xh, gap = row_confidence(z)
    assert xh == 3
    assert gap == pytest.approx(0.0, abs=1e-16)
    assert c == pytest.approx(math.exp(5) / (3 * math.exp(5) + 7), rel=1e-14)


def test_large_logits_do_not_overflow():
    z = np.array([1000.0, 999.0, -1000.0])
    c, xh, _ = row_confidence(z)
    assert xh == 0 and c == pytest.approx(1 / (1 + math.exp(-1)), rel=1e-14)


def _state(B=3, K=8, V=12, seed=0, std=3.0):
    g = np.random.default_rng(seed)
    logits = g.normal(0, std, size=(B, K, V))
    masked = (g.uniform(size=(B, K)) < 0.6).astype(np.uint8)
    tokens = g.integers(0, V, size=(B, K))
    tokens[masked != 0] = wl.MASK_TOKEN
    return logits, tokens, masked


def _brute_step(logits, tokens, masked, tau0, alpha, eos_id, tau_eos, eos_seen):
    """Independent scalar re-statement of Eq. 4, 10, 9, 5 used as a cross-check."""
    B, K, V = logits.shape
    tokens = tokens.copy(); masked = masked.copy(); eos = list(eos_seen)
    ncom, done = [0] * B, [0] * B
    for b in range(B):
        idx = [i for i in range(K) if masked[b, i]]
        if not idx:
            done[b] = 1
            continue
        cs, xs = {}, {}
        for i in idx:
            e = [math.exp(float(v) - float(max(logits[b, i]))) for v in logits[b, i]]
            p = [v / sum(e) for v in e]
            xs[i] = max(range(V), key=lambda j: (p[j], -j))
            cs[i] = p[xs[i]]
        r = len(idx) / K
        tau = tau0 * (1 - alpha * (1 - r))
        sel = [i for i in idx if cs[i] >= tau]
        if not sel:
            sel = [max(idx, key=lambda i: (cs[i], -i))]
        for i in sel:
            tokens[b, i] = xs[i]; masked[b, i] = 0
            if eos_id >= 0 and xs[i] == eos_id and cs[i] >= tau_eos:
                eos[b] = 1
        ncom[b] = len(sel); done[b] = int(len(sel) == len(idx))
    return tokens, masked, ncom, done, eos


@pytest.mark.parametrize("seed,tau0,alpha", [(0, 0.9, 0.3), (1, 0.5, 0.7), (2, 0.3, 0.0), (3, 0.9, 0.6)])
def test_step_brute_force(seed, tau0, alpha):
    logits, tokens, masked = _state(seed=seed)
    got = confidence_unmask(logits, tokens, masked, tau0, alpha, eos_id=2, tau_eos=0.4)
    t, m, n, d, e = _brute_step(logits, tokens, masked, tau0, alpha, 2, 0.4, [0, 0, 0])
    np.testing.assert_array_equal(got["tokens"], t)
    np.testing.assert_array_equal(got["masked"], m)
    np.testing.assert_array_equal(got["n_committed"], n)
    np.testing.assert_array_equal(got["block_done"], d)
    np.testing.assert_array_equal(got["eos_seen"], e)


def test_tau_zero_commits_every_masked_position():
    logits, tokens, masked = _state(seed=4)
    got = confidence_unmask(logits, tokens, masked, 0.0, 0.3)
    assert (got["masked"] == 0).all()
    np.testing.assert_array_equal(got["n_committed"], masked.sum(axis=1))
    assert (got["block_done"] == 1).all()
    assert (got["fallback"] == 0)[masked.sum(axis=1) > 0].all()
    # committed ids are the row argmaxes
    for b, i in zip(*np.nonzero(masked)):
        assert got["tokens"][b, i] == int(np.argmax(logits[b, i]))


def test_tau_above_one_commits_exactly_one_per_sequence():
    logits, tokens, masked = _state(seed=5)
    masked[1] = 0
    tokens[1] = 7
    got = confidence_unmask(logits, tokens, masked, 1.5, 0.0)
    m = masked.sum(axis=1)
    np.testing.assert_array_equal(got["n_committed"], (m > 0).astype(int))
    assert got["n_committed"][1] == 0 and got["block_done"][1] == 1
    for b in (0, 2):
        i = int(np.nanargmax(got["confidence"][b]))
        assert got["masked"][b, i] == 0 and masked[b, i] == 1
        assert got["fallback"][b] == 1


def test_fallback_tie_takes_the_lowest_position():
    """Two masked positions with identical logit rows have identical confidence; when no position
    reaches the threshold the single fallback commit goes to the lower one (a stated reading)."""
    logits, tokens, masked = _state(B=1, K=6, V=9, seed=11)
    masked[:] = 0
    masked[0, [1, 2, 4]] = 1
    logits[0, 4] = logits[0, 2]                     # positions 2 and 4 tie ...
    logits[0, 1] = logits[0, 2] * 0.5               # ... and position 1 is flatter, hence less confident
    got = confidence_unmask(logits, tokens, masked, 1.5, 0.0)
    assert got["confidence"][0, 2] == got["confidence"][0, 4] > got["confidence"][0, 1]
    assert got["n_committed"][0] == 1 and got["fallback"][0] == 1
    assert got["masked"][0].tolist() == [0, 1, 0, 0, 1, 0]


def test_committed_never_remask_and_unmasked_untouched():
    logits, tokens, masked = _state(seed=6)
    got = confidence_unmask(logits, tokens, masked, 0.6, 0.3)
    was_unmasked = masked == 0
    np.testing.assert_array_equal(got["tokens"][was_unmasked], tokens[was_unmasked])
    assert (got["masked"][was_unmasked] == 0).all()           # never re-masked
    assert ((got["masked"] != 0) <= (masked != 0)).all()      # mask set only shrinks
    still = got["masked"] != 0
    np.testing.assert_array_equal(got["tokens"][still], tokens[still])
    assert np.isnan(got["confidence"][was_unmasked]).all()


def test_repeated_fallback_terminates_in_m_steps():
    logits, tokens, masked = _state(seed=7, B=2, K=6)
    masked[:] = 1
    tokens[:] = wl.MASK_TOKEN
    steps = 0
    counts = []
    while masked.any():
        out = confidence_unmask(logits, tokens, masked, 2.0, 0.0)
        tokens, masked = out["tokens"], out["masked"]
        counts.append(int(masked.sum()))
        steps += 1
        assert steps <= 6
    assert steps == 6
    assert counts == sorted(counts, reverse=True)
    assert (out["block_done"] == 1).all()


def test_block_done_iff_no_mask_left():
    for seed in range(8):
        logits, tokens, masked = _state(seed=seed, std=6.0)
        out = confidence_unmask(logits, tokens, masked, 0.9, 0.3)
        np.testing.assert_array_equal(out["block_done"], (out["masked"].sum(axis=1) == 0).astype(np.uint8))


def test_threshold_uses_state_before_commit_and_per_sequence():
    logits, tokens, masked = _state(seed=9)
    out = confidence_unmask(logits, tokens, masked, 0.9, 0.3)
    for b in range(3):
        m = int(masked[b].sum())
        if m:
            assert out["tau"][b] == pytest.approx(0.9 * (1 - 0.3 * (1 - m / 8)), abs=1e-15)


def test_query_wide_mask_ratio_reading():
    logits, tokens, masked = _state(seed=10)
    out = confidence_unmask(logits, tokens, masked, 0.9, 0.3, extra_masked=8, extra_total=8)
    for b in range(3):
        m = int(masked[b].sum())
        if m:
            assert out["tau"][b] == pytest.approx(0.9 * (1 - 0.3 * (1 - (m + 8) / 16)), abs=1e-15)


def test_ge_comparison_at_exact_threshold():
    # two logits (0, 0) give c = 0.5 exactly; tau0 = 0.5, alpha = 0 -> committed by ">="
    logits = np.zeros((1, 2, 2))
    logits[0, 1] = [0.0, -50.0]
    tokens = np.full((1, 2), wl.MASK_TOKEN)
    masked = np.ones((1, 2), dtype=np.uint8)
    out = confidence_unmask(logits, tokens, masked, 0.5, 0.0)
    assert out["n_committed"][0] == 2 and out["fallback"][0] == 0


def test_eos_flag_sticky_and_conditional():
    V = 6
    logits = np.full((2, 2, V), -20.0)
    logits[0, 0, 4] = 10.0      # sequence 0 commits token 4 (= eos) with c ~ 1
    logits[0, 1, 1] = 10.0
    logits[1, 0, 2] = 10.0      # sequence 1 commits non-eos tokens
    logits[1, 1, 3] = 10.0
    tokens = np.full((2, 2), wl.MASK_TOKEN)
    masked = np.ones((2, 2), dtype=np.uint8)
    out = confidence_unmask(logits, tokens, masked, 0.9, 0.0, eos_id=4)
    np.testing.assert_array_equal(out["eos_seen"], [1, 0])
    # sticky: a later call that commits nothing keeps the flag
    out2 = confidence_unmask(logits, out["tokens"], out["masked"], 0.9, 0.0, eos_id=4, eos_seen=out["eos_seen"])
    np.testing.assert_array_equal(out2["eos_seen"], [1, 0])
    # disabled with eos_id < 0
    out3 = confidence_unmask(logits, tokens, masked, 0.9, 0.0, eos_id=-1)
    np.testing.assert_array_equal(out3["eos_seen"], [0, 0])
    # eos committed through the fallback with low confidence does not set the flag
    flat = np.zeros((1, 1, V)); flat[0, 0, 4] = 0.1
    out4 = confidence_unmask(flat, np.full((1, 1), wl.MASK_TOKEN), np.ones((1, 1), dtype=np.uint8), 0.9, 0.0, eos_id=4)
    assert out4["tokens"][0, 0] == 4 and out4["eos_seen"][0] == 0


def test_padded_row_stride_is_ignored():
    logits, tokens, masked = _state(seed=11, V=12)
    pad = np.concatenate([logits, np.full((3, 8, 5), 100.0)], axis=2)
    a = confidence_unmask(logits, tokens, masked, 0.7, 0.3)
    b = confidence_unmask(pad, tokens, masked, 0.7, 0.3, V=12)
    np.testing.assert_array_equal(a["tokens"], b["tokens"])
    np.testing.assert_array_equal(a["masked"], b["masked"])


def test_block_size_limits():
    """K = 1 (autoregressive-like) always commits its single masked position; K = L behaves the same rule-wise."""
    logits = np.random.default_rng(3).normal(size=(4, 1, 9))
    tokens = np.full((4, 1), wl.MASK_TOKEN)
    masked = np.ones((4, 1), dtype=np.uint8)
    out = confidence_unmask(logits, tokens, masked, 0.99, 0.5)
    assert (out["n_committed"] == 1).all() and (out["block_done"] == 1).all()
