"""Pins for the vocabulary-projection oracle (oracle/lm_head.py: the last map of Eq. 3 feeding Eq. 4).
None re-uses its matrix product: scalar loops with Python floats, projections whose result can be read
off the operands (identity, one-hot rows and columns), closed-form confidences, exact integer
arithmetic, and the chain into the unmask oracle on logits formed by the scalar loops."""
import math
from fractions import Fraction

import numpy as np

import workloads as wl
from oracle import confidence_unmask, lm_head_logits, lm_head_unmask


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=seed))


def _loops(h, W):
    rows, Hd = h.shape
    V = W.shape[0]
    z = [[0.0] * V for _ in range(rows)]
    for r in range(rows):
        for v in range(V):
            acc = 0.0
            for k in range(Hd):
                acc += float(h[r, k]) * float(W[v, k])
            z[r][v] = acc
    return np.array(z)


def test_scalar_loops_on_tiny_inputs():
    g = _rng(11)
    h, W = g.standard_normal((5, 7)), g.standard_normal((9, 7))      # V != Hd != rows: a transposed
    z = lm_head_logits(h, W)                                          # operand cannot even be formed
    assert z.shape == (5, 9)
    assert np.allclose(z, _loops(h, W), rtol=0, atol=1e-13)


def test_square_projection_is_not_transposed():
    # V == Hd: W and its transpose have the same shape, only the values tell them apart.
    # Row v of W is the template of token v: W = [[1,2],[0,1]], h = (1,0) -> z = (1*1+2*0, 0) = (1, 0);
    # the transposed product would give (1, 2).
    W = np.array([[1.0, 2.0], [0.0, 1.0]])
    assert np.array_equal(lm_head_logits(np.array([1.0, 0.0]), W), [1.0, 0.0])
    assert np.array_equal(lm_head_logits(np.array([0.0, 1.0]), W), [2.0, 1.0])


def test_identity_one_hot_rows_and_columns():
    g = _rng(5)
    h = g.standard_normal((2, 3, 6))
    assert np.array_equal(lm_head_logits(h, np.eye(6)), h)                       # W = I: logits are the hidden state
    W = g.standard_normal((10, 6))
    for k in range(6):                                                             # h = e_k reads column k of W
        e = np.zeros(6); e[k] = 1.0
        assert np.array_equal(lm_head_logits(e, W), W[:, k])
    Wsel = np.zeros((4, 6)); Wsel[2, 5] = 3.0                                      # a single entry: z_2 = 3 h_5
    z = lm_head_logits(h, Wsel)
    assert np.array_equal(z[..., 2], 3.0 * h[..., 5]) and not z[..., [0, 1, 3]].any()


def test_exact_integer_arithmetic_across_slices():
    # small integers: every product and sum is exact in float64, so the result must equal rational arithmetic;
    # the slice length is set below V so that several slices and a ragged last one are walked
    g = _rng(3)
    h = g.integers(-9, 10, size=(3, 33)).astype(np.float64)
    W = g.integers(-9, 10, size=(29, 33)).astype(np.float64)
    z = lm_head_logits(h, W, rows_per_chunk=8)
    for r in range(3):
        for v in range(29):
            want = sum(Fraction(int(h[r, k])) * Fraction(int(W[v, k])) for k in range(33))
            assert Fraction(z[r, v]) == want
    assert np.array_equal(z, lm_head_logits(h, W, rows_per_chunk=1000))


def test_bf16_operands_are_widened_exactly():
    w = wl.WORKLOADS["small_bf16"]
    t = wl.make_lm_head_inputs(w, seed=2, V=40, Hd=64)
    h32, W32 = wl.bf16_bits_to_f32(t["hidden"]), wl.bf16_bits_to_f32(t["lm_weight"])
    z = lm_head_logits(h32, W32)
    assert z.dtype == np.float64
    assert np.allclose(z[1, 3], _loops(h32[1, 3:4].astype(np.float64), W32.astype(np.float64))[0], rtol=0, atol=1e-12)


def test_closed_form_confidence_through_the_projection():
    # h = (1,1,1,1), W rows = a_v/4 * (1,1,1,1): z_v = a_v.  a = (ln 3, 0, 0) -> softmax max = 3/5, id 0.
    h = np.ones((1, 2, 4))
    W = np.outer([math.log(3.0), 0.0, 0.0], np.full(4, 0.25))
    r = lm_head_unmask(h, W, np.full((1, 2), -1), np.array([[1, 0]], dtype=np.uint8), tau0=0.5, alpha=0.0)
    assert abs(r["confidence"][0, 0] - 0.6) < 1e-15 and r["xhat"][0, 0] == 0
    assert np.isnan(r["confidence"][0, 1])                     # the unmasked position is never projected / ranked
    assert r["n_committed"][0] == 1 and r["block_done"][0] == 1 and r["tokens"][0, 0] == 0
    # tau0 above 0.6 and nothing else masked: the fallback still commits it
    r = lm_head_unmask(h, W, np.full((1, 2), -1), np.array([[1, 0]], dtype=np.uint8), tau0=0.9, alpha=0.0)
    assert r["fallback"][0] == 1 and r["n_committed"][0] == 1


def test_chain_equals_unmask_on_loop_logits_and_skips_unmasked_rows():
    g = _rng(9)
    B, K, Hd, V = 2, 6, 5, 12
    h, W = g.standard_normal((B, K, Hd)), 2.0 * g.standard_normal((V, Hd))
    masked = np.array([[1, 0, 1, 1, 0, 1], [0, 0, 1, 0, 0, 0]], dtype=np.uint8)
    tokens = np.where(masked != 0, -1, 7)
    z = _loops(h.reshape(-1, Hd), W).reshape(B, K, V)
    want = confidence_unmask(z, tokens, masked, 0.3, 0.5, eos_id=4, tau_eos=0.2)
    got = lm_head_unmask(h, W, tokens, masked, 0.3, 0.5, eos_id=4, tau_eos=0.2)
    for k in ("tokens", "masked", "n_committed", "block_done", "eos_seen", "xhat", "fallback"):
        assert np.array_equal(got[k], want[k]), k
    assert np.allclose(got["confidence"], want["confidence"], rtol=1e-12, equal_nan=True)
    # hidden states of unmasked positions cannot matter: poison them
    h2 = h.copy(); h2[masked == 0] = np.nan
    got2 = lm_head_unmask(h2, W, tokens, masked, 0.3, 0.5, eos_id=4, tau_eos=0.2)
    assert np.array_equal(got2["tokens"], want["tokens"]) and np.array_equal(got2["n_committed"], want["n_committed"])


def test_generated_projection_follows_the_logit_law():
    # the recipe promises logits ~ N(0, logit_std^2) with one boosted token per row standing out at 18..26
    w = wl.WORKLOADS["small_bf16"]
    t = wl.make_lm_head_inputs(w, seed=0, V=3000, Hd=256)
    z = lm_head_logits(wl.bf16_bits_to_f32(t["hidden"]), wl.bf16_bits_to_f32(t["lm_weight"]))
    assert abs(z.std() - w.logit_std) < 0.25
    top = z.max(axis=-1)
    assert (top > 17.5).all() and (top < 26.5).all()
