"""GPU parity: sdllm_confidence_unmask against the fp64 oracle (paper Eq. 4, 5, 9, 10, block
termination, EOS early exit).

Bar: committed token ids and the unmask set bit-exact, except positions whose oracle confidence
lies within 1e-3 of the threshold or whose top-2 probability gap is under 1e-3; those are
excluded and counted.  Confidence values: relative error <= 2e-5 (fp32 streaming sum vs fp64)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import confidence_unmask as oracle_unmask
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

CONF_RTOL = 2e-5


def run_gpu(sd, logits, tokens, masked, tau0, alpha, V=None, eos_id=-1, tau_eos=None, eos_seen=None,
            extra=(0, 0)):
    lg = to_dev(logits)
    tk = torch.from_numpy(tokens.astype(np.int32)).cuda()
    mk = torch.from_numpy(masked.astype(np.uint8)).cuda()
    B, K = tokens.shape
    conf = torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
    es = None if eos_seen is None else torch.from_numpy(eos_seen.astype(np.uint8)).cuda()
    ncom, done = sd.confidence_unmask(lg, tk, mk, tau0, alpha, V=V, confidence=conf, eos_seen=es, eos_id=eos_id,
                                      tau_eos=tau_eos, r_extra_masked=extra[0], r_extra_total=extra[1])
    torch.cuda.synchronize()
    return {"tokens": tk.cpu().numpy(), "masked": mk.cpu().numpy(), "confidence": conf.cpu().numpy(),
            "n_committed": ncom.cpu().numpy(), "block_done": done.cpu().numpy(),
            "eos_seen": None if es is None else es.cpu().numpy()}


def compare(got, logits, tokens, masked, tau0, alpha, V=None, eos_id=-1, tau_eos=None, eos_seen=None,
            extra=(0, 0)):
    """Element-by-element comparison with the oracle.

    Returns (n_gap, n_band, skipped, want):
      n_gap   masked positions whose top-2 probability gap is < 1e-3.  The rule allows excluding them;
              because both sides take the argmax on the exact logits with the same lowest-id tie-break
              they are compared anyway and must match;
      n_band  masked positions with |c - tau| < 1e-3: excluded from the commit-set comparison;
      skipped sequences whose commit set cannot be compared at all (an in-band position decides whether
              the fallback fires, or the fallback's two best confidences agree to 1e-6 relative)."""
    # both sides see the fp32-rounded parameters
    t0, al = float(np.float32(tau0)), float(np.float32(alpha))
    te = None if tau_eos is None else float(np.float32(tau_eos))
    want = oracle_unmask(wl.to_f64(logits), tokens, masked, t0, al, eos_id=eos_id, tau_eos=te,
                         extra_masked=extra[0], extra_total=extra[1], eos_seen=eos_seen, V=V)
    B, K = tokens.shape
    was = masked != 0
    np.testing.assert_allclose(got["confidence"][was], want["confidence"][was], rtol=CONF_RTOL, atol=0)
    assert (got["confidence"][~was] == -7.0).all()          # untouched where not masked
    n_gap = int((want["gap"][was] < 1e-3).sum())
    band = was & (np.abs(np.nan_to_num(want["confidence"]) - np.nan_to_num(want["tau"])[:, None]) < 1e-3)
    n_band = int(band.sum())
    skipped = 0
    for b in range(B):
        if not was[b].any():
            assert got["n_committed"][b] == 0 and got["block_done"][b] == 1
            continue
        c = want["confidence"][b]
        if want["fallback"][b]:
            top = np.sort(c[was[b]])[::-1]
            if band[b].any() or (top.size > 1 and (top[0] - top[1]) <= 1e-6 * top[0]):
                skipped += 1
                continue
        firm = was[b] & ~band[b] & (np.nan_to_num(c) >= want["tau"][b])
        if band[b].any() and not firm.any():
            skipped += 1                                     # an in-band position decides the fallback
            continue
        keep = ~band[b]
        assert (got["masked"][b][keep] == want["masked"][b][keep]).all(), b
        assert (got["tokens"][b][keep] == want["tokens"][b][keep]).all(), b
        if not band[b].any():
            assert got["n_committed"][b] == want["n_committed"][b]
            assert got["block_done"][b] == want["block_done"][b]
            if eos_seen is not None:
                assert got["eos_seen"][b] == want["eos_seen"][b]
    # every committed id is the oracle's argmax, in-band or not
    newly = was & (got["masked"] == 0)
    assert (got["tokens"][newly] == want["xhat"][newly]).all()
    # properties that hold regardless of exclusions
    assert ((got["masked"] != 0) <= was).all()
    assert (got["tokens"][~newly] == tokens[~newly]).all()
    assert (got["block_done"] == (got["masked"].sum(axis=1) == 0)).all()
    assert (got["n_committed"] == was.sum(axis=1) - (got["masked"] != 0).sum(axis=1)).all()
    return n_gap, n_band, skipped, want


@pytest.mark.parametrize("name", ["cfg1", "small_bf16"])
def test_unmask_small_configs(gpu_lib, name):
    w = wl.WORKLOADS[name]
    u = wl.make_unmask_inputs(w, seed=0)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    n_gap, n_band, skip, want = compare(got, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    print(f"{name}: gap<1e-3={n_gap} in-band={n_band} skipped_seqs={skip} committed={int(want['n_committed'].sum())}")
    assert skip == 0


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("V,ld", [(1, 8), (7, 8), (8, 8), (9, 16), (2049, 2056), (5000, 5000), (33000, 33008)])
def test_unmask_ragged_vocab_and_stride(gpu_lib, dtype, V, ld):
    B, K = 3, 8
    lg = wl.make_logits(dtype, B, K, V, 3.0, V > 100, seed=V, ld=ld)
    # poison the padding: it must never be read as a logit
    if dtype == "bf16":
        lg[:, :, V:] = wl.f32_to_bf16_bits(np.full((1,), 1000.0, dtype=np.float32))[0]
    else:
        lg[:, :, V:] = 1000.0
    g = np.random.default_rng(V)
    masked = (g.uniform(size=(B, K)) < 0.7).astype(np.uint8)
    masked[2] = 0
    tokens = g.integers(0, V, size=(B, K)).astype(np.int32)
    tokens[masked != 0] = wl.MASK_TOKEN
    got = run_gpu(gpu_lib, lg, tokens, masked, 0.6, 0.3, V=V)
    compare(got, lg, tokens, masked, 0.6, 0.3, V=V)


def test_unmask_threshold_zero_and_above_one(gpu_lib):
    w = wl.WORKLOADS["small_bf16"]
    u = wl.make_unmask_inputs(w, seed=2)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], 0.0, 0.3)
    assert (got["masked"] == 0).all() and (got["block_done"] == 1).all()
    assert (got["n_committed"] == u["masked"].sum(axis=1)).all()
    compare(got, u["logits"], u["tokens"], u["masked"], 0.0, 0.3)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], 1.5, 0.0)
    assert (got["n_committed"] == 1).all()
    compare(got, u["logits"], u["tokens"], u["masked"], 1.5, 0.0)


def test_unmask_ties_take_lowest_id_and_position(gpu_lib):
    V, B, K = 4099, 2, 4
    lg = np.zeros((B, K, 4104), dtype=np.float32)
    lg[0, 0, [4098, 17, 2000]] = 9.0          # three equal maxima -> id 17
    lg[0, 1, [3000, 4098]] = 9.0              # two equal maxima in different splits / lanes -> 3000
    lg[0, 2, 5] = 20.0
    lg[0, 3, 6] = 20.0                        # same confidence as position 2
    lg[1] = lg[0]
    bits = wl.f32_to_bf16_bits(lg)
    tokens = np.full((B, K), wl.MASK_TOKEN, dtype=np.int32)
    masked = np.ones((B, K), dtype=np.uint8)
    masked[1, 2] = 0
    tokens[1, 2] = 11
    got = run_gpu(gpu_lib, bits, tokens, masked, 2.0, 0.0, V=V)     # fallback only
    assert got["tokens"][0].tolist() == [wl.MASK_TOKEN, wl.MASK_TOKEN, 5, wl.MASK_TOKEN]   # lowest position of the tie
    assert got["tokens"][1].tolist() == [wl.MASK_TOKEN, wl.MASK_TOKEN, 11, 6]
    got = run_gpu(gpu_lib, bits, tokens, masked, 0.0, 0.0, V=V)     # commit all: check the ids
    assert got["tokens"][0].tolist() == [17, 3000, 5, 6]


def test_unmask_eos_flag(gpu_lib):
    V, B, K = 3000, 3, 4
    lg = np.full((B, K, V), -10.0, dtype=np.float32)
    lg[0, 0, 7] = 12.0; lg[0, 1, 1] = 12.0; lg[0, 2, 2] = 12.0; lg[0, 3, 3] = 12.0      # commits eos (7)
    lg[1, :, 5] = 12.0                                                                  # commits non-eos
    lg[2, 0, 7] = -9.9                                                                  # eos through fallback, low c
    tokens = np.full((B, K), wl.MASK_TOKEN, dtype=np.int32)
    masked = np.ones((B, K), dtype=np.uint8)
    es = np.array([0, 0, 0], dtype=np.uint8)
    got = run_gpu(gpu_lib, lg, tokens, masked, 0.9, 0.0, eos_id=7, eos_seen=es)
    assert got["eos_seen"].tolist() == [1, 0, 0]
    compare(got, lg, tokens, masked, 0.9, 0.0, eos_id=7, eos_seen=es)
    es2 = np.array([0, 1, 0], dtype=np.uint8)        # sticky
    got = run_gpu(gpu_lib, lg, tokens, masked, 0.9, 0.0, eos_id=7, eos_seen=es2)
    assert got["eos_seen"].tolist() == [1, 1, 0]


def test_unmask_query_wide_ratio(gpu_lib):
    w = wl.WORKLOADS["small_bf16"]
    u = wl.make_unmask_inputs(w, seed=5)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], 0.9, 0.6, extra=(33, 33))
    compare(got, u["logits"], u["tokens"], u["masked"], 0.9, 0.6, extra=(33, 33))


def test_unmask_multi_step_to_block_done(gpu_lib):
    """Loop fresh-seeded steps until the block is finished; every step must agree with the oracle
    and the mask count must never grow (committed tokens never re-mask)."""
    w = wl.WORKLOADS["small_bf16"]
    tokens = np.full((w.B, w.K), wl.MASK_TOKEN, dtype=np.int32)
    masked = np.ones((w.B, w.K), dtype=np.uint8)
    for step in range(64):
        lg = wl.make_logits("bf16", w.B, w.K, w.V, w.logit_std, True, seed=11, step=step)
        got = run_gpu(gpu_lib, lg, tokens, masked, 0.9, 0.3)
        compare(got, lg, tokens, masked, 0.9, 0.3)
        assert got["masked"].sum() < masked.sum()
        tokens, masked = got["tokens"], got["masked"]
        if got["block_done"].all():
            break
    assert got["block_done"].all() and step < 40


def test_unmask_cfg2_full_size(gpu_lib):
    w = wl.WORKLOADS["cfg2"]
    u = wl.make_unmask_inputs(w, seed=0)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    n_gap, n_band, skip, want = compare(got, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    print(f"cfg2: gap<1e-3={n_gap} in-band={n_band} skipped_seqs={skip} committed={int(want['n_committed'].sum())} "
          f"conf range {np.nanmin(want['confidence']):.3f}..{np.nanmax(want['confidence']):.3f}")
    assert skip == 0


@pytest.mark.parametrize("name", ["cfg3A", "cfg4", "cfg4boost", "cfg5", "cfgBC"])
def test_unmask_full_size_configs(gpu_lib, name):
    w = wl.WORKLOADS[name]
    u = wl.make_unmask_inputs(w, seed=0)
    got = run_gpu(gpu_lib, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    n_gap, n_band, skip, want = compare(got, u["logits"], u["tokens"], u["masked"], w.tau0, w.alpha)
    print(f"{name}: gap<1e-3={n_gap} in-band={n_band} skipped_seqs={skip} committed={int(want['n_committed'].sum())} "
          f"done={int(want['block_done'].sum())}/{w.B}")
    assert skip <= w.B // 8


@pytest.mark.parametrize("frac", [0.5, 1.0])
def test_unmask_longest_block(gpu_lib, frac):
    # K = 4096, the longest block the entry point takes (four passes of the commit kernel over the positions,
    # 32 KB of its LDS), ragged vocabulary, padded rows; two sequences with different masked counts
    B, K, V, ld = 2, 4096, 523, 528
    logits = wl.make_logits("bf16", B, K, V, 3.0, True, seed=11, ld=ld)
    g = np.random.Generator(np.random.Philox(key=4096))
    masked = (g.uniform(size=(B, K)) < np.array([[frac], [frac / 2]])).astype(np.uint8)
    tokens = g.integers(0, V, size=(B, K)).astype(np.int32)
    tokens[masked != 0] = wl.MASK_TOKEN
    got = run_gpu(gpu_lib, logits, tokens, masked, 0.9, 0.3, V=V)
    n_gap, n_band, skip, want = compare(got, logits, tokens, masked, 0.9, 0.3, V=V)
    assert skip == 0 and want["n_committed"].min() >= 1


def test_unmask_non_finite_logits_stay_in_bounds(gpu_lib):
    """NaN / inf logits are outside the method's domain (the oracle defines nothing for them); the
    kernel must still stay in bounds and keep its invariants: exactly the fallback's single commit per
    sequence when nothing finite passes the threshold, a valid position, counters consistent."""
    B, K, V = 3, 8, 777 + 7
    g = np.random.Generator(np.random.Philox(key=77))
    logits = g.standard_normal((B, K, V), dtype=np.float32) * 3
    masked = np.ones((B, K), dtype=np.uint8)
    masked[1, :3] = 0
    logits[0] = np.nan                          # every row of sequence 0
    logits[1, 4, 10] = np.inf                   # one +inf in one row of sequence 1
    logits[2, :, ::2] = -np.inf                 # -inf is a legitimate "impossible token": finite results
    tokens = np.full((B, K), wl.MASK_TOKEN, dtype=np.int32)
    got = run_gpu(gpu_lib, logits, tokens, masked, 2.0, 0.0)      # tau0 > 1: only the fallback can commit
    assert (got["n_committed"] == 1).all()
    for b in range(B):
        newly = (masked[b] != 0) & (got["masked"][b] == 0)
        assert newly.sum() == 1
        assert (got["masked"][b][masked[b] == 0] == 0).all()
    assert got["masked"][0, 0] == 0             # all-NaN sequence: the lowest masked position is taken
    assert got["tokens"][0, 0] == 0             # a row without any finite logit commits id 0 (a valid id)
    newly_all = (masked != 0) & (got["masked"] == 0)
    assert ((got["tokens"][newly_all] >= 0) & (got["tokens"][newly_all] < V)).all()
    assert (got["block_done"] == 0).all()
    # the sequence with -inf entries is inside the domain: compare it with the oracle
    want = oracle_unmask(wl.to_f64(logits[2:3]), tokens[2:3], masked[2:3], 2.0, 0.0)
    assert (got["tokens"][2] == want["tokens"][0]).all() and (got["masked"][2] == want["masked"][0]).all()


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_unmask_fallback_tie_takes_lowest_position(gpu_lib, dtype):
    """Identical logit rows give bit-identical confidences on the GPU as well (same reduction order for
    equal data), so the fallback tie is exact and must go to the lower position."""
    B, K, V = 2, 40, 3001
    lg = wl.make_logits(dtype, B, K, V, 3.0, False, seed=5, ld=3008)
    masked = np.zeros((B, K), dtype=np.uint8)
    masked[0, [3, 17, 30]] = 1
    masked[1, [0, 39]] = 1
    lg[0, 30] = lg[0, 17]
    lg[0, 3] = lg[0, 17]                       # three-way tie: position 3 wins
    lg[1, 39] = lg[1, 0]
    tokens = np.full((B, K), 5, dtype=np.int32)
    tokens[masked != 0] = wl.MASK_TOKEN
    got = run_gpu(gpu_lib, lg, tokens, masked, 1.5, 0.0, V=V)
    want = oracle_unmask(wl.to_f64(lg), tokens, masked, 1.5, 0.0, V=V)
    assert (got["masked"] == want["masked"]).all() and (got["tokens"] == want["tokens"]).all()
    assert got["masked"][0, 3] == 0 and got["masked"][0, 17] == 1 and got["masked"][1, 0] == 0
    assert (got["n_committed"] == 1).all()
