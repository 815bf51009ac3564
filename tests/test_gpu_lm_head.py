"""GPU parity: sdllm_lm_head_unmask (vocabulary projection fused into the unmask; paper Eq. 3 -> Eq. 4, then
Eq. 10, 9, 5 and the exit flags) against the fp64 oracle.

Bar: committed token ids and the unmask set bit-exact, except positions whose oracle confidence lies
within 1e-3 of the threshold or whose top-2 probability gap is under 1e-3 (fp32 accumulation of a logit
over Hd terms can reorder two near-equal logits); those are excluded and counted.  Confidence values:
relative error <= 2e-4 -- a logit is a sum of Hd exact bf16 x bf16 products accumulated in fp32, absolute
error ~ sqrt(Hd) * 2^-24 * |z| ~ 1e-5 at Hd = 4096, and d(ln c) is a probability-weighted mean of those."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import lm_head_unmask as oracle_lm_head_unmask
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

CONF_RTOL = 2e-4


def run_gpu(sd, hidden, weight, tokens, masked, tau0, alpha, eos_id=-1, tau_eos=None, eos_seen=None, extra=(0, 0),
            packed=False):
    """hidden / weight: device bf16 tensors (possibly strided views); packed: the projection goes through
    sdllm_lm_head_pack_weight first and the call reads the packed image."""
    if packed:
        weight = sd.lm_head_pack_weight(weight)
    tk = torch.from_numpy(tokens.astype(np.int32)).cuda()
    mk = torch.from_numpy(masked.astype(np.uint8)).cuda()
    B, K = tokens.shape
    conf = torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
    es = None if eos_seen is None else torch.from_numpy(eos_seen.astype(np.uint8)).cuda()
    ncom, done = sd.lm_head_unmask(hidden, weight, tk, mk, tau0, alpha, confidence=conf, eos_seen=es, eos_id=eos_id,
                                   tau_eos=tau_eos, r_extra_masked=extra[0], r_extra_total=extra[1])
    torch.cuda.synchronize()
    return {"tokens": tk.cpu().numpy(), "masked": mk.cpu().numpy(), "confidence": conf.cpu().numpy(),
            "n_committed": ncom.cpu().numpy(), "block_done": done.cpu().numpy(),
            "eos_seen": None if es is None else es.cpu().numpy()}


def compare(got, want, tokens, masked, seqs=None, eos=False):
    """Element by element against the oracle's result dict `want` (sequences `seqs` only, default all).
    Returns (n_gap, n_band, skipped sequences)."""
    B, K = tokens.shape
    seqs = range(B) if seqs is None else seqs
    was = masked != 0
    n_gap = n_band = skipped = 0
    for b in seqs:
        wb = was[b]
        assert (got["confidence"][b][~wb] == -7.0).all()            # untouched where not masked
        if not wb.any():
            assert got["n_committed"][b] == 0 and got["block_done"][b] == 1
            assert (got["tokens"][b] == tokens[b]).all() and (got["masked"][b] == 0).all()
            continue
        c, tau = want["confidence"][b], want["tau"][b]
        np.testing.assert_allclose(got["confidence"][b][wb], c[wb], rtol=CONF_RTOL, atol=0)
        gap = wb & (np.nan_to_num(want["gap"][b], nan=1.0) < 1e-3)
        band = wb & (np.abs(np.nan_to_num(c) - tau) < 1e-3)
        n_gap += int(gap.sum()); n_band += int(band.sum())
        newly = wb & (got["masked"][b] == 0)
        sure = newly & ~gap
        assert (got["tokens"][b][sure] == want["xhat"][b][sure]).all(), b   # every committed id is the arg-max
        assert (got["tokens"][b][~newly] == tokens[b][~newly]).all(), b
        assert got["n_committed"][b] == newly.sum()
        assert got["block_done"][b] == (0 if (got["masked"][b] != 0).any() else 1)
        if want["fallback"][b]:
            top = np.sort(c[wb])[::-1]
            if band.any() or (top.size > 1 and (top[0] - top[1]) <= 1e-4 * top[0]):
                skipped += 1
                continue
        firm = wb & ~band & (np.nan_to_num(c) >= tau)
        if band.any() and not firm.any():
            skipped += 1                                                  # an in-band position decides the fallback
            continue
        keep = ~band
        assert (got["masked"][b][keep] == want["masked"][b][keep]).all(), b
        if not band.any():
            assert got["n_committed"][b] == want["n_committed"][b]
            assert got["block_done"][b] == want["block_done"][b]
            if eos and not gap.any():
                assert got["eos_seen"][b] == want["eos_seen"][b]
    return n_gap, n_band, skipped


def _host_case(B, K, Hd, V, seed, std=4.0, boost=True, frac=0.6, ld_h=None, ld_w=None):
    """Small host-drawn case; returns host bits and device tensors (strided when ld_* is given)."""
    g = np.random.Generator(np.random.Philox(key=seed))
    h = wl.f32_to_bf16_bits(g.standard_normal((B, K, Hd), dtype=np.float32))
    W = g.standard_normal((V, Hd), dtype=np.float32) * np.float32(std / np.sqrt(Hd))
    if boost:
        hf = wl.bf16_bits_to_f32(h)
        for b in range(B):
            for k in range(K):
                W[g.integers(0, V)] = np.float32(g.uniform(6.0, 14.0)) * hf[b, k] / np.float32(np.dot(hf[b, k], hf[b, k]))
    W = wl.f32_to_bf16_bits(W)
    masked = (g.uniform(size=(B, K)) < frac).astype(np.uint8)
    tokens = g.integers(0, V, size=(B, K)).astype(np.int32)
    tokens[masked != 0] = wl.MASK_TOKEN
    poison = wl.f32_to_bf16_bits(np.full((1,), np.nan, dtype=np.float32))[0]
    ld_h = Hd if ld_h is None else ld_h
    ld_w = Hd if ld_w is None else ld_w
    hp = np.full((B, K, ld_h), poison, dtype=np.uint16); hp[..., :Hd] = h      # the padding must never be read
    Wp = np.full((V, ld_w), poison, dtype=np.uint16); Wp[:, :Hd] = W
    hd, Wd = to_dev(hp)[..., :Hd], to_dev(Wp)[:, :Hd]
    return h, W, tokens, masked, hd, Wd


def _oracle(h, W, tokens, masked, tau0, alpha, **kw):
    t0, al = float(np.float32(tau0)), float(np.float32(alpha))
    if kw.get("tau_eos") is not None:
        kw["tau_eos"] = float(np.float32(kw["tau_eos"]))
    return oracle_lm_head_unmask(wl.bf16_bits_to_f32(h), wl.bf16_bits_to_f32(W), tokens, masked, t0, al, **kw)


# rows <= 32 / <= 64 / > 64 select the three kernel shapes; V and Hd chosen to leave ragged vocabulary tiles,
# a hidden width below one LDS chunk, and widths that end inside a chunk
@pytest.mark.parametrize("B,K,Hd,V", [
    (1, 8, 32, 1), (1, 32, 64, 100), (2, 16, 96, 129), (1, 32, 1056, 1000), (1, 32, 512, 4099),
    (2, 32, 288, 300), (3, 20, 544, 777), (1, 64, 1024, 2048), (2, 24, 1568, 1100),
    (3, 32, 288, 300), (4, 25, 544, 777), (1, 128, 1024, 2048), (4, 32, 1568, 1100), (2, 60, 32, 40000),
    (5, 32, 160, 513), (3, 64, 416, 1500), (9, 32, 1024, 700), (2, 160, 256, 2000),
    (4, 600, 64, 300),        # 2400 positions: ten passes of the mask scan, ten row chunks, two triples per position
    (2, 600, 64, 20000),      # 79 triples per position and more positions than the commit kernel has lanes to spare
])
@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_shapes(gpu_lib, B, K, Hd, V, packed):
    h, W, tokens, masked, hd, Wd = _host_case(B, K, Hd, V, seed=B * 1000 + K + Hd + V)
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.7, 0.3, packed=packed)
    want = _oracle(h, W, tokens, masked, 0.7, 0.3)
    n_gap, n_band, skipped = compare(got, want, tokens, masked)
    print(f"B{B} K{K} Hd{Hd} V{V}: gap<1e-3={n_gap} in-band={n_band} skipped_seqs={skipped} "
          f"committed={int(want['n_committed'].sum())}")
    assert skipped <= 1


_TILE_CASES = [3000, 12000, 20000, 30000, 45000, 50000, 60000, 80000, 90000, 100000, 126464, 152064]


def test_tile_cases_cover_every_compiled_stream_kernel(gpu_lib):
    seen32 = {gpu_lib.plan_lm_head(gpu_lib.lm_head_params(1, 32, V, 64, 64, 64, 0.9, 0.3)).vocab_rows_per_tile // 32
              for V in _TILE_CASES}
    seen64 = {gpu_lib.plan_lm_head(gpu_lib.lm_head_params(2, 32, V, 64, 64, 64, 0.9, 0.3)).vocab_rows_per_tile // 32
              for V in _TILE_CASES}
    seen128 = {gpu_lib.plan_lm_head(gpu_lib.lm_head_params(4, 32, V, 64, 64, 64, 0.9, 0.3)).vocab_rows_per_tile // 32
               for V in _TILE_CASES}
    assert seen32 == {2, 4, 8, 12, 16, 20} and seen64 == {2, 4, 8, 10, 12, 16} and seen128 == {1, 2, 3, 4, 6, 8, 10, 16}
    packed = lambda B, V: gpu_lib.plan_lm_head(gpu_lib.lm_head_params(B, 32, V, 64, 64, 0, 0.9, 0.3, weight_packed=1))
    assert {packed(1, V).vocab_rows_per_tile // 64 for V in _TILE_CASES} == {1, 2, 4, 6, 8, 10}
    assert {packed(2, V).vocab_rows_per_tile // 32 for V in _TILE_CASES} == {1, 2, 3, 4, 6, 8, 10, 16}


@pytest.mark.parametrize("V", _TILE_CASES)
@pytest.mark.parametrize("B", [1, 2, 4])
@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_every_vocabulary_tile_size(gpu_lib, B, V, packed):
    # the stream kernels are compiled for a list of tile sizes and the vocabulary size picks one: every one of
    # them runs here (narrow hidden width, so that the oracle stays cheap), about 24, 48 and 96 masked positions
    K, Hd = 32, 64
    h, W, tokens, masked, hd, Wd = _host_case(B, K, Hd, V, seed=V + B, frac=0.75, std=1.0)
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.3, 0.3, packed=packed)
    want = _oracle(h, W, tokens, masked, 0.3, 0.3)
    n_gap, n_band, skipped = compare(got, want, tokens, masked)
    assert skipped <= 1 and n_gap <= masked.sum() // 2      # most positions have a clear arg-max to compare


@pytest.mark.parametrize("B,K", [(2, 32), (4, 32), (5, 32), (9, 64)])
@pytest.mark.parametrize("n_masked", [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 160])
@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_shape_follows_the_masked_count(gpu_lib, B, K, n_masked, packed):
    # the masked count is device data: every shape that B x K admits is launched and the one whose range holds
    # the count does the work; counts on both sides of each boundary, spread over the sequences, with V chosen so
    # that the narrower tiles of the wide shape leave an odd number of triple slots per position
    if n_masked > B * K:
        pytest.skip("more masked positions than positions")
    Hd, V = 1056, 1100
    h, W, tokens, masked, hd, Wd = _host_case(B, K, Hd, V, seed=77 * B + n_masked, frac=0.0)
    g = np.random.Generator(np.random.Philox(key=n_masked))
    flat = g.permutation(B * K)[:n_masked]
    masked.reshape(-1)[flat] = 1
    tokens.reshape(-1)[flat] = wl.MASK_TOKEN
    assert int(masked.sum()) == n_masked
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.7, 0.3, packed=packed)
    want = _oracle(h, W, tokens, masked, 0.7, 0.3)
    n_gap, n_band, skipped = compare(got, want, tokens, masked)
    assert skipped <= 1


@pytest.mark.parametrize("B,K,Hd,V,ld_h,ld_w", [(2, 16, 64, 200, 72, 80), (2, 32, 320, 1000, 328, 384),
                                                 (4, 32, 320, 1000, 328, 384),
                                                 (3, 32, 320, 1000, 328, 384)])
@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_row_strides_and_poisoned_padding(gpu_lib, B, K, Hd, V, ld_h, ld_w, packed):
    h, W, tokens, masked, hd, Wd = _host_case(B, K, Hd, V, seed=77, ld_h=ld_h, ld_w=ld_w)
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.6, 0.2, packed=packed)
    assert np.isfinite(got["confidence"]).all()
    compare(got, _oracle(h, W, tokens, masked, 0.6, 0.2), tokens, masked)


def test_lm_head_unmasked_rows_are_never_read_and_empty_sequences(gpu_lib):
    B, K, Hd, V = 4, 32, 256, 900
    h, W, tokens, masked, _, Wd = _host_case(B, K, Hd, V, seed=5)
    masked[1] = 0                                       # a finished sequence
    masked[3] = 0; masked[3, 17] = 1                    # a single masked position: it must be committed
    tokens = np.where(masked != 0, wl.MASK_TOKEN, np.abs(tokens) % V).astype(np.int32)
    hp = h.copy()
    hp[masked == 0] = wl.f32_to_bf16_bits(np.full((1,), np.nan, dtype=np.float32))[0]   # poison the unmasked rows
    got = run_gpu(gpu_lib, to_dev(hp), Wd, tokens, masked, 0.7, 0.3)
    assert np.isfinite(got["confidence"][masked != 0]).all()
    want = _oracle(h, W, tokens, masked, 0.7, 0.3)
    compare(got, want, tokens, masked)
    assert got["n_committed"][1] == 0 and got["block_done"][1] == 1
    assert got["n_committed"][3] == 1 and got["block_done"][3] == 1 and got["masked"][3].sum() == 0
    # nothing masked anywhere
    none = np.zeros_like(masked)
    tk = np.abs(tokens) % V
    got = run_gpu(gpu_lib, to_dev(hp), Wd, tk.astype(np.int32), none, 0.7, 0.3)
    assert (got["n_committed"] == 0).all() and (got["block_done"] == 1).all() and (got["tokens"] == tk).all()


def test_lm_head_threshold_extremes_eos_and_query_wide_ratio(gpu_lib):
    B, K, Hd, V = 3, 32, 192, 640
    h, W, tokens, masked, hd, Wd = _host_case(B, K, Hd, V, seed=13)
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.0, 0.3)                 # tau0 = 0 commits every masked position
    assert (got["masked"] == 0).all() and (got["n_committed"] == masked.sum(axis=1)).all()
    compare(got, _oracle(h, W, tokens, masked, 0.0, 0.3), tokens, masked)
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 1.5, 0.0)                 # tau0 > 1: the fallback alone
    assert (got["n_committed"] == (masked.sum(axis=1) > 0)).all()
    compare(got, _oracle(h, W, tokens, masked, 1.5, 0.0), tokens, masked)
    # EOS flag: take the id the oracle commits at some position as eos_id
    base = _oracle(h, W, tokens, masked, 0.5, 0.3)
    committed = (masked != 0) & (base["masked"] == 0)
    b0, i0 = np.argwhere(committed)[0]
    eos_id = int(base["xhat"][b0, i0])
    eos0 = np.zeros(B, dtype=np.uint8); eos0[(b0 + 1) % B] = 1             # sticky
    got = run_gpu(gpu_lib, hd, Wd, tokens, masked, 0.5, 0.3, eos_id=eos_id, tau_eos=0.2, eos_seen=eos0, extra=(7, 9))
    want = _oracle(h, W, tokens, masked, 0.5, 0.3, eos_id=eos_id, tau_eos=0.2, eos_seen=eos0, extra_masked=7, extra_total=9)
    compare(got, want, tokens, masked, eos=True)
    assert got["eos_seen"][b0] == 1 and got["eos_seen"][(b0 + 1) % B] == 1


@pytest.mark.parametrize("n_masked", [40, 100, 65536])
def test_lm_head_most_positions(gpu_lib, n_masked):
    # B x K = 65536, the most positions the entry point takes (256 passes of the mask count and of the row
    # compaction, 256 row chunks in the grid when all are masked), K = 4096 the longest block; a narrow
    # projection keeps the oracle cheap.  40 / 100 masked positions go to two of the stream shapes.
    B, K, Hd, V = 16, 4096, 32, 300
    g = np.random.Generator(np.random.Philox(key=65536 + n_masked))
    h = wl.f32_to_bf16_bits(g.standard_normal((B, K, Hd), dtype=np.float32))
    W = wl.f32_to_bf16_bits(g.standard_normal((V, Hd), dtype=np.float32) * np.float32(2.0 / np.sqrt(Hd)))
    masked = np.zeros((B, K), dtype=np.uint8)
    masked.reshape(-1)[g.permutation(B * K)[:n_masked]] = 1
    tokens = g.integers(0, V, size=(B, K)).astype(np.int32)
    tokens[masked != 0] = wl.MASK_TOKEN
    got = run_gpu(gpu_lib, to_dev(h), to_dev(W), tokens, masked, 0.2, 0.3)
    want = _oracle(h, W, tokens, masked, 0.2, 0.3)
    n_gap, n_band, skipped = compare(got, want, tokens, masked)
    assert skipped <= 2


@pytest.mark.parametrize("V,Hd,ld_w", [(1, 32, 32), (16, 64, 64), (17, 96, 104), (1000, 544, 552), (5003, 4096, 4096)])
def test_pack_weight_is_the_stated_permutation(gpu_lib, V, Hd, ld_w):
    # image[nb][ks][lane][e] = W[min(16 nb + lane % 16, V - 1)][32 ks + 8 (lane / 16) + e], bit for bit
    g = np.random.Generator(np.random.Philox(key=V * 7 + Hd))
    Wp = g.integers(0, 1 << 16, size=(V, ld_w), dtype=np.uint16)
    Wd = to_dev(Wp)[:, :Hd]
    packed = gpu_lib.lm_head_pack_weight(Wd)
    torch.cuda.synchronize()
    got = packed.data.view(torch.int16).cpu().numpy().view(np.uint16)
    NB, NK = (V + 15) // 16, Hd // 32
    assert packed.V == V and packed.Hd == Hd and got.shape == (NB * NK * 512,)
    nb, ks, lane, e = np.meshgrid(np.arange(NB), np.arange(NK), np.arange(64), np.arange(8), indexing="ij")
    want = Wp[np.minimum(16 * nb + lane % 16, V - 1), 32 * ks + 8 * (lane // 16) + e]
    assert (got.reshape(NB, NK, 64, 8) == want).all()


def _full_size(gpu_lib, name, seqs=None, B=None, packed=False):
    w = wl.WORKLOADS[name]
    if B is not None:
        w = dataclasses.replace(w, B=B)
    t = wl.make_lm_head_inputs_device(w, seed=0)
    got = run_gpu(gpu_lib, t["hidden"], t["lm_weight"], t["tokens"], t["masked"], w.tau0, w.alpha, packed=packed)
    # the oracle sees the same bits: copy the operands back (bf16 -> fp32 is exact)
    h = t["hidden"].float().cpu().numpy()
    W = t["lm_weight"].float().cpu().numpy()
    seqs = list(range(w.B)) if seqs is None else seqs
    sub = np.array(seqs)
    want = oracle_lm_head_unmask(h[sub], W, t["tokens"][sub], t["masked"][sub], float(np.float32(w.tau0)),
                                 float(np.float32(w.alpha)))
    got_sub = {k: (v[sub] if v is not None else None) for k, v in got.items()}
    n_gap, n_band, skipped = compare(got_sub, want, t["tokens"][sub], t["masked"][sub])
    print(f"{name}: sequences {seqs} gap<1e-3={n_gap} in-band={n_band} skipped_seqs={skipped} "
          f"committed={int(want['n_committed'].sum())} fallback={int(want['fallback'].sum())}")
    return skipped, want


@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_cfg2_full_size(gpu_lib, packed):
    skipped, want = _full_size(gpu_lib, "cfg2", packed=packed)
    assert skipped == 0 and want["n_committed"][0] >= 1


@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_cfg2_two_sequences_full_size(gpu_lib, packed):
    # 64 positions: the stream shape that keeps the hidden chunk in LDS, at the full vocabulary and width
    skipped, _ = _full_size(gpu_lib, "cfg2", B=2, packed=packed)
    assert skipped == 0


@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_cfg2_four_sequences_full_size(gpu_lib, packed):
    # 128 positions: the stream shape fed by global -> LDS transfers, at the full vocabulary and width
    skipped, _ = _full_size(gpu_lib, "cfg2", B=4, packed=packed)
    assert skipped <= 1


@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_cfg3A_full_size(gpu_lib, packed):
    # 256 masked rows = two row chunks per vocabulary tile; the oracle projects every row (a few tens of seconds)
    skipped, _ = _full_size(gpu_lib, "cfg3A", packed=packed)
    assert skipped <= 1


@pytest.mark.parametrize("packed", [False, True])
def test_lm_head_cfg4boost_sampled_sequences(gpu_lib, packed):
    # 16 x 32 positions, a different masked count per sequence (rows compacted across sequences), V = 152064,
    # Hd = 3584 (seven LDS chunks); the oracle runs on four of the sixteen sequences
    skipped, _ = _full_size(gpu_lib, "cfg4boost", seqs=[0, 5, 10, 15], packed=packed)
    assert skipped <= 1
