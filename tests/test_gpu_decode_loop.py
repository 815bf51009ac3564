"""GPU integration: the three calls in the paper's decode loop (section 3.1 / 3.3) over several blocks --
suffix rule -> attention per layer -> unmask steps until the block is done -> KV append -> next block,
with the EOS early exit -- checked against the oracle at every step.  The model forward is out of scope,
so Q/K/V and logits are seeded tensors of the right shapes."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
import oracle
from gpu_util import to_dev, to_f64_host

pytestmark = pytest.mark.gpu


def test_block_loop_with_append_and_early_exit(gpu_lib):
    sd = gpu_lib
    B, Hq, Hkv, D, prompt, gen, K, V, L = 2, 4, 2, 128, 70, 96, 32, 3000, 2
    cap = prompt + gen
    tau0, alpha, eos_id = 0.9, 0.3, 5
    N = gen // K
    base = wl.make_append_inputs("bf16", L, B, Hkv, D, K, cap, seed=21)
    k_host, v_host = base["k_caches"].copy(), base["v_caches"].copy()        # oracle's caches (bit patterns)
    k_dev, v_dev = to_dev(k_host), to_dev(v_host)
    eos_dev = torch.zeros(B, dtype=torch.uint8, device="cuda")
    eos_host = np.zeros(B, dtype=np.uint8)
    blocks_decoded = 0
    for c in range(N):
        P, S = prompt + c * K, gen - (c + 1) * K
        keep = sd.suffix_keep_indices(S, K, 1, True)
        assert keep == oracle.suffix_keep_indices(prompt, gen, K, c, 1, True)
        keep_np = np.asarray(keep, dtype=np.int32)
        # attention of every layer over [cache[0:P] | block | kept suffix]
        blk = []
        for layer in range(L):
            t = wl.make_custom_attention_inputs("bf16", B, Hq, Hkv, D, P, cap, K, max(S, 1), keep_np, seed=100 * c + layer)
            t["k_cache"], t["v_cache"] = k_host[layer], v_host[layer]
            d = {k: to_dev(v) for k, v in t.items() if k not in ("k_cache", "v_cache")}
            nk = len(keep)
            out = sd.block_attention(d["q_block"], d["q_suffix"] if nk else None, k_dev[layer], v_dev[layer],
                                     d["k_block"], d["v_block"], d["k_suffix"] if nk else None,
                                     d["v_suffix"] if nk else None, d["keep_idx"] if nk else None, P)
            f = {k: (wl.to_f64(v) if k != "keep_idx" else v) for k, v in t.items()}
            want = oracle.block_attention(f["q_block"], f["q_suffix"], f["k_cache"], f["v_cache"], f["k_block"],
                                          f["v_block"], f["k_suffix"], f["v_suffix"], keep_np, P)
            torch.cuda.synchronize()
            assert np.abs(to_f64_host(out) - want).max() <= 2e-2, (c, layer)
            blk.append((t["k_block"], t["v_block"]))
        # diffusion steps of the block
        tokens = np.full((B, K), wl.MASK_TOKEN, dtype=np.int32)
        masked = np.ones((B, K), dtype=np.uint8)
        tk, mk = torch.from_numpy(tokens).cuda(), torch.from_numpy(masked).cuda()
        for step in range(64):
            lg = wl.make_logits("bf16", B, K, V, 4.0, True, seed=7 + c, step=step)
            if c == 1 and step == 0:
                lg[0, 3, :] = wl.f32_to_bf16_bits(np.full(V, -20.0, dtype=np.float32))
                lg[0, 3, eos_id] = wl.f32_to_bf16_bits(np.array([20.0], dtype=np.float32))[0]   # sequence 0 emits EOS in block 1
            ncom, done = sd.confidence_unmask(to_dev(lg), tk, mk, tau0, alpha, eos_id=eos_id, eos_seen=eos_dev)
            ref = oracle.confidence_unmask(wl.to_f64(lg), tokens, masked, float(np.float32(tau0)), float(np.float32(alpha)),
                                           eos_id=eos_id, eos_seen=eos_host)
            torch.cuda.synchronize()
            band = (masked != 0) & (np.abs(np.nan_to_num(ref["confidence"]) - np.nan_to_num(ref["tau"])[:, None]) < 1e-3)
            assert not band.any(), "seeded logits must not sit on the threshold"
            assert (tk.cpu().numpy() == ref["tokens"]).all() and (mk.cpu().numpy() == ref["masked"]).all()
            assert (ncom.cpu().numpy() == ref["n_committed"]).all() and (done.cpu().numpy() == ref["block_done"]).all()
            assert (eos_dev.cpu().numpy() == ref["eos_seen"]).all()
            assert ref["masked"].sum() < masked.sum()                       # the block terminates
            tokens, masked, eos_host = ref["tokens"].astype(np.int32), ref["masked"], ref["eos_seen"]
            if ref["block_done"].all():
                break
        assert ref["block_done"].all()
        # the finished block joins the prefix of every layer (only sequences that are still decoding)
        kb = np.stack([b_[0] for b_ in blk]); vb = np.stack([b_[1] for b_ in blk])
        still = (1 - eos_host).astype(np.uint8) if c > 0 else np.ones(B, dtype=np.uint8)
        sd.kv_append(k_dev, v_dev, to_dev(kb), to_dev(vb), P, do_append=torch.from_numpy(still).cuda())
        k_host, v_host = oracle.kv_append(k_host, v_host, kb, vb, P, do_append=still)
        torch.cuda.synchronize()
        assert (k_dev.view(torch.int16).cpu().numpy().view(np.uint16) == k_host).all()
        assert (v_dev.view(torch.int16).cpu().numpy().view(np.uint16) == v_host).all()
        blocks_decoded += 1
        if eos_host.all():                                                  # early exit: later blocks are skipped
            break
    assert eos_host[0] == 1 and blocks_decoded >= 2


@pytest.mark.parametrize("B,K,boost_at", [(None, None, 6), (8, 32, 30)])
def test_block_steps_fed_by_the_vocabulary_projection(gpu_lib, B, K, boost_at):
    """The diffusion steps of one block with the logits coming from the projection of seeded hidden states
    (never stored): every step is checked against the oracle from the same state, up to block termination.
    An unboosted projection keeps the confidences low, so most steps go through the fallback of Eq. 9 and
    commit one position per sequence; a boosted projection at step boost_at commits what is left at once.
    With 8 x 32 positions the masked count goes 256, 248, ... down through every range that picks another
    kernel shape of the projection (above 128, 65-128, 33-64, at most 32)."""
    sd = gpu_lib
    w = wl.WORKLOADS["small_bf16"]
    if B is not None:
        w = dataclasses.replace(w, B=B, K=K)
    B, K, Hd, V = w.B, w.K, 256, 1500
    counts = []
    tau0, alpha = 0.9, 0.3
    w_plain = dataclasses.replace(w, boost=False)
    plain = wl.make_lm_head_inputs(w_plain, seed=3, V=V, Hd=Hd)        # a projection without any boosted row
    tokens = np.full((B, K), wl.MASK_TOKEN, dtype=np.int32)
    masked = np.ones((B, K), dtype=np.uint8)
    tk, mk = torch.from_numpy(tokens).cuda(), torch.from_numpy(masked).cuda()
    conf = torch.zeros((B, K), dtype=torch.float32, device="cuda")
    steps = checked = 0
    while masked.any():
        assert steps <= B * K, "the block must terminate"
        boosted = steps == boost_at                                      # fallback steps, then a confident one
        counts.append(int(masked.sum()))
        t = wl.make_lm_head_inputs(w if boosted else w_plain, seed=3, step=steps, V=V, Hd=Hd)
        h, W = t["hidden"], (t["lm_weight"] if boosted else plain["lm_weight"])
        ncom, done = sd.lm_head_unmask(to_dev(h), to_dev(W), tk, mk, tau0, alpha, confidence=conf)
        ref = oracle.lm_head_unmask(wl.bf16_bits_to_f32(h), wl.bf16_bits_to_f32(W), tokens, masked,
                                    float(np.float32(tau0)), float(np.float32(alpha)))
        torch.cuda.synchronize()
        g_tok, g_msk = tk.cpu().numpy(), mk.cpu().numpy()
        was = masked != 0
        np.testing.assert_allclose(conf.cpu().numpy()[was], ref["confidence"][was], rtol=2e-4, atol=0)
        for b in range(B):
            if not was[b].any():
                assert ncom[b].item() == 0 and done[b].item() == 1
                continue
            c = ref["confidence"][b]
            band = was[b] & (np.abs(np.nan_to_num(c) - ref["tau"][b]) < 1e-3)
            top = np.sort(c[was[b]])[::-1]
            ambiguous = band.any() or (ref["fallback"][b] and top.size > 1 and (top[0] - top[1]) <= 1e-4 * top[0])
            newly = was[b] & (g_msk[b] == 0)
            assert newly.any() and ncom[b].item() == newly.sum()           # progress in every step (Eq. 9's fallback)
            assert done[b].item() == (0 if g_msk[b].any() else 1)
            if not ambiguous:
                assert (g_msk[b] == ref["masked"][b]).all(), (steps, b)
                sure = newly & (np.nan_to_num(ref["gap"][b], nan=1.0) >= 1e-3)
                assert (g_tok[b][sure] == ref["xhat"][b][sure]).all(), (steps, b)
                checked += 1
            assert (g_tok[b][~newly] == tokens[b][~newly]).all()            # Eq. 5: nothing else moves
        tokens, masked = g_tok.copy(), g_msk.copy()                          # the next step starts from the GPU's state
        steps += 1
    assert steps >= 4 and checked >= steps                                   # many steps, most of them comparable
    if B * K > 128:
        assert any(c > 128 for c in counts) and any(64 < c <= 128 for c in counts)
        assert any(32 < c <= 64 for c in counts) and any(0 < c <= 32 for c in counts)
