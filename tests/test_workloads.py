"""The seeded generators: shapes of the workload configurations, determinism, bf16 rounding."""
import numpy as np

import workloads as wl


def test_config_shapes():
    w = wl.WORKLOADS
    assert (w["cfg1"].P, w["cfg1"].S, w["cfg1"].Nq, w["cfg1"].Nkv) == (64, 224, 48, 112)
    assert (w["cfg2"].P, w["cfg2"].S, w["cfg2"].Nq, w["cfg2"].Nkv) == (608, 128, 64, 672)
    assert (w["cfg3A"].P, w["cfg3A"].S, w["cfg3A"].Nq, w["cfg3A"].Nkv) == (1024, 992, 64, 1088)
    assert (w["cfg3B"].Nq, w["cfg3B"].Nkv) == (1024, 2048)
    assert (w["cfg4"].P, w["cfg4"].S, w["cfg4"].Nq, w["cfg4"].Nkv) == (512, 224, 64, 576)
    assert (w["cfg5"].P, w["cfg5"].S, w["cfg5"].Nq, w["cfg5"].Nkv) == (5120, 960, 128, 5248)
    assert w["cfg2"].attn_flops() == 4 * 32 * 64 * 672 * 128


def test_keep_idx_rules():
    k = wl.make_keep_idx(wl.WORKLOADS["cfg2"])
    assert k.dtype == np.int32 and k.shape == (32,)
    assert list(k[:31]) == list(range(31)) and k[31] == 127
    assert list(wl.make_keep_idx(wl.WORKLOADS["cfg1"])) == list(range(16))
    assert list(wl.make_keep_idx(wl.WORKLOADS["cfg3B"])) == list(range(992))
    assert (np.diff(k) > 0).all()


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-9 rounds up
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0078125 and back[3] == 1.015625
    assert back[4] == -2.5 and back[5] == 0.0 and back[6] == 3.140625
    assert wl.to_f64(bits).dtype == np.float64


def test_determinism_and_independence():
    w = wl.WORKLOADS["small_bf16"]
    a = wl.make_attention_inputs(w, seed=0)
    b = wl.make_attention_inputs(w, seed=0)
    c = wl.make_attention_inputs(w, seed=1)
    for k in a:
        assert (a[k] == b[k]).all()
    assert (a["q_block"] != c["q_block"]).any()
    assert (a["k_block"] != a["v_block"]).any()
    u = wl.make_unmask_inputs(w, seed=0)
    assert u["logits"].shape == (w.B, w.K, w.V) and u["masked"].sum(axis=1).tolist() == [16, 16]
    assert (u["tokens"][u["masked"] != 0] == wl.MASK_TOKEN).all()


def test_boost_and_fraction_rules():
    w = wl.WORKLOADS["cfg4boost"]
    m = wl.make_masked(w, seed=0)
    assert m.shape == (16, 32) and (m.sum(axis=1) >= 3).all() and len(set(m.sum(axis=1).tolist())) > 3
    lg = wl.to_f64(wl.make_logits("bf16", 2, 4, 3000, 4.0, True, seed=3))
    assert (lg.max(axis=2) >= 17.9).all() and (lg.max(axis=2) <= 26.1).all()
