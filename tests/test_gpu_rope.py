"""GPU parity: sdllm_rope_gathered against the fp64 oracle (paper section 3.3, sentence before Eq. 7:
pruned rows keep their original RoPE position ids).
Bar: fp32 |err| <= 2e-6 * max(1, |want|) (cos / sin come from double precision; two fp32 products
and one sum per element); bf16: the fp32 result rounded to nearest even, i.e. at most half a bf16
ulp (2^-9 relative) plus the fp32 error -- tested as |err| <= 2^-8 * max(1e-2, |want|)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import rope_gathered as oracle_rope
from gpu_util import to_dev, to_f64_host

pytestmark = pytest.mark.gpu


def _inputs(dtype, B, H, D, K, S, seed):
    t = wl.make_custom_attention_inputs(dtype, B, H, H, D, 0, 1, K, max(S, 1), (), seed=seed)
    return t["q_block"], t["q_suffix"]


def _check(sd, dtype, B, H, D, K, S, keep, pos0, base, interleaved, in_place, seed=0):
    xb, xs = _inputs(dtype, B, H, D, K, S, seed)
    keep = np.asarray(keep, dtype=np.int32)
    dxb, dxs = to_dev(xb), to_dev(xs)
    dkeep = torch.from_numpy(keep).cuda() if keep.size else None
    if in_place:
        ob, os_ = dxb.clone(), dxs.clone()
        sd.rope_gathered(ob, os_ if keep.size else None, dkeep, pos0, base, interleaved)
    else:
        ob = torch.full_like(dxb, float("nan")); os_ = torch.full_like(dxs, 7.0)
        sd.rope_gathered(dxb, dxs if keep.size else None, dkeep, pos0, base, interleaved,
                         out_block=ob, out_suffix=os_ if keep.size else None)
    torch.cuda.synchronize()
    fb, fs = wl.to_f64(xb), wl.to_f64(xs)
    want_b, want_s = oracle_rope(fb, fs, keep, pos0, base, interleaved)
    got_b, got_s_full = to_f64_host(ob), to_f64_host(os_)
    if dtype == "fp32":
        tol = lambda w: 2e-6 * np.maximum(1.0, np.abs(w))
    else:
        tol = lambda w: 2.0 ** -8 * np.maximum(1e-2, np.abs(w))
    assert (np.abs(got_b - want_b) <= tol(want_b)).all()
    if keep.size:
        got_s = got_s_full[:, :, keep, :]
        assert (np.abs(got_s - want_s) <= tol(want_s)).all()
    # rows that are not kept are untouched: bit-identical to the input (in place) or to the fill value
    rest = np.setdiff1d(np.arange(S), keep)
    if rest.size:
        if in_place:
            assert np.array_equal(got_s_full[:, :, rest, :], fs[:, :, rest, :])
        else:
            assert (got_s_full[:, :, rest, :] == 7.0).all()
    return np.abs(got_b - want_b).max()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("B,H,D,K,S,keep,pos0,base", [
    (1, 2, 64, 4, 8, (0, 1, 7), 10, 10000.0),
    (2, 3, 128, 32, 100, tuple(range(31)) + (99,), 608, 500000.0),
    (1, 1, 16, 1, 0, (), 0, 10000.0),                         # one row, no suffix, position 0 = identity
    (3, 5, 256, 33, 70, tuple(range(5, 60, 3)), 4000, 1000000.0),
    (1, 40, 128, 7, 9, (8,), 123456, 10000.0),                # many heads: several chunks; large position
])
def test_rope_shapes(gpu_lib, dtype, interleaved, B, H, D, K, S, keep, pos0, base):
    _check(gpu_lib, dtype, B, H, D, K, S, keep, pos0, base, interleaved, in_place=False, seed=D + K)
    _check(gpu_lib, dtype, B, H, D, K, S, keep, pos0, base, interleaved, in_place=True, seed=D + K + 1)


def test_rope_cfg2_shape_q_and_k(gpu_lib):
    """The bench workload's shapes: 32 query heads, the paper-rule keep list (31 nearest + trailing)."""
    w = wl.WORKLOADS["cfg2"]
    keep = wl.make_keep_idx(w)
    err = _check(gpu_lib, "bf16", w.B, w.Hq, w.D, w.K, w.S, keep, w.P, 500000.0, False, in_place=True)
    print(f"rope cfg2 max-abs err {err:.3e}")


def test_rope_then_attention_matches_oracle_chain(gpu_lib):
    """RoPE'd q and k (block + kept suffix) fed to the attention call: the chain of the two oracles
    gives the same output.  The cache holds already rotated keys (that is how a prefix cache is kept)."""
    from oracle import block_attention as oracle_attention, rope_rotate
    sd = gpu_lib
    B, Hq, Hkv, D, P, K, S = 1, 4, 2, 128, 96, 32, 64
    keep = np.array(list(range(16)) + [63], dtype=np.int32)
    t = wl.make_custom_attention_inputs("bf16", B, Hq, Hkv, D, P, P, K, S, keep, seed=21)
    d = {k: to_dev(v) for k, v in t.items() if k != "keep_idx"}
    dkeep = torch.from_numpy(keep).cuda()
    sd.rope_gathered(d["q_block"], d["q_suffix"], dkeep, P, 10000.0)
    sd.rope_gathered(d["k_block"], d["k_suffix"], dkeep, P, 10000.0)
    out = sd.block_attention(d["q_block"], d["q_suffix"], d["k_cache"], d["v_cache"], d["k_block"], d["v_block"],
                             d["k_suffix"], d["v_suffix"], dkeep, P)
    torch.cuda.synchronize()
    f = {k: wl.to_f64(v) for k, v in t.items() if k != "keep_idx"}
    def rot(xb, xs):
        ob = rope_rotate(xb, P + np.arange(K), 10000.0)
        os_ = xs.copy()
        os_[:, :, keep, :] = rope_rotate(xs[:, :, keep, :], P + K + keep, 10000.0)
        # the GPU keeps bf16 between the two calls: round the oracle's intermediate the same way
        rnd = lambda a: wl.to_f64(wl.f32_to_bf16_bits(a.astype(np.float32)))
        return rnd(ob), rnd(os_)
    qb, qs = rot(f["q_block"], f["q_suffix"])
    kb, ks = rot(f["k_block"], f["k_suffix"])
    want = oracle_attention(qb, qs, f["k_cache"], f["v_cache"], kb, f["v_block"], ks, f["v_suffix"], keep, P, None)
    err = np.abs(to_f64_host(out) - want).max()
    print(f"rope -> attention chain max-abs err {err:.3e}")
    assert err <= 2e-2
