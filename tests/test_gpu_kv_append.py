"""GPU parity: sdllm_kv_append against the oracle, bit for bit (paper section 3.3, prefix K/V reuse)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import kv_append as oracle_append
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


@pytest.mark.parametrize("dtype,L,B,Hkv,D,K,cap,P", [
    ("bf16", 1, 1, 4, 128, 32, 96, 64),
    ("bf16", 3, 2, 2, 128, 32, 200, 75),
    ("fp32", 2, 3, 1, 64, 32, 70, 38),
    ("bf16", 5, 2, 3, 64, 17, 40, 23),      # ragged sizes, last block flush with the cache end
    ("fp32", 1, 1, 1, 4, 1, 1, 0),          # smallest legal problem
])
def test_append_bit_exact(gpu_lib, dtype, L, B, Hkv, D, K, cap, P):
    t = wl.make_append_inputs(dtype, L, B, Hkv, D, K, cap, seed=3)
    kc, vc, kb, vb = (to_dev(t[k]) for k in ("k_caches", "v_caches", "k_blocks", "v_blocks"))
    gpu_lib.kv_append(kc, vc, kb, vb, P)
    torch.cuda.synchronize()
    want_k, want_v = oracle_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], P)
    assert (_bits(kc) == want_k).all()
    assert (_bits(vc) == want_v).all()


def test_append_do_append_flags(gpu_lib):
    t = wl.make_append_inputs("bf16", 2, 4, 2, 128, 32, 128, seed=4)
    kc, vc, kb, vb = (to_dev(t[k]) for k in ("k_caches", "v_caches", "k_blocks", "v_blocks"))
    flags = np.array([1, 0, 0, 1], dtype=np.uint8)
    gpu_lib.kv_append(kc, vc, kb, vb, 64, do_append=torch.from_numpy(flags).cuda())
    torch.cuda.synchronize()
    want_k, want_v = oracle_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], 64, do_append=flags)
    assert (_bits(kc) == want_k).all() and (_bits(vc) == want_v).all()


CANARY = 0x7FC1          # a NaN bit pattern no seeded draw produces


def test_append_cfg5_real_capacity(gpu_lib):
    """The long-context stack at its real size: 32 layers x 4 x 32 heads, cap = 6144 rows, P = 5120, K = 64 --
    two 6.4 GB caches, destination offsets far beyond 4 GiB.  The caches start as a canary pattern; afterwards
    (i) a seeded sample of (layer, batch, head) runs -- first and last of each included -- is compared with the
    oracle on slices copied back, neighbours on both sides included; (ii) over the WHOLE cache exactly the
    appended rows differ from the canary and they equal the blocks bit for bit."""
    L, B, Hkv, D, K, cap, P = 32, 4, 32, 128, 64, 6144, 5120
    t = wl.make_append_inputs("bf16", L, B, Hkv, D, K, K, seed=5)          # only the blocks are used
    kb, vb = to_dev(t["k_blocks"]), to_dev(t["v_blocks"])
    kc = torch.full((L, B, Hkv, cap, D), CANARY, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    vc = torch.full((L, B, Hkv, cap, D), CANARY, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    assert kc.numel() * 2 >= (6 << 30)          # offsets far beyond 4 GiB
    gpu_lib.kv_append(kc, vc, kb, vb, P)
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.Philox(key=6144))
    sample = {(0, 0, 0), (L - 1, B - 1, Hkv - 1), (L - 1, 0, 0), (0, B - 1, Hkv - 1), (21, 2, 31), (22, 0, 0)}
    while len(sample) < 40:
        sample.add((int(rng.integers(L)), int(rng.integers(B)), int(rng.integers(Hkv))))
    lo, hi = P - 3, P + K + 3
    for (l, b, h) in sorted(sample):
        for cache, blocks, host_blocks in ((kc, kb, t["k_blocks"]), (vc, vb, t["v_blocks"])):
            got = _bits(cache[l, b, h, lo:hi])
            before = np.full((1, 1, 1, hi - lo, D), CANARY, dtype=np.uint16)
            want, _ = oracle_append(before, before.copy(), host_blocks[l:l + 1, b:b + 1, h:h + 1],
                                    host_blocks[l:l + 1, b:b + 1, h:h + 1], P - lo)
            assert (got == want[0, 0, 0]).all(), (l, b, h)
    for cache, blocks in ((kc, kb), (vc, vb)):
        ci = cache.view(torch.int16)
        assert torch.equal(ci[:, :, :, P:P + K], blocks.view(torch.int16))
        touched = int((ci != CANARY).sum())
        assert touched == int((blocks.view(torch.int16) != CANARY).sum()) == L * B * Hkv * K * D


def test_append_padded_layer_strides(gpu_lib):
    """Layers that are not densely packed: cache layers 4096 elements apart beyond the dense size, block layers
    64 beyond.  The padding holds a canary and must be untouched; the layers themselves match the oracle."""
    L, B, Hkv, D, K, cap, P = 3, 2, 3, 128, 32, 100, 37
    t = wl.make_append_inputs("bf16", L, B, Hkv, D, K, cap, seed=8)
    dense_c, dense_b = B * Hkv * cap * D, B * Hkv * K * D
    pad_c, pad_b = 4096, 64
    bufs = {}
    for name, dense, pad in (("k_caches", dense_c, pad_c), ("v_caches", dense_c, pad_c),
                             ("k_blocks", dense_b, pad_b), ("v_blocks", dense_b, pad_b)):
        flat = torch.full((L, dense + pad), CANARY, dtype=torch.int16, device="cuda")
        flat[:, :dense] = torch.from_numpy(t[name].view(np.int16).reshape(L, dense)).cuda()
        bufs[name] = flat
    def view(name, shape):
        return bufs[name].view(torch.bfloat16)[:, :int(np.prod(shape))].unflatten(1, shape)

    kc, vc = view("k_caches", (B, Hkv, cap, D)), view("v_caches", (B, Hkv, cap, D))
    kb, vb = view("k_blocks", (B, Hkv, K, D)), view("v_blocks", (B, Hkv, K, D))
    assert kc.stride(0) == dense_c + pad_c and kb.stride(0) == dense_b + pad_b and not kc.is_contiguous()
    gpu_lib.kv_append(kc, vc, kb, vb, P)
    torch.cuda.synchronize()
    want_k, want_v = oracle_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], P)
    assert (_bits(kc.contiguous()) == want_k).all() and (_bits(vc.contiguous()) == want_v).all()
    for name, dense in (("k_caches", dense_c), ("v_caches", dense_c), ("k_blocks", dense_b), ("v_blocks", dense_b)):
        assert bool((bufs[name][:, dense:] == CANARY).all()), name


def test_append_rejects_overflow(gpu_lib):
    t = wl.make_append_inputs("bf16", 1, 1, 1, 128, 32, 40, seed=6)
    kc, vc, kb, vb = (to_dev(t[k]) for k in ("k_caches", "v_caches", "k_blocks", "v_blocks"))
    with pytest.raises(gpu_lib.SdllmError) as e:
        gpu_lib.kv_append(kc, vc, kb, vb, 16)
    assert e.value.status == gpu_lib.ERR_INVALID_ARG
