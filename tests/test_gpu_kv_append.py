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


def test_append_cfg5_shape_sampled(gpu_lib):
    """Full-size launch (32 layers x 4 x 32 heads x 64 rows x 128): the oracle copy is cheap, so compare all."""
    L, B, Hkv, D, K, cap, P = 32, 4, 32, 128, 64, 256, 128      # cap reduced; the launch geometry depends on K, not cap
    t = wl.make_append_inputs("bf16", L, B, Hkv, D, K, cap, seed=5)
    kc, vc, kb, vb = (to_dev(t[k]) for k in ("k_caches", "v_caches", "k_blocks", "v_blocks"))
    gpu_lib.kv_append(kc, vc, kb, vb, P)
    torch.cuda.synchronize()
    want_k, want_v = oracle_append(t["k_caches"], t["v_caches"], t["k_blocks"], t["v_blocks"], P)
    assert (_bits(kc) == want_k).all() and (_bits(vc) == want_v).all()


def test_append_rejects_overflow(gpu_lib):
    t = wl.make_append_inputs("bf16", 1, 1, 1, 128, 32, 40, seed=6)
    kc, vc, kb, vb = (to_dev(t[k]) for k in ("k_caches", "v_caches", "k_blocks", "v_blocks"))
    with pytest.raises(gpu_lib.SdllmError) as e:
        gpu_lib.kv_append(kc, vc, kb, vb, 16)
    assert e.value.status == gpu_lib.ERR_INVALID_ARG
