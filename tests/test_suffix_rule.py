"""The suffix keep-index rule (paper Eq. 7): pins for the oracle and host-side parity of the C ABI helper
(integer only, runs without a GPU)."""
import os

import pytest

import paper_2601_17917_amd as sd
from oracle import suffix_keep_indices as oracle_keep


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sd.LIB_PATH):
        from paper_2601_17917_amd.build import build
        build(verbose=False)
    return sd.load_library()


def test_oracle_closed_forms():
    # gen 256 in blocks of 32, block 3 active: suffix = 128 positions; window of 1 block + trailing
    assert oracle_keep(512, 256, 32, 3, 1) == list(range(32)) + [127]
    # window 0: only the trailing position; no trailing: nothing
    assert oracle_keep(64, 256, 32, 0, 0) == [223]
    assert oracle_keep(64, 256, 32, 0, 0, keep_trailing=False) == []
    # window reaching the end keeps everything exactly once
    assert oracle_keep(10, 128, 32, 1, 5) == list(range(64))
    assert oracle_keep(10, 128, 32, 1, 2) == list(range(64))
    # last block: empty suffix
    assert oracle_keep(10, 128, 32, 3, 2) == []
    # count = w*K + 1 while the window stays inside the suffix (the sizes of the paper's hyper-parameter table)
    for w_tokens in (32, 64, 96, 128, 256):
        assert len(oracle_keep(100, 1024, 32, 0, w_tokens // 32)) == w_tokens + 1


def test_oracle_brute_force_membership():
    """A position is kept iff its block index is in (c, c+w] or it is the final position."""
    p_L, L, K = 7, 96, 8
    for c in range(12):
        for w in range(0, 14):
            got = set(oracle_keep(p_L, L, K, c, w))
            start = p_L + (c + 1) * K
            want = set()
            for pos in range(start, p_L + L):
                n = (pos - p_L) // K
                if c < n <= c + w or pos == p_L + L - 1:
                    want.add(pos - start)
            assert got == want, (c, w)


@pytest.mark.parametrize("prompt,gen,K", [(64, 256, 32), (512, 256, 32), (100, 1024, 32), (7, 96, 8), (4096, 2048, 64)])
def test_abi_helper_matches_oracle(lib, prompt, gen, K):
    N = gen // K
    for c in range(N):
        S = gen - (c + 1) * K
        for w in (0, 1, 2, 3, 8, N + 2):
            for trailing in (True, False):
                got = sd.suffix_keep_indices(S, K, w, trailing)
                assert got == oracle_keep(prompt, gen, K, c, w, trailing), (c, w, trailing)
                assert all(a < b for a, b in zip(got, got[1:]))
                assert all(0 <= i < S for i in got)


def test_abi_helper_validation(lib):
    import ctypes
    buf = (ctypes.c_int32 * 4)()
    n = ctypes.c_int32(0)
    assert lib.sdllm_suffix_keep_indices(100, 32, 1, 1, buf, 4, ctypes.byref(n)) == sd.ERR_INVALID_ARG   # capacity
    assert lib.sdllm_suffix_keep_indices(-1, 32, 1, 1, buf, 4, ctypes.byref(n)) == sd.ERR_INVALID_ARG
    assert lib.sdllm_suffix_keep_indices(10, 0, 1, 1, buf, 4, ctypes.byref(n)) == sd.ERR_INVALID_ARG
    assert lib.sdllm_suffix_keep_indices(10, 32, 1, 1, None, 4, ctypes.byref(n)) == sd.ERR_INVALID_ARG
    assert lib.sdllm_suffix_keep_indices(3, 32, 0, 1, buf, 4, ctypes.byref(n)) == sd.SDLLM_OK and n.value == 1 and buf[0] == 2


def test_workload_generator_uses_the_rule():
    import workloads as wl
    w = wl.WORKLOADS["cfg2"]
    assert list(wl.make_keep_idx(w)) == oracle_keep(w.prompt, w.gen, w.K, w.active_block, 1)[:31] + [w.S - 1]
