"""GPU: the calls of a decode step can be recorded into a HIP graph (stream capture) and replayed.

One step of a small multi-layer stack -- attention for every layer (with key-range splits, so the merge kernel
is in the graph), the confidence unmask, the KV append -- is captured once after sdllm_init() and replayed
several times, with eager work and synchronisations between the replays.  Every replay must be bit-identical to
the eager calls on the same inputs and agree with the oracle.  (Per-layer forward feeding Eq. 4: paper Eq. 3;
the step's kernels only launch: no memset or copy nodes.)"""
import numpy as np
import pytest
import torch

import workloads as wl
import oracle
from gpu_util import to_dev, to_f64_host, attention_error_ratio

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def test_step_graph_replays_match_eager_and_oracle(gpu_lib):
    sd = gpu_lib
    sd.init()
    w = wl.WORKLOADS["small_bf16"]
    L = 3
    layers = [wl.make_attention_inputs(w, seed=40 + l) for l in range(L)]
    dev = [{k: to_dev(v) for k, v in t.items()} for t in layers]
    k_caches = torch.stack([d["k_cache"] for d in dev]); v_caches = torch.stack([d["v_cache"] for d in dev])
    k_blocks = torch.stack([d["k_block"] for d in dev]); v_blocks = torch.stack([d["v_block"] for d in dev])
    caches0 = (k_caches.clone(), v_caches.clone())
    u = wl.make_unmask_inputs(w, seed=40)
    logits = to_dev(u["logits"])
    tok0, msk0 = torch.from_numpy(u["tokens"]).cuda(), torch.from_numpy(u["masked"]).cuda()
    eos0 = torch.zeros((w.B,), dtype=torch.uint8, device="cuda")

    def make_state():
        return dict(out=[torch.zeros((w.B, w.Hq, w.Nq, w.D), dtype=torch.bfloat16, device="cuda") for _ in range(L)],
                    tok=tok0.clone(), msk=msk0.clone(), conf=torch.full((w.B, w.K), -7.0, device="cuda"),
                    ncom=torch.zeros((w.B,), dtype=torch.int32, device="cuda"),
                    done=torch.zeros((w.B,), dtype=torch.uint8, device="cuda"), eos=eos0.clone())

    def bind(st, stream):
        calls = []
        for l, d in enumerate(dev):
            p = sd.attn_params(sd.BF16, w.B, w.Hq, w.Hkv, w.D, w.P, w.cap, w.K, w.S, w.n_keep, 0.0, 2)
            ws = torch.empty((sd.attention_workspace_bytes(p),), dtype=torch.uint8, device="cuda")
            calls.append(sd.bind_block_attention(d["q_block"], d["q_suffix"], k_caches[l], v_caches[l], d["k_block"],
                                                 d["v_block"], d["k_suffix"], d["v_suffix"], d["keep_idx"], w.P,
                                                 out=st["out"][l], kv_splits=2, workspace=ws, stream=stream))
        calls.append(sd.bind_confidence_unmask(logits, st["tok"], st["msk"], w.tau0, w.alpha, confidence=st["conf"],
                                               n_committed=st["ncom"], block_done=st["done"], eos_seen=st["eos"],
                                               eos_id=3, stream=stream))
        calls.append(sd.bind_kv_append(k_caches, v_caches, k_blocks, v_blocks, w.P, stream=stream))
        return calls

    # ---- eager
    eager = make_state()
    for call in bind(eager, torch.cuda.current_stream()):
        call()
    torch.cuda.synchronize()
    eager_caches = (k_caches.clone(), v_caches.clone())

    # ---- the oracle on the same inputs
    for l, t in enumerate(layers):
        f = {k: (wl.to_f64(v) if k != "keep_idx" else v) for k, v in t.items()}
        want = oracle.block_attention(f["q_block"], f["q_suffix"], f["k_cache"], f["v_cache"], f["k_block"], f["v_block"],
                                      f["k_suffix"], f["v_suffix"], f["keep_idx"], w.P)
        want_abs = oracle.block_attention(f["q_block"], f["q_suffix"], f["k_cache"], np.abs(f["v_cache"]), f["k_block"],
                                          np.abs(f["v_block"]), f["k_suffix"], np.abs(f["v_suffix"]), f["keep_idx"], w.P)
        assert attention_error_ratio(to_f64_host(eager["out"][l]), want, want_abs) <= 1.0
    ref = oracle.confidence_unmask(wl.to_f64(u["logits"]), u["tokens"], u["masked"], float(np.float32(w.tau0)),
                                   float(np.float32(w.alpha)), eos_id=3)
    band = (u["masked"] != 0) & (np.abs(np.nan_to_num(ref["confidence"]) - np.nan_to_num(ref["tau"])[:, None]) < 1e-3)
    assert not band.any(), "seeded input must not sit on the threshold"
    assert (eager["tok"].cpu().numpy() == ref["tokens"]).all() and (eager["msk"].cpu().numpy() == ref["masked"]).all()
    assert (eager["ncom"].cpu().numpy() == ref["n_committed"]).all()
    wk, wv = oracle.kv_append(np.stack([t["k_cache"] for t in layers]), np.stack([t["v_cache"] for t in layers]),
                              np.stack([t["k_block"] for t in layers]), np.stack([t["v_block"] for t in layers]), w.P)
    assert (_bits(eager_caches[0]) == wk).all() and (_bits(eager_caches[1]) == wv).all()

    # ---- capture once, replay several times
    k_caches.copy_(caches0[0]); v_caches.copy_(caches0[1])
    st = make_state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        calls = bind(st, side)                      # marshalling and workspace allocation happen before the capture
        torch.cuda.synchronize()
        graph.capture_begin()
        for call in calls:
            call()
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        # eager work and synchronisation between replays: restore the state the step mutates, poison the outputs
        st["tok"].copy_(tok0); st["msk"].copy_(msk0); st["eos"].copy_(eos0)
        st["conf"].fill_(-7.0); st["ncom"].fill_(-1); st["done"].fill_(9)
        for o in st["out"]:
            o.fill_(float(rep + 1))
        k_caches.copy_(caches0[0]); v_caches.copy_(caches0[1])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(st["out"][l].view(torch.int16), eager["out"][l].view(torch.int16)), (rep, l)
        for k in ("tok", "msk", "ncom", "done", "eos"):
            assert torch.equal(st[k], eager[k]), (rep, k)
        assert torch.equal(st["conf"], eager["conf"]), rep
        assert torch.equal(k_caches.view(torch.int16), eager_caches[0].view(torch.int16)), rep
        assert torch.equal(v_caches.view(torch.int16), eager_caches[1].view(torch.int16)), rep


def test_validate_keep_idx_on_device_lists(gpu_lib):
    sd = gpu_lib
    good = torch.tensor([0, 1, 2, 5, 31], dtype=torch.int32, device="cuda")
    sd.validate_keep_idx(good, 32)
    sd.validate_keep_idx(torch.from_numpy(wl.make_keep_idx(wl.WORKLOADS["cfg5"])).cuda(), wl.WORKLOADS["cfg5"].S)
    for bad, S in ((torch.tensor([0, 2, 2], dtype=torch.int32), 8),       # a duplicate would count a key twice
                   (torch.tensor([3, 1], dtype=torch.int32), 8),          # decreasing
                   (torch.tensor([0, 8], dtype=torch.int32), 8),          # beyond the suffix
                   (torch.tensor([-1, 2], dtype=torch.int32), 8)):
        with pytest.raises(sd.SdllmError) as e:
            sd.validate_keep_idx(bad.cuda(), S)
        assert e.value.status == sd.ERR_INVALID_ARG


def test_init_and_first_calls_from_several_threads(gpu_lib):
    """sdllm_init and the launchers' own first-use set-up are safe when several threads run them at once (the
    opt-in of a kernel to its LDS size is idempotent and recorded atomically per device)."""
    import threading
    sd = gpu_lib
    w = wl.WORKLOADS["small_bf16"]
    t = wl.make_attention_inputs(w, seed=77)
    d = {k: to_dev(v) for k, v in t.items()}
    torch.cuda.synchronize()
    outs, errors = [None] * 6, []

    def work(i):
        try:
            torch.cuda.set_device(0)
            sd.init()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.default_stream())
            outs[i] = sd.block_attention(d["q_block"], d["q_suffix"], d["k_cache"], d["v_cache"], d["k_block"], d["v_block"],
                                         d["k_suffix"], d["v_suffix"], d["keep_idx"], w.P, kv_splits=1 + i % 3, stream=s)
            s.synchronize()
        except Exception as e:          # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(6)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    f = {k: (wl.to_f64(v) if k != "keep_idx" else v) for k, v in t.items()}
    want = oracle.block_attention(f["q_block"], f["q_suffix"], f["k_cache"], f["v_cache"], f["k_block"], f["v_block"],
                                  f["k_suffix"], f["v_suffix"], f["keep_idx"], w.P)
    for o in outs:
        assert np.abs(to_f64_host(o) - want).max() <= 2e-2
