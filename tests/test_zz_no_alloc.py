"""GPU: sdllm_confidence_unmask_noalloc (the entry point that allocates nothing: its partial results live in a
device-resident array of the library) against sdllm_confidence_unmask with a caller workspace -- same kernels,
so every output must agree bit for bit (ids, mask, flags, counters and the confidences).  Two calls in a row on
the same GPU, the second with a smaller input, so that the shared array still holds the first call's contents."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _run(sd, entry, u, w, V=None):
    lg = to_dev(u["logits"])
    tk, mk = torch.from_numpy(u["tokens"]).cuda(), torch.from_numpy(u["masked"]).cuda()
    B, K = u["tokens"].shape
    conf = torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
    es = torch.zeros((B,), dtype=torch.uint8, device="cuda")
    ncom = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    done = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    entry(lg, tk, mk, w.tau0, w.alpha, V=V, confidence=conf, n_committed=ncom, block_done=done, eos_seen=es, eos_id=3)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in (tk, mk, conf, ncom, done, es)]


def test_noalloc_matches_workspace_entry_point_twice_in_a_row(gpu_lib):
    sd = gpu_lib
    # first call: the LLaDA-shaped batch of 8 sequences (256 rows x 126464, 8 vocabulary splits per row);
    # second call, right after it: the small ragged case (64 rows x 5000) -- fewer rows and fewer splits, so most
    # of the scratch still holds triples of the first call
    for name in ("cfg3A", "small_bf16"):
        w = wl.WORKLOADS[name]
        u = wl.make_unmask_inputs(w, seed=2)
        p = sd.unmask_params(sd.BF16, w.B, w.K, w.V, w.V, w.tau0, w.alpha)
        assert sd.unmask_workspace_bytes(p) <= sd.NOALLOC_SCRATCH_BYTES
        got = _run(sd, sd.confidence_unmask_noalloc, u, w)
        want = _run(sd, sd.confidence_unmask, u, w)
        for g, x, what in zip(got, want, ("tokens", "masked", "confidence", "n_committed", "block_done", "eos_seen")):
            assert g.dtype == x.dtype and g.tobytes() == x.tobytes(), (name, what)
        assert (got[3] >= 1).all()


def test_noalloc_call_replays_from_a_captured_graph(gpu_lib):
    """What the entry point is for: recorded into a HIP graph (no allocation, no workspace to keep alive) and
    replayed, with eager work between the replays; every replay must equal the eager workspace entry point."""
    sd = gpu_lib
    sd.init()                                            # scratch address looked up before the capture
    w = wl.WORKLOADS["small_bf16"]
    u = wl.make_unmask_inputs(w, seed=4)
    want = _run(sd, sd.confidence_unmask, u, w)
    lg = to_dev(u["logits"])
    tok0, msk0 = torch.from_numpy(u["tokens"]).cuda(), torch.from_numpy(u["masked"]).cuda()
    tk, mk = tok0.clone(), msk0.clone()
    B, K = u["tokens"].shape
    conf = torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
    es = torch.zeros((B,), dtype=torch.uint8, device="cuda")
    ncom = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    done = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call = sd.bind_confidence_unmask_noalloc(lg, tk, mk, w.tau0, w.alpha, confidence=conf, n_committed=ncom,
                                                 block_done=done, eos_seen=es, eos_id=3, stream=side)
        torch.cuda.synchronize()
        graph.capture_begin()
        call()
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        tk.copy_(tok0); mk.copy_(msk0); conf.fill_(-7.0); es.zero_(); ncom.fill_(-1); done.fill_(9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.cpu().numpy() for x in (tk, mk, conf, ncom, done, es)]
        for g, x, what in zip(got, want, ("tokens", "masked", "confidence", "n_committed", "block_done", "eos_seen")):
            assert g.tobytes() == x.tobytes(), (rep, what)


def test_noalloc_rejects_sizes_beyond_its_scratch(gpu_lib):
    sd = gpu_lib
    lib = sd.load_library()
    p = sd.unmask_params(sd.BF16, 64, 4096, 126464, 126464, 0.9, 0.3)           # 262144 rows: more triples than 1 MiB holds
    assert sd.unmask_workspace_bytes(p) > sd.NOALLOC_SCRATCH_BYTES
    vp = ctypes.c_void_p
    rc = lib.sdllm_confidence_unmask_noalloc(ctypes.byref(p), vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096),
                                             None, None)
    assert rc == sd.ERR_UNSUPPORTED and b"scratch" in lib.sdllm_last_error()
