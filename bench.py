#!/usr/bin/env python3
"""Benchmark of one block-wise diffusion decode step on one MI355X.

A step = one pass of the whole hot path over one batch of seeded synthetic input that is already
resident in HBM: pruned-suffix attention for every layer of the workload, the confidence-aware
unmask over the block's logits, and the append of the block's K/V to the prefix caches.
Prints ONE JSON line (metric: committed tokens per second of decode-step time), with the roofline
figures of the dominant kernel (HIP events inside the timed region) and the CPU oracle timed on
this machine's host cores as a baseline.  Outside the timed step it also reports per-kernel timings, the fused
vocabulary projection + unmask call, and what plain read / copy / matrix-instruction kernels reach on the box.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--graph]

The default workload is the largest single-GPU one: the 32-layer long-context stack (cfg5).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
# vector-ALU issue slots the unmask rows kernel spends per logit (from its instruction mix per 32 logits of a lane:
# see the kernel's header comment), v_exp_f32 weighted 2.4
UNMASK_VALU_SLOTS_PER_ELEMENT = {"bf16": (156 + 33 * 2.4) / 32.0, "fp32": (124 + 33 * 2.4) / 32.0}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg5", choices=[k for k in wl.WORKLOADS if k != "small_bf16"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region (roofline.achieved = null)")
    ap.add_argument("--event-every", type=int, default=0,
                    help="bracket the calls of a step with HIP events on every n-th timed step (0 = every step for the "
                         "multi-layer stack, whose step is milliseconds long; every 8th for the single-layer workloads, "
                         "where an event costs about as much as a small kernel and would distort the step time)")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="before the warm-up steps, keep the GPU busy with the step's attention calls for this long "
                         "(wall clock) so that a short run is timed at the steady clock a long one reaches by itself "
                         "(20 timed steps read 2.5 %% slower without it); 0 = off")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step (state restore + every call) as ONE captured HIP graph instead of launching it "
                         "eagerly; the JSON line then describes the graph replays (per-call events are not taken)")
    ap.add_argument("--no-lm-head", action="store_true",
                    help="skip the per-kernel figure of the fused vocabulary projection + unmask (it draws the "
                         "V x Hd projection, about 1 GB, on the device)")
    ap.add_argument("--kv-splits", type=int, default=0, help="force the attention key-range split count")
    ap.add_argument("--kv-copies", type=int, default=0,
                    help="single-layer workloads: number of distinct K/V/Q sets the steps cycle through, so that a "
                         "step reads its operands from HBM and not from the 256 MB last-level cache a previous step "
                         "left them in (0 = as many as make the sets exceed 512 MB, at most 64)")
    return ap.parse_args()


def to_dev(x):
    import torch
    if isinstance(x, np.ndarray):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(x).cuda()
    return x


class Step:
    """All device buffers of one workload, allocated before the timed region."""

    def __init__(self, sd, w: wl.Workload, seed: int, n_states: int, kv_splits: int = 0, kv_copies: int = 0):
        import torch
        self.sd, self.w = sd, w
        self.layers = []
        for layer in range(w.n_layers):
            if w.n_layers > 1:
                t = wl.make_attention_inputs_device(w, seed, layer)
            else:
                t = {k: to_dev(v) for k, v in wl.make_attention_inputs(w, seed, layer).items()}
            self.layers.append(t)
        # A real model walks through the caches of all its layers between two visits of the same one; a
        # single-layer workload that re-read one set of operands every step would find them in the
        # last-level cache.  Cycle through enough distinct sets (same shapes and law, drawn on the device).
        self.copies = 1
        if w.n_layers == 1 and w.dtype == "bf16":
            self.copies = kv_copies if kv_copies > 0 else min(64, max(1, -(-(512 << 20) // w.attn_bytes())))
            for c in range(1, self.copies):
                self.layers.append(wl.make_attention_inputs_device(w, seed, 1000 + c))
        dt = self.layers[0]["q_block"].dtype
        self.out = torch.empty((w.B, w.Hq, w.Nq, w.D), dtype=dt, device="cuda")
        self.attn_p = sd.attn_params(sd.FP32 if w.dtype == "fp32" else sd.BF16, w.B, w.Hq, w.Hkv, w.D, w.P, w.cap,
                                     w.K, w.S, w.n_keep, 0.0, kv_splits)
        self.attn_ws = torch.empty((max(sd.attention_workspace_bytes(self.attn_p), 16),), dtype=torch.uint8, device="cuda")
        self.plan = sd.plan_attention(self.attn_p)
        # unmask state: one private copy of (tokens, masked) per step, so that every step does the same work
        u = wl.make_unmask_inputs(w, seed)
        self.host_unmask = u
        self.logits = to_dev(u["logits"])
        self.tokens = to_dev(np.ascontiguousarray(np.broadcast_to(u["tokens"], (n_states,) + u["tokens"].shape)))
        self.masked = to_dev(np.ascontiguousarray(np.broadcast_to(u["masked"], (n_states,) + u["masked"].shape)))
        self.n_committed = torch.zeros((n_states, w.B), dtype=torch.int32, device="cuda")
        self.block_done = torch.zeros((n_states, w.B), dtype=torch.uint8, device="cuda")
        self.eos_seen = torch.zeros((w.B,), dtype=torch.uint8, device="cuda")
        self.unmask_p = sd.unmask_params(sd.FP32 if w.dtype == "fp32" else sd.BF16, w.B, w.K, w.V, w.V, w.tau0, w.alpha)
        self.unmask_ws = torch.empty((max(sd.unmask_workspace_bytes(self.unmask_p), 16),), dtype=torch.uint8, device="cuda")
        # append: the block K/V of every layer into every layer's cache (one launch).  Single-layer workloads
        # append into the layer's own cache; the stack keeps [L,...] tensors so that one launch covers all layers.
        if w.n_layers > 1:
            self.k_caches = torch.stack([t["k_cache"] for t in self.layers])
            self.v_caches = torch.stack([t["v_cache"] for t in self.layers])
            for l, t in enumerate(self.layers):          # attention reads the stacked storage: no second copy
                t["k_cache"], t["v_cache"] = self.k_caches[l], self.v_caches[l]
            self.k_blocks = torch.stack([t["k_block"] for t in self.layers])
            self.v_blocks = torch.stack([t["v_block"] for t in self.layers])
        else:
            t = self.layers[0]                           # the append goes into the first set's cache
            self.k_caches, self.v_caches = t["k_cache"][None], t["v_cache"][None]
            self.k_blocks, self.v_blocks = t["k_block"][None], t["v_block"][None]

        # marshal every call once: in the loop a call is one foreign-function call
        self.kv_splits = kv_splits
        self.attention = self._bind_attention(None)
        self.unmask = [self._bind_unmask(i, None) for i in range(n_states)]
        self.append = sd.bind_kv_append(self.k_caches, self.v_caches, self.k_blocks, self.v_blocks, w.P)
        torch.cuda.synchronize()

    def _bind_attention(self, stream):
        sd, w, nk = self.sd, self.w, self.w.n_keep
        return [sd.bind_block_attention(
            t["q_block"], t["q_suffix"] if nk else None, t["k_cache"], t["v_cache"], t["k_block"], t["v_block"],
            t["k_suffix"] if nk else None, t["v_suffix"] if nk else None, t["keep_idx"] if nk else None, w.P,
            out=self.out, kv_splits=self.kv_splits, workspace=self.attn_ws, stream=stream) for t in self.layers]

    def _bind_unmask(self, i, stream):
        sd, w = self.sd, self.w
        return sd.bind_confidence_unmask(
            self.logits, self.tokens[i], self.masked[i], w.tau0, w.alpha, n_committed=self.n_committed[i],
            block_done=self.block_done[i], eos_seen=self.eos_seen, workspace=self.unmask_ws, stream=stream)

    def bind_on(self, stream):
        """The calls of one step on state slot 0, bound to `stream` (for stream capture)."""
        attn = self._bind_attention(stream)
        attn = attn[:1] if self.w.n_layers == 1 else attn
        return attn + [self._bind_unmask(0, stream),
                       self.sd.bind_kv_append(self.k_caches, self.v_caches, self.k_blocks, self.v_blocks, self.w.P,
                                              stream=stream)]

    def run(self, i: int, events=None):
        """One step on state slot i.  `events`: five HIP events recorded on the launch stream around the layer-0
        attention call, the remaining layers, the unmask call and the append call."""
        if self.w.n_layers == 1:
            calls = (self.attention[i % self.copies],)
        else:
            calls = self.attention
        if events is not None:
            events[0].record()
            calls[0]()
            events[1].record()
            for call in calls[1:]:
                call()
            events[2].record()
            self.unmask[i]()
            events[3].record()
            self.append()
            events[4].record()
        else:
            for call in calls:
                call()
            self.unmask[i]()
            self.append()


def time_kernel(fn, iters=50, warm=5):
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters     # ms per call, back-to-back launches


def time_call_with_events(prepare, call, iters=50, warm=5):
    """Mean HIP-event time (ms) of `call()` alone: `prepare()` (untimed; e.g. restoring the state the call
    mutates) runs before every call, the event pair brackets only the call on the stream it is launched on."""
    import torch
    pairs = []
    for it in range(warm + iters):
        prepare()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        call()
        e1.record()
        if it >= warm:
            pairs.append((e0, e1))
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(b) for a, b in pairs]))


def cpu_baseline(w: wl.Workload, seed: int):
    """The oracle, as it stands, on this machine's host cores: one decode step (bounded sample for the
    big workloads).  Returns the cpu_baseline object."""
    from threadpoolctl import threadpool_info
    import oracle
    t = wl.make_attention_inputs(w, seed, 0) if w.n_layers == 1 and w.attn_flops() < 4e10 else None
    note = []
    # --- attention: all (batch, head) pairs when cheap, else a sample of pairs scaled up
    n_pairs = w.B * w.Hq
    per_pair_flops = 4 * w.Nq * w.Nkv * w.D
    sample_pairs = max(1, min(n_pairs, int(2e10 // per_pair_flops)))
    rng = np.random.default_rng(seed)

    def rand(*shape):
        return rng.standard_normal(shape)

    g = w.Hq // w.Hkv
    hq_s = min(w.Hq, max(g, sample_pairs))
    hq_s -= hq_s % g
    hkv_s = hq_s // g
    b_s = max(1, min(w.B, sample_pairs // hq_s))
    keep = wl.make_keep_idx(w)
    if t is not None:      # the workload's own tensors (cheap to draw), restricted to the sampled pairs
        f = {k: wl.to_f64(v) for k, v in t.items() if k != "keep_idx"}
        args = (f["q_block"][:b_s, :hq_s], f["q_suffix"][:b_s, :hq_s], f["k_cache"][:b_s, :hkv_s], f["v_cache"][:b_s, :hkv_s],
                f["k_block"][:b_s, :hkv_s], f["v_block"][:b_s, :hkv_s], f["k_suffix"][:b_s, :hkv_s], f["v_suffix"][:b_s, :hkv_s])
    else:                  # same shapes and law drawn directly in fp64 (the oracle's time does not depend on values)
        args = (rand(b_s, hq_s, w.K, w.D), rand(b_s, hq_s, w.S, w.D), rand(b_s, hkv_s, w.P, w.D), rand(b_s, hkv_s, w.P, w.D),
                rand(b_s, hkv_s, w.K, w.D), rand(b_s, hkv_s, w.K, w.D), rand(b_s, hkv_s, w.S, w.D), rand(b_s, hkv_s, w.S, w.D))
    t0 = time.perf_counter()
    oracle.block_attention(*args, keep, w.P)
    t_attn_sample = time.perf_counter() - t0
    frac = (b_s * hq_s) / n_pairs
    t_attn = t_attn_sample / frac * w.n_layers
    note.append(f"attention: {b_s * hq_s} of {n_pairs} (batch, head) pairs of one layer"
                + (f", scaled x{n_pairs / (b_s * hq_s):.0f} x {w.n_layers} layers" if frac < 1 or w.n_layers > 1 else ""))
    # --- unmask: a bounded number of sequences, scaled
    u = wl.make_unmask_inputs(w, seed)
    masked_rows = int((u["masked"] != 0).sum())
    b_u = w.B
    while b_u > 1 and int((u["masked"][:b_u] != 0).sum()) * w.V > 4e7:
        b_u //= 2
    lg = wl.to_f64(u["logits"][:b_u])
    t0 = time.perf_counter()
    res = oracle.confidence_unmask(lg, u["tokens"][:b_u], u["masked"][:b_u], float(np.float32(w.tau0)), float(np.float32(w.alpha)))
    t_unmask_sample = time.perf_counter() - t0
    rows_s = int((u["masked"][:b_u] != 0).sum())
    t_unmask = t_unmask_sample * masked_rows / max(rows_s, 1)
    committed_s = int(res["n_committed"].sum())
    # exclusion counts of the parity rule on the sampled sequences (the oracle's view): positions whose top-2
    # probability gap is under 1e-3, positions within 1e-3 of the threshold, sequences whose fallback is ambiguous
    was = u["masked"][:b_u] != 0
    n_gap = int((np.nan_to_num(res["gap"], nan=1.0)[was] < 1e-3).sum())
    band = was & (np.abs(np.nan_to_num(res["confidence"]) - np.nan_to_num(res["tau"])[:, None]) < 1e-3)
    n_amb = 0
    for b in range(b_u):
        c = np.sort(res["confidence"][b][was[b]])[::-1]
        if res["fallback"][b] and c.size > 1 and (c[0] - c[1]) <= 1e-6 * c[0]:
            n_amb += 1
    exclusions = {"sequences_checked": b_u, "masked_positions_checked": int(was.sum()), "top2_gap_lt_1e-3": n_gap,
                  "within_1e-3_of_threshold": int(band.sum()), "fallback_ambiguous_sequences": n_amb,
                  "oracle_tokens": res["tokens"], "oracle_masked": res["masked"], "band": band}
    note.append(f"unmask: {b_u} of {w.B} sequences ({rows_s} of {masked_rows} masked rows)" + (", scaled" if b_u < w.B else ""))
    # --- append: one layer, scaled
    a = wl.make_append_inputs(w.dtype, 1, w.B, w.Hkv, w.D, w.K, w.P + w.K, seed)
    t0 = time.perf_counter()
    oracle.kv_append(a["k_caches"], a["v_caches"], a["k_blocks"], a["v_blocks"], w.P)
    t_append = (time.perf_counter() - t0) * w.n_layers
    note.append("append: one layer" + (f" x {w.n_layers}" if w.n_layers > 1 else ""))
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"t_step_s": t_attn + t_unmask + t_append, "t_attention_s": t_attn, "t_unmask_s": t_unmask,
            "t_append_s": t_append, "cores": threads, "sample": "; ".join(note),
            "committed_sample": committed_s, "b_u": b_u, "exclusions": exclusions}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every box has one; the path shards by batch / head without "
              "communication); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2601_17917_amd as sd
    sd.load_library()                     # raises if the HIP library is missing: no fallback
    w = wl.WORKLOADS[args.workload]
    K, W = args.steps, args.warmup
    st = Step(sd, w, args.seed, K + W, args.kv_splits, args.kv_copies)

    sd.init()                             # every kernel opt-in done: the calls below only launch
    if args.prewarm_ms > 0:               # clocks: untimed attention calls (they mutate nothing), not steps
        t_end = time.perf_counter() + args.prewarm_ms * 1e-3
        while time.perf_counter() < t_end:
            for call in st.attention:
                call()
            torch.cuda.synchronize()
    use_ev = not args.no_kernel_events and not args.graph
    every = args.event_every if args.event_every > 0 else (1 if w.n_layers > 1 else 8)
    if args.graph:
        # the whole step as one graph: restore the state slot the unmask mutates (two small copy kernels), then
        # every call.  All replays work on slot 0, so every replay does the same work.
        tok0, msk0 = st.tokens[0].clone(), st.masked[0].clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            calls = st.bind_on(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            graph.capture_begin()
            st.tokens[0].copy_(tok0); st.masked[0].copy_(msk0)
            for call in calls:
                call()
            graph.capture_end()
        torch.cuda.synchronize()
        for i in range(W):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st.n_committed[W:] = st.n_committed[0]
        evs = {}
    else:
        for i in range(W):
            st.run(i)
        torch.cuda.synchronize()
        evs = {i: [torch.cuda.Event(enable_timing=True) for _ in range(5)] for i in range(0, K, every)} if use_ev else {}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            st.run(W + i, evs.get(i))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    committed = st.n_committed[W:].sum(dim=1).cpu().numpy()
    assert (committed == committed[0]).all(), "every timed step must do the same work"
    committed_per_step = int(committed[0])
    value = committed_per_step / (ms_per_step * 1e-3)

    # ---- dominant kernel: the attention call of layer 0 (main kernel + split merge), events inside the timed region
    def ev_mean(a, b):
        return float(np.mean([e[a].elapsed_time(e[b]) for e in evs.values()])) if use_ev else None

    # the attention call: mean over the layers of a step (events before the first and after the last layer); the
    # first layer's own duration is reported too (it follows the previous step's append and reads 3-4 % slower)
    layer0_ms_ev, unmask_ms_ev, append_ms_ev = ev_mean(0, 1), ev_mean(2, 3), ev_mean(3, 4)
    # (a single-layer workload has just the one call between events 0 and 1; going on to event 2 would add an event)
    attn_ms_ev = (ev_mean(0, 2) / w.n_layers if w.n_layers > 1 else layer0_ms_ev) if use_ev else None
    attn_bytes = w.attn_bytes()
    attn_flops = w.attn_flops()
    intensity = attn_flops / attn_bytes
    bound = "mfma" if intensity > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9) and w.dtype == "bf16" else "hbm"

    # ---- per-kernel timings outside the timed region (back-to-back launches of one call)
    rot = [0]

    def attention_rotating():                           # same rotation as the timed steps
        st.attention[rot[0] % len(st.attention)]()
        rot[0] += 1

    t_attn = time_kernel(attention_rotating, iters=300, warm=100)    # long enough to sit at the steady clock
    # the unmask call alone: HIP events around the real call, the state slot restored (untimed) before every call
    tok_fresh, msk_fresh = to_dev(st.host_unmask["tokens"]), to_dev(st.host_unmask["masked"])

    def restore_slot():
        st.tokens[1].copy_(tok_fresh); st.masked[1].copy_(msk_fresh)

    t_unm = time_call_with_events(restore_slot, st.unmask[1])
    t_app = time_kernel(st.append)
    # RoPE of the pruned q and k rows (the step before the attention call; NOT part of the timed step):
    # in place on copies, q and k back to back
    t0_ = st.layers[0]
    nk = w.n_keep
    rq = sd.bind_rope_gathered(t0_["q_block"].clone(), t0_["q_suffix"].clone() if nk else None,
                               t0_["keep_idx"] if nk else None, w.P, 500000.0)
    rk = sd.bind_rope_gathered(t0_["k_block"].clone(), t0_["k_suffix"].clone() if nk else None,
                               t0_["keep_idx"] if nk else None, w.P, 500000.0)

    def rope_qk():
        rq(); rk()

    t_rope = time_kernel(rope_qk)
    rope_bytes = 2 * w.B * (w.Hq + w.Hkv) * w.Nq * w.D * w.elem_bytes      # rows read + rows written
    masked_rows = int((st.host_unmask["masked"] != 0).sum())
    unmask_bytes = masked_rows * w.V * w.elem_bytes
    append_bytes = 2 * 2 * w.n_layers * w.B * w.Hkv * w.K * w.D * w.elem_bytes
    kernels = {
        "attention_call": {"ms": t_attn, "tflops": attn_flops / t_attn / 1e9, "gbs": attn_bytes / t_attn / 1e6,
                           "frac_mfma_peak": attn_flops / t_attn / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                           "frac_hbm_peak": attn_bytes / t_attn / 1e6 / HBM_PEAK_GBS,
                           "kv_splits": st.plan.kv_splits, "workgroups": st.plan.workgroups, "layers_per_step": w.n_layers,
                           "operand_sets_cycled": len(st.attention)},
        "unmask_call": {"ms": t_unm, "gbs": unmask_bytes / t_unm / 1e6, "frac_hbm_peak": unmask_bytes / t_unm / 1e6 / HBM_PEAK_GBS,
                        "masked_rows": masked_rows},
        "append_call": {"ms": t_app, "gbs": append_bytes / t_app / 1e6, "frac_hbm_peak": append_bytes / t_app / 1e6 / HBM_PEAK_GBS},
        "rope_q_and_k_calls": {"ms": t_rope, "gbs": rope_bytes / t_rope / 1e6, "frac_hbm_peak": rope_bytes / t_rope / 1e6 / HBM_PEAK_GBS,
                               "in_timed_step": False},
    }
    if w.dtype == "bf16" and not args.no_lm_head:
        # the unmask fed by the vocabulary projection of the hidden states instead of stored logits (the step on
        # the other side of Eq. 4; NOT part of the timed step, whose logits are inputs).  W (V x Hd) is larger
        # than the last-level cache, so every call streams it from HBM.
        lm = wl.make_lm_head_inputs_device(w, args.seed)
        tok0 = torch.from_numpy(lm["tokens"]).cuda(); msk0 = torch.from_numpy(lm["masked"]).cuda()
        tok, msk = tok0.clone(), msk0.clone()

        def lm_restore():
            tok.copy_(tok0); msk.copy_(msk0)

        lm_rows = int((lm["masked"] != 0).sum())
        lm_bytes = w.V * w.Hd * 2 + lm_rows * w.Hd * 2
        lm_flops = 2.0 * lm_rows * w.V * w.Hd

        def time_lm(weight):
            lm_call = sd.bind_lm_head_unmask(lm["hidden"], weight, tok, msk, w.tau0, w.alpha)
            t_lm = time_call_with_events(lm_restore, lm_call, iters=20)
            return {"ms": t_lm, "gbs": lm_bytes / t_lm / 1e6, "frac_hbm_peak": lm_bytes / t_lm / 1e6 / HBM_PEAK_GBS,
                    "tflops": lm_flops / t_lm / 1e9, "frac_mfma_peak": lm_flops / t_lm / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                    "masked_rows": lm_rows, "hidden": w.Hd, "in_timed_step": False}

        kernels["lm_head_unmask_call"] = time_lm(lm["lm_weight"])
        # the same call over the image that sdllm_lm_head_pack_weight writes once for a model weight
        packed_w = sd.lm_head_pack_weight(lm["lm_weight"])
        kernels["lm_head_unmask_call_packed_weight"] = time_lm(packed_w)
        del lm, packed_w
    # ---- what plain kernels reach on this machine (library diagnostics): the practical ceilings next to the
    # published peaks the fractions are quoted against
    buf = torch.empty((1 << 31,), dtype=torch.uint8, device="cuda").random_(0, 256)
    half = buf.numel() // 2
    sink = torch.zeros((16,), dtype=torch.float32, device="cuda")
    t_rd = time_kernel(lambda: sd.probe_read(buf, sink), iters=10, warm=2)
    t_cp = time_kernel(lambda: sd.probe_copy(buf[half:], buf[:half]), iters=10, warm=2)
    iters_mfma = 4000
    fl = sd.probe_mfma_bf16(iters_mfma, 0, sink)
    t_m0 = time_kernel(lambda: sd.probe_mfma_bf16(iters_mfma, 0, sink), iters=5, warm=1)
    t_m1 = time_kernel(lambda: sd.probe_mfma_bf16(iters_mfma, 1, sink), iters=5, warm=1)
    ceilings = {"read_gbs": buf.numel() / t_rd / 1e6, "copy_gbs_read_plus_write": 2 * half / t_cp / 1e6,
                "mfma_bf16_tflops_smooth_operands": fl / t_m0 / 1e9, "mfma_bf16_tflops_random_operands": fl / t_m1 / 1e9,
                "note": "plain read / copy kernels over 2 GiB / 1 GiB and a loop of independent "
                        "v_mfma_f32_16x16x32_bf16 (sdllm_probe_*); not part of the timed step"}
    del buf
    dur = attn_ms_ev if use_ev else None
    if bound == "hbm":
        ach = attn_bytes / dur / 1e6 if dur else None
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS if ach else None, "traffic": None}
    else:
        ach = attn_flops / dur / 1e9 if dur else None
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS if ach else None, "traffic": None}
    # HBM traffic of the same call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs, scaled by what the
    # counters read for the kv_append copy of known size): read from the committed profile, NOT measured in this run
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            prof = json.load(f)
        tr = prof["workloads"].get(w.name)
        if tr is not None:
            roof["traffic"] = tr["attention_call_bytes"]
            roof["traffic_unit"] = "bytes per launch (read + write, main kernel + split merge)"
            roof["traffic_source"] = ("profiles/hbm_traffic.json (rocprofv3 --pmc runs of this bench, "
                                      f"{prof.get('measured_with', 'kernels as committed with the file')}); "
                                      "not measured in this run")
    except (OSError, KeyError, ValueError):
        pass
    roof["measured_ceiling"] = ceilings["read_gbs"] if bound == "hbm" else ceilings["mfma_bf16_tflops_random_operands"]
    roof["frac_of_measured_ceiling"] = (roof["achieved"] / roof["measured_ceiling"]) if roof["achieved"] else None
    roof.update({"kernel": "sdllm_block_attention, one layer (attn_bf16_kernel + attn_combine_kernel)" if w.dtype == "bf16"
                 else "sdllm_block_attention (attention_f32_kernel)",
                 "launch_ms": dur, "algorithmic_bytes": attn_bytes, "algorithmic_flops": attn_flops,
                 "frac_mfma_peak": (attn_flops / dur / 1e9 / MFMA_BF16_PEAK_TFLOPS) if dur and w.dtype == "bf16" else None,
                 "layer0_launch_ms": layer0_ms_ev,
                 "events": ((f"HIP events before the first and after the last attention call of {len(evs)} of {K} timed "
                             f"steps, divided by the {w.n_layers} layers") if w.n_layers > 1 else
                            f"HIP events around the attention call of {len(evs)} of {K} timed steps") if use_ev else None})
    # the other two calls of the step, each bracketed by HIP events inside the timed region (same steps)
    elems = masked_rows * w.V
    # plain-ALU roof of the row reduction: vector-ALU issue slots per logit (a wave-wide instruction occupies its
    # SIMD for 4 cycles; v_exp_f32 is counted at the 2.4 slots it measures against an FMA on this chip) over
    # 256 CUs x 4 SIMDs at 2.4 GHz
    slots = UNMASK_VALU_SLOTS_PER_ELEMENT[w.dtype]
    alu_ms = elems * slots / 64.0 * 4.0 / (256 * 4 * 2.4e9) * 1e3
    others = []
    if unmask_ms_ev:
        g = unmask_bytes / unmask_ms_ev / 1e6
        others.append({"kernel": "sdllm_confidence_unmask (unmask_rows_kernel + unmask_commit_kernel)", "bound": "hbm",
                       "achieved": g, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": g / HBM_PEAK_GBS,
                       "launch_ms": unmask_ms_ev, "algorithmic_bytes": unmask_bytes, "masked_rows": masked_rows,
                       "alu_roof": {"valu_slots_per_logit": slots, "logits": elems, "roof_ms": alu_ms,
                                    "frac_of_alu_roof": alu_ms / unmask_ms_ev}})
    if append_ms_ev:
        g = append_bytes / append_ms_ev / 1e6
        others.append({"kernel": "sdllm_kv_append (kv_append_kernel, all layers, K and V)", "bound": "hbm",
                       "achieved": g, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": g / HBM_PEAK_GBS,
                       "launch_ms": append_ms_ev, "algorithmic_bytes": append_bytes})
    roof["others"] = others

    out = {
        "metric": "committed tokens/sec per decode step", "value": value, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} Hq/Hkv={w.Hq}/{w.Hkv} D={w.D} P={w.P} K={w.K} S={w.S} kept={w.n_keep} "
                               f"V={w.V} layers={w.n_layers} tau0={w.tau0} alpha={w.alpha}",
                   "committed_tokens_per_step": committed_per_step, "seed": args.seed,
                   "launch": "one captured HIP graph per step (state restore + every call)" if args.graph
                   else "eager, pre-marshalled C-ABI calls",
                   "prewarm_ms": args.prewarm_ms},
        "roofline": roof,
        "kernels": kernels,
        "device_ceilings": ceilings,
    }
    if not args.no_cpu_baseline:
        cb = cpu_baseline(w, args.seed)
        # committed tokens per step are the same on both sides (checked by the parity tests)
        ex = cb["exclusions"]
        # the first timed step's state against the oracle on the sampled sequences (positions in the threshold band
        # excluded, as the parity rule says)
        b_u, keep = ex["sequences_checked"], ~ex.pop("band")
        slot = 0 if args.graph else W
        got_t, got_m = st.tokens[slot, :b_u].cpu().numpy(), st.masked[slot, :b_u].cpu().numpy()
        ex["gpu_matches_oracle_outside_band"] = bool((got_t[keep] == ex.pop("oracle_tokens")[keep]).all()
                                                     and (got_m[keep] == ex.pop("oracle_masked")[keep]).all())
        out["exclusions"] = ex
        out["cpu_baseline"] = {"value": committed_per_step / cb["t_step_s"], "unit": "tokens/s", "cores": cb["cores"],
                               "kind": "oracle", "sample": cb["sample"], "step_seconds": cb["t_step_s"],
                               "attention_s": cb["t_attention_s"], "unmask_s": cb["t_unmask_s"], "append_s": cb["t_append_s"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
