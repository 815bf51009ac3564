"""Seeded synthetic inputs for one block-wise diffusion decode step.

This module only *draws and rounds numbers*: it holds no attention, softmax,
threshold or commit arithmetic.  Both the CPU oracle's tests and the HIP path's
tests / bench take their inputs from here, so that the two sides see identical
bits.  The tensors stand in for the *shapes* of the 7-8B diffusion-LLM workloads
the paper evaluates (heads, head_dim, vocabulary, prompt / generation / block
lengths, threshold tau0 = 0.9, alpha 0.1..0.7, block 32 -- paper Table 12); no
benchmark item or trained weight is involved.

Notation (paper section 3.1 / 3.3): B batch, Hq / Hkv query / KV heads, D head
dim, P prefix length (prompt + committed blocks), K block length, S full suffix
length, s = n_keep kept suffix rows, V vocabulary.

Layouts (row-major, last dim contiguous):
  q_block  [B,Hq,K,D]   q_suffix [B,Hq,S,D]
  k_cache / v_cache [B,Hkv,cap,D]  (rows 0..P-1 valid)
  k_block / v_block [B,Hkv,K,D]    k_suffix / v_suffix [B,Hkv,S,D]
  keep_idx [s] int32, strictly increasing, values in [0,S)
  logits [B,K,ld] (first V of each row valid), tokens [B,K] int32, masked [B,K] uint8
  hidden [B,K,Hd] final hidden states, lm_weight [V,Hd] vocabulary projection (Hd = Hq*D)

bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even from
fp32, done once here); `to_f64` widens either dtype exactly to float64.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, Optional

import numpy as np

MASK_TOKEN = -1  # placeholder id stored in `tokens` at masked positions


# --------------------------------------------------------------------------
# dtype helpers (data preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (nearest even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(x: np.ndarray) -> np.ndarray:
    """Exact widening of a generated tensor (bf16 bits or fp32) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def _rng(seed: int, name: str, layer: int = 0) -> np.random.Generator:
    """One independent Philox stream per (seed, tensor name, layer)."""
    tag = zlib.crc32(name.encode()) & 0xFFFFFFFF
    return np.random.Generator(np.random.Philox(key=[(seed << 32) | tag, layer]))


def _normal(seed, name, layer, shape, std, dtype):
    g = _rng(seed, name, layer)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "fp32" | "bf16"
    B: int
    Hq: int
    Hkv: int
    D: int
    prompt: int
    gen: int
    K: int                # block length
    active_block: int     # 0-based index of the block being decoded
    n_keep: int           # kept suffix rows (s)
    keep_rule: str        # "first" | "window+last" | "all"
    V: int
    qkv_std: float
    logit_std: float
    boost: bool           # one boosted logit per row, U(18,26)
    masked_rule: str      # "half" | "all" | "fraction"
    tau0: float
    alpha: float
    n_layers: int = 1

    @property
    def P(self) -> int:
        return self.prompt + self.active_block * self.K

    @property
    def S(self) -> int:
        return self.gen - (self.active_block + 1) * self.K

    @property
    def cap(self) -> int:
        return self.prompt + self.gen

    @property
    def Nq(self) -> int:
        return self.K + self.n_keep

    @property
    def Nkv(self) -> int:
        return self.P + self.K + self.n_keep

    @property
    def Hd(self) -> int:
        """Model width (Hq * D): 4096 for the LLaDA-8B-shaped workloads, 3584 for the Dream-7B-shaped one."""
        return self.Hq * self.D

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def attn_flops(self) -> int:
        """4*B*Hq*Nq*Nkv*D per layer (QK^T and PV, 2 flop per multiply-add)."""
        return 4 * self.B * self.Hq * self.Nq * self.Nkv * self.D

    def attn_bytes(self) -> int:
        """Algorithmic HBM bytes of one attention layer: every K and V row of every
        KV head once, the gathered Q rows once, the output once."""
        kv = 2 * self.B * self.Hkv * self.Nkv * self.D * self.elem_bytes
        qo = 2 * self.B * self.Hq * self.Nq * self.D * self.elem_bytes
        return kv + qo


WORKLOADS: Dict[str, Workload] = {
    # tiny single-layer step, fp32
    "cfg1": Workload("cfg1", "fp32", 1, 4, 4, 64, 64, 256, 32, 0, 16, "first", 2048,
                     1.0, 3.0, False, "half", 0.9, 0.0),
    # LLaDA-8B-shaped layer step (0-based block 3 of 8: P = 608, S = 128)
    "cfg2": Workload("cfg2", "bf16", 1, 32, 32, 128, 512, 256, 32, 3, 32, "window+last", 126464,
                     1.0 / float(np.sqrt(128.0)), 4.0, True, "half", 0.9, 0.3),
    # suffix-pruning ablation pair: A keeps 32 of 992, B keeps all 992
    "cfg3A": Workload("cfg3A", "bf16", 8, 32, 32, 128, 1024, 1024, 32, 0, 32, "window+last", 126464,
                      1.0, 4.0, False, "all", 0.9, 0.0),
    "cfg3B": Workload("cfg3B", "bf16", 8, 32, 32, 128, 1024, 1024, 32, 0, 992, "all", 126464,
                      1.0, 4.0, False, "all", 0.9, 0.0),
    # Dream-7B-shaped GQA step
    "cfg4": Workload("cfg4", "bf16", 16, 28, 4, 128, 256, 512, 32, 8, 32, "window+last", 152064,
                     1.0, 4.0, False, "fraction", 0.9, 0.3),
    # same shapes with boosted rows, so block_done varies across the batch
    "cfg4boost": Workload("cfg4boost", "bf16", 16, 28, 4, 128, 256, 512, 32, 8, 32, "window+last", 152064,
                          1.0, 4.0, True, "fraction", 0.9, 0.3),
    # long-context 32-layer stack
    "cfg5": Workload("cfg5", "bf16", 4, 32, 32, 128, 4096, 2048, 64, 16, 64, "window+last", 126464,
                     1.0, 4.0, False, "all", 0.9, 0.3, n_layers=32),
    # block-causal (next-block) topology of the paper's extension section: the active block is the last
    # visible one, so there is no suffix at all (S = 0, nothing kept) and only the temporal rule applies;
    # GQA 32/8, last block of a 256-token generation after a 1024-token prompt
    "cfgBC": Workload("cfgBC", "bf16", 8, 32, 8, 128, 1024, 256, 32, 7, 0, "first", 152064,
                      1.0, 4.0, True, "half", 0.9, 0.3),
    # small bf16 case the oracle finishes instantly; spans several 32-key tiles and a ragged tail
    "small_bf16": Workload("small_bf16", "bf16", 2, 4, 2, 128, 75, 160, 32, 1, 33, "window+last", 5000,
                           1.0, 4.0, True, "half", 0.9, 0.3),
}


def make_keep_idx(w: Workload) -> np.ndarray:
    """Index list of kept suffix rows (an *input* of the hot path)."""
    S, s = w.S, w.n_keep
    if s == 0:
        return np.zeros((0,), dtype=np.int32)
    if w.keep_rule == "first":
        idx = np.arange(s)
    elif w.keep_rule == "all":
        assert s == S
        idx = np.arange(S)
    elif w.keep_rule == "window+last":
        # nearest s-1 suffix positions plus the trailing position (paper Eq. 7 / Fig. 4)
        idx = np.concatenate([np.arange(min(s - 1, S - 1)), [S - 1]])
    else:
        raise ValueError(w.keep_rule)
    idx = np.unique(idx).astype(np.int32)
    assert idx.shape[0] == s, (idx.shape, s)
    return idx


def make_attention_inputs(w: Workload, seed: int = 0, layer: int = 0) -> Dict[str, np.ndarray]:
    B, Hq, Hkv, D, K, S, P, cap = w.B, w.Hq, w.Hkv, w.D, w.K, w.S, w.P, w.cap
    sd, dt = w.qkv_std, w.dtype
    out = {
        "q_block": _normal(seed, "q_block", layer, (B, Hq, K, D), sd, dt),
        "q_suffix": _normal(seed, "q_suffix", layer, (B, Hq, S, D), sd, dt),
        "k_cache": _normal(seed, "k_cache", layer, (B, Hkv, cap, D), sd, dt),
        "v_cache": _normal(seed, "v_cache", layer, (B, Hkv, cap, D), sd, dt),
        "k_block": _normal(seed, "k_block", layer, (B, Hkv, K, D), sd, dt),
        "v_block": _normal(seed, "v_block", layer, (B, Hkv, K, D), sd, dt),
        "k_suffix": _normal(seed, "k_suffix", layer, (B, Hkv, S, D), sd, dt),
        "v_suffix": _normal(seed, "v_suffix", layer, (B, Hkv, S, D), sd, dt),
        "keep_idx": make_keep_idx(w),
    }
    return out


def make_custom_attention_inputs(dtype: str, B: int, Hq: int, Hkv: int, D: int, P: int, cap: int, K: int,
                                 S: int, keep_idx, seed: int = 0, std: float = 1.0) -> Dict[str, np.ndarray]:
    """Free-form shapes for edge-case tests (ragged tails, empty suffix, ...)."""
    keep_idx = np.asarray(keep_idx, dtype=np.int32).reshape(-1)
    out = {
        "q_block": _normal(seed, "q_block", 0, (B, Hq, K, D), std, dtype),
        "q_suffix": _normal(seed, "q_suffix", 0, (B, Hq, S, D), std, dtype),
        "k_cache": _normal(seed, "k_cache", 0, (B, Hkv, cap, D), std, dtype),
        "v_cache": _normal(seed, "v_cache", 0, (B, Hkv, cap, D), std, dtype),
        "k_block": _normal(seed, "k_block", 0, (B, Hkv, K, D), std, dtype),
        "v_block": _normal(seed, "v_block", 0, (B, Hkv, K, D), std, dtype),
        "k_suffix": _normal(seed, "k_suffix", 0, (B, Hkv, S, D), std, dtype),
        "v_suffix": _normal(seed, "v_suffix", 0, (B, Hkv, S, D), std, dtype),
        "keep_idx": keep_idx,
    }
    return out


def make_masked(w: Workload, seed: int = 0, B: Optional[int] = None, K: Optional[int] = None,
                rule: Optional[str] = None) -> np.ndarray:
    B = w.B if B is None else B
    K = w.K if K is None else K
    rule = w.masked_rule if rule is None else rule
    g = _rng(seed, "masked", 0)
    masked = np.zeros((B, K), dtype=np.uint8)
    for b in range(B):
        if rule == "all":
            m = K
        elif rule == "half":
            m = K // 2
        elif rule == "fraction":
            f = g.uniform(0.1, 1.0)
            m = max(1, int(np.floor(K * f)))
        else:
            raise ValueError(rule)
        pos = g.permutation(K)[:m]
        masked[b, pos] = 1
    return masked


def make_logits(dtype: str, B: int, K: int, V: int, std: float, boost: bool, seed: int = 0,
                ld: Optional[int] = None, step: int = 0) -> np.ndarray:
    """[B,K,ld] logits ~ N(0, std^2); with `boost`, one seeded random token per row is
    overwritten with u ~ U(18, 26) so that max-probabilities straddle the threshold."""
    ld = V if ld is None else ld
    assert ld >= V
    g = _rng(seed, "logits", step)
    x = g.standard_normal(size=(B, K, ld), dtype=np.float32)
    x *= np.float32(std)
    if boost:
        gb = _rng(seed, "boost", step)
        tok = gb.integers(0, V, size=(B, K))
        val = gb.uniform(18.0, 26.0, size=(B, K)).astype(np.float32)
        bi, ki = np.meshgrid(np.arange(B), np.arange(K), indexing="ij")
        x[bi, ki, tok] = val
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x


def make_unmask_inputs(w: Workload, seed: int = 0, step: int = 0, ld: Optional[int] = None) -> Dict[str, np.ndarray]:
    masked = make_masked(w, seed)
    g = _rng(seed, "tokens", 0)
    tokens = g.integers(0, w.V, size=(w.B, w.K)).astype(np.int32)
    tokens[masked != 0] = MASK_TOKEN
    return {
        "logits": make_logits(w.dtype, w.B, w.K, w.V, w.logit_std, w.boost, seed, ld, step),
        "tokens": tokens,
        "masked": masked,
        "eos_seen": np.zeros((w.B,), dtype=np.uint8),
    }


def make_lm_head_inputs(w: Workload, seed: int = 0, step: int = 0, V: Optional[int] = None,
                        Hd: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Final hidden states [B,K,Hd] ~ N(0,1) and a vocabulary projection [V,Hd] ~ N(0, (logit_std/sqrt(Hd))^2),
    so that a logit (a dot product over Hd) follows the N(0, logit_std^2) law of make_logits.  With `boost`,
    one seeded random token per row is made to stand out with a logit of u ~ U(18, 26): its projection row
    is replaced by u * h / |h|^2, h being that row's hidden state (the other rows see ~u/sqrt(Hd) there)."""
    V = w.V if V is None else V
    Hd = w.Hd if Hd is None else Hd
    g = _rng(seed, "hidden", step)
    h = g.standard_normal(size=(w.B, w.K, Hd), dtype=np.float32)
    hb = f32_to_bf16_bits(h)
    gw = _rng(seed, "lm_weight", 0)
    W = gw.standard_normal(size=(V, Hd), dtype=np.float32)
    W *= np.float32(w.logit_std / np.sqrt(Hd))
    if w.boost:
        gb = _rng(seed, "boost", step)
        tok = gb.integers(0, V, size=(w.B, w.K))
        val = gb.uniform(18.0, 26.0, size=(w.B, w.K)).astype(np.float32)
        hr = bf16_bits_to_f32(hb)
        for b in range(w.B):
            for k in range(w.K):
                W[tok[b, k]] = val[b, k] * hr[b, k] / np.float32(np.dot(hr[b, k], hr[b, k]))
    masked = make_masked(w, seed)
    gt = _rng(seed, "tokens", 0)
    tokens = gt.integers(0, V, size=(w.B, w.K)).astype(np.int32)
    tokens[masked != 0] = MASK_TOKEN
    return {"hidden": hb, "lm_weight": f32_to_bf16_bits(W), "tokens": tokens, "masked": masked,
            "eos_seen": np.zeros((w.B,), dtype=np.uint8)}


def make_lm_head_inputs_device(w: Workload, seed: int = 0, device: str = "cuda"):
    """Device-side draw of make_lm_head_inputs' tensors for the full-size projection (V x Hd ~ 0.5e9
    elements); same laws, torch's seeded device generator.  Returns bf16 tensors `hidden`, `lm_weight`
    and the host-drawn `tokens` / `masked` state; parity checks copy them back for the oracle."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed << 16) + 0x1ead)
    h = torch.randn((w.B, w.K, w.Hd), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    W = torch.empty((w.V, w.Hd), device=device, dtype=torch.bfloat16)
    rows = 16384
    for v0 in range(0, w.V, rows):                     # fp32 draws in slices: bounded temporary
        n = min(rows, w.V - v0)
        x = torch.randn((n, w.Hd), generator=g, device=device, dtype=torch.float32)
        W[v0:v0 + n] = (x * (w.logit_std / float(np.sqrt(w.Hd)))).to(torch.bfloat16)
    if w.boost:
        gb = _rng(seed, "boost", 0)
        tok = torch.from_numpy(gb.integers(0, w.V, size=(w.B, w.K))).to(device)
        val = torch.from_numpy(gb.uniform(18.0, 26.0, size=(w.B, w.K)).astype(np.float32)).to(device)
        hf = h.float()
        add = val[..., None] * hf / (hf * hf).sum(-1, keepdim=True)
        for b in range(w.B):
            for k in range(w.K):
                W[tok[b, k]] = add[b, k].to(torch.bfloat16)
    masked = make_masked(w, seed)
    gt = _rng(seed, "tokens", 0)
    tokens = gt.integers(0, w.V, size=(w.B, w.K)).astype(np.int32)
    tokens[masked != 0] = MASK_TOKEN
    return {"hidden": h, "lm_weight": W, "tokens": tokens, "masked": masked,
            "eos_seen": np.zeros((w.B,), dtype=np.uint8)}


def make_append_inputs(dtype: str, n_layers: int, B: int, Hkv: int, D: int, K: int, cap: int,
                       seed: int = 0) -> Dict[str, np.ndarray]:
    """Caches [L,B,Hkv,cap,D] pre-filled with seeded data (so untouched rows can be
    checked bit-for-bit) and block K/V [L,B,Hkv,K,D]."""
    return {
        "k_caches": _normal(seed, "k_caches", 0, (n_layers, B, Hkv, cap, D), 1.0, dtype),
        "v_caches": _normal(seed, "v_caches", 0, (n_layers, B, Hkv, cap, D), 1.0, dtype),
        "k_blocks": _normal(seed, "k_blocks", 0, (n_layers, B, Hkv, K, D), 1.0, dtype),
        "v_blocks": _normal(seed, "v_blocks", 0, (n_layers, B, Hkv, K, D), 1.0, dtype),
    }


def make_attention_inputs_device(w: Workload, seed: int = 0, layer: int = 0, device: str = "cuda"):
    """Device-side generation for workloads too large to draw on the host in reasonable time
    (the 32-layer long-context stack: ~11 GB of K/V).  Same shapes and N(0, qkv_std^2) law as
    make_attention_inputs, drawn with torch's seeded device generator (seed + layer); parity
    checks copy the needed slices back so that the oracle sees identical bits."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed << 16) + layer)
    dt = torch.float32 if w.dtype == "fp32" else torch.bfloat16
    B, Hq, Hkv, D, K, S, cap = w.B, w.Hq, w.Hkv, w.D, w.K, w.S, w.cap

    def draw(*shape):
        x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        if w.qkv_std != 1.0:
            x *= w.qkv_std
        return x.to(dt)

    return {
        "q_block": draw(B, Hq, K, D), "q_suffix": draw(B, Hq, S, D),
        "k_cache": draw(B, Hkv, cap, D), "v_cache": draw(B, Hkv, cap, D),
        "k_block": draw(B, Hkv, K, D), "v_block": draw(B, Hkv, K, D),
        "k_suffix": draw(B, Hkv, S, D), "v_suffix": draw(B, Hkv, S, D),
        "keep_idx": torch.from_numpy(make_keep_idx(w)).to(device),
    }
