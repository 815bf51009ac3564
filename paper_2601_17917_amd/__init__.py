"""Thin Python binding of the sdllm C ABI (include/sdllm.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels of
libsdllm.so.  PyTorch tensors provide device memory and the stream.  There is no CPU
fallback: if the library has not been built, `load_library` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdllm.so")

SDLLM_OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4
FP32, BF16 = 0, 1

EXPORTED_SYMBOLS = (
    "sdllm_block_attention", "sdllm_attention_workspace_bytes", "sdllm_plan_attention",
    "sdllm_confidence_unmask", "sdllm_unmask_workspace_bytes",
    "sdllm_lm_head_unmask", "sdllm_lm_head_unmask_workspace_bytes", "sdllm_plan_lm_head",
    "sdllm_lm_head_pack_weight", "sdllm_lm_head_packed_weight_bytes",
    "sdllm_kv_append", "sdllm_suffix_keep_indices", "sdllm_rope_gathered",
    "sdllm_probe_read", "sdllm_probe_copy", "sdllm_probe_mfma_bf16",
    "sdllm_status_string", "sdllm_last_error", "sdllm_version", "sdllm_init", "sdllm_validate_keep_idx",
    "sdllm_confidence_unmask_noalloc",
)


class AttnParams(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("prefix_len", ctypes.c_int32), ("prefix_cap", ctypes.c_int32),
                ("K", ctypes.c_int32), ("S", ctypes.c_int32), ("n_keep", ctypes.c_int32),
                ("scale", ctypes.c_float), ("kv_splits", ctypes.c_int32)]


class UnmaskParams(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("K", ctypes.c_int32), ("V", ctypes.c_int32),
                ("ld", ctypes.c_int64), ("tau0", ctypes.c_float), ("alpha", ctypes.c_float),
                ("r_extra_masked", ctypes.c_int32), ("r_extra_total", ctypes.c_int32),
                ("eos_id", ctypes.c_int32), ("tau_eos", ctypes.c_float)]


class LmHeadParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("K", ctypes.c_int32), ("V", ctypes.c_int32), ("Hd", ctypes.c_int32),
                ("ld_h", ctypes.c_int64), ("ld_w", ctypes.c_int64), ("tau0", ctypes.c_float), ("alpha", ctypes.c_float),
                ("r_extra_masked", ctypes.c_int32), ("r_extra_total", ctypes.c_int32),
                ("eos_id", ctypes.c_int32), ("tau_eos", ctypes.c_float), ("weight_packed", ctypes.c_int32)]


class LmHeadPlan(ctypes.Structure):
    _fields_ = [("rows_per_chunk", ctypes.c_int32), ("vocab_rows_per_tile", ctypes.c_int32),
                ("vocab_tiles", ctypes.c_int32), ("row_chunks", ctypes.c_int32), ("workgroups", ctypes.c_int32),
                ("lds_bytes", ctypes.c_int32), ("triples_per_position", ctypes.c_int32)]


class AppendParams(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("B", ctypes.c_int32),
                ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32), ("K", ctypes.c_int32),
                ("prefix_len", ctypes.c_int32), ("prefix_cap", ctypes.c_int32),
                ("cache_layer_stride", ctypes.c_int64), ("block_layer_stride", ctypes.c_int64)]


class RopeParams(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
                ("K", ctypes.c_int32), ("S", ctypes.c_int32), ("n_keep", ctypes.c_int32),
                ("pos0", ctypes.c_int32), ("theta_base", ctypes.c_float), ("interleaved", ctypes.c_int32)]


class AttnPlan(ctypes.Structure):
    _fields_ = [("kv_splits", ctypes.c_int32), ("rows_per_workgroup", ctypes.c_int32),
                ("workgroups", ctypes.c_int32), ("key_tiles_per_split", ctypes.c_int32),
                ("workgroup_shape", ctypes.c_int32), ("ring_stages", ctypes.c_int32)]


class SdllmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"sdllm status {status}: {text}")
        self.status = status


_lib = None


def load_library(path: Optional[str] = None):
    """Load libsdllm.so (once).  Raises if it has not been built -- there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch brings its own copy of the HIP runtime: it has to be the one already in the process when
    # libsdllm.so resolves its runtime symbols, or kernels are launched through a second, uninitialised copy
    import torch  # noqa: F401
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2601_17917_amd.build`")
    lib = ctypes.CDLL(path)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.sdllm_version.restype = i32
    lib.sdllm_init.restype = i32
    lib.sdllm_init.argtypes = []
    lib.sdllm_validate_keep_idx.restype = i32
    lib.sdllm_validate_keep_idx.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp]
    lib.sdllm_last_error.restype = ctypes.c_char_p
    lib.sdllm_status_string.restype = ctypes.c_char_p
    lib.sdllm_status_string.argtypes = [i32]
    lib.sdllm_attention_workspace_bytes.restype = sz
    lib.sdllm_attention_workspace_bytes.argtypes = [ctypes.POINTER(AttnParams)]
    lib.sdllm_plan_attention.restype = i32
    lib.sdllm_plan_attention.argtypes = [ctypes.POINTER(AttnParams), ctypes.POINTER(AttnPlan)]
    lib.sdllm_block_attention.restype = i32
    lib.sdllm_block_attention.argtypes = [ctypes.POINTER(AttnParams)] + [vp] * 10 + [vp, sz, vp]
    lib.sdllm_unmask_workspace_bytes.restype = sz
    lib.sdllm_unmask_workspace_bytes.argtypes = [ctypes.POINTER(UnmaskParams)]
    lib.sdllm_confidence_unmask.restype = i32
    lib.sdllm_confidence_unmask.argtypes = [ctypes.POINTER(UnmaskParams)] + [vp] * 7 + [vp, sz, vp]
    lib.sdllm_confidence_unmask_noalloc.restype = i32
    lib.sdllm_confidence_unmask_noalloc.argtypes = [ctypes.POINTER(UnmaskParams)] + [vp] * 7 + [vp]
    lib.sdllm_lm_head_unmask_workspace_bytes.restype = sz
    lib.sdllm_lm_head_unmask_workspace_bytes.argtypes = [ctypes.POINTER(LmHeadParams)]
    lib.sdllm_plan_lm_head.restype = i32
    lib.sdllm_plan_lm_head.argtypes = [ctypes.POINTER(LmHeadParams), ctypes.POINTER(LmHeadPlan)]
    lib.sdllm_lm_head_unmask.restype = i32
    lib.sdllm_lm_head_unmask.argtypes = [ctypes.POINTER(LmHeadParams)] + [vp] * 8 + [vp, sz, vp]
    lib.sdllm_lm_head_packed_weight_bytes.restype = sz
    lib.sdllm_lm_head_packed_weight_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.sdllm_lm_head_pack_weight.restype = i32
    lib.sdllm_lm_head_pack_weight.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, vp, vp, vp]
    lib.sdllm_suffix_keep_indices.restype = i32
    lib.sdllm_suffix_keep_indices.argtypes = [ctypes.c_int32] * 4 + [ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                                                    ctypes.POINTER(ctypes.c_int32)]
    lib.sdllm_kv_append.restype = i32
    lib.sdllm_kv_append.argtypes = [ctypes.POINTER(AppendParams)] + [vp] * 5 + [vp]
    lib.sdllm_rope_gathered.restype = i32
    lib.sdllm_rope_gathered.argtypes = [ctypes.POINTER(RopeParams)] + [vp] * 5 + [vp]
    lib.sdllm_probe_read.restype = i32
    lib.sdllm_probe_read.argtypes = [vp, sz, vp, vp]
    lib.sdllm_probe_copy.restype = i32
    lib.sdllm_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.sdllm_probe_mfma_bf16.restype = i32
    lib.sdllm_probe_mfma_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    _lib = lib
    return lib


def _check(status: int):
    if status != SDLLM_OK:
        raise SdllmError(status, load_library().sdllm_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return FP32
    if t.dtype == torch.bfloat16:
        return BF16
    raise SdllmError(ERR_UNSUPPORTED, f"dtype {t.dtype} not supported (float32, bfloat16)")


def _require(t, name, dtype=None):
    if t is None:
        return
    if not t.is_cuda:
        raise SdllmError(ERR_INVALID_ARG, f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise SdllmError(ERR_INVALID_ARG, f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise SdllmError(ERR_INVALID_ARG, f"{name} must have dtype {dtype}, has {t.dtype}")


def init():
    """sdllm_init on the current device: every kernel opt-in done, so that later calls only launch."""
    _check(load_library().sdllm_init())


def validate_keep_idx(keep_idx, S: int, stream=None):
    """sdllm_validate_keep_idx (debug; synchronises): raises SdllmError unless keep_idx is strictly increasing
    within [0, S)."""
    import torch
    _require(keep_idx, "keep_idx", torch.int32)
    n = 0 if keep_idx is None else int(keep_idx.shape[0])
    _check(load_library().sdllm_validate_keep_idx(_ptr(keep_idx), n, S, _stream(stream)))


# ---------------------------------------------------------------------------------------------
def attn_params(dtype, B, Hq, Hkv, D, prefix_len, prefix_cap, K, S, n_keep, scale=0.0, kv_splits=0) -> AttnParams:
    return AttnParams(dtype, B, Hq, Hkv, D, prefix_len, prefix_cap, K, S, n_keep, scale, kv_splits)


def attention_workspace_bytes(p: AttnParams) -> int:
    n = load_library().sdllm_attention_workspace_bytes(ctypes.byref(p))
    if n == ctypes.c_size_t(-1).value:
        raise SdllmError(ERR_INVALID_ARG, load_library().sdllm_last_error().decode())
    return n


def plan_attention(p: AttnParams) -> AttnPlan:
    plan = AttnPlan()
    _check(load_library().sdllm_plan_attention(ctypes.byref(p), ctypes.byref(plan)))
    return plan


class BoundCall:
    """One C-ABI call with its arguments marshalled once; calling it enqueues the work again on the
    stream it was bound to.  Keeps the tensors alive.  For tight loops where per-call Python
    marshalling would cost more than the kernels."""

    __slots__ = ("_fn", "_args", "_keep", "result")

    def __init__(self, fn, args, keep, result):
        self._fn, self._args, self._keep, self.result = fn, args, keep, result

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != SDLLM_OK:
            _check(rc)
        return self.result


def block_attention(*args, **kw):
    """sdllm_block_attention.  Tensors in [B,H,T,D] layout; returns out [B,Hq,K+n_keep,D].
    The cache tensors may be None when prefix_len == 0, the suffix tensors when keep_idx is empty.
    Signature: see bind_block_attention."""
    return bind_block_attention(*args, **kw)()


def bind_block_attention(q_block, q_suffix, k_cache, v_cache, k_block, v_block, k_suffix, v_suffix, keep_idx,
                         prefix_len: int, out=None, scale: float = 0.0, kv_splits: int = 0, workspace=None,
                         stream=None) -> BoundCall:
    import torch
    B, Hq, K, D = q_block.shape
    Hkv = k_block.shape[1]
    S = 0 if q_suffix is None else q_suffix.shape[2]
    n_keep = 0 if keep_idx is None else int(keep_idx.shape[0])
    cap = prefix_len if k_cache is None else k_cache.shape[2]
    for name, t in (("q_block", q_block), ("q_suffix", q_suffix), ("k_cache", k_cache), ("v_cache", v_cache),
                    ("k_block", k_block), ("v_block", v_block), ("k_suffix", k_suffix), ("v_suffix", v_suffix)):
        _require(t, name, q_block.dtype)
    _require(keep_idx, "keep_idx", torch.int32)
    p = attn_params(_dtype_code(q_block), B, Hq, Hkv, D, prefix_len, cap, K, S, n_keep, scale, kv_splits)
    if out is None:
        out = torch.empty((B, Hq, K + n_keep, D), dtype=q_block.dtype, device=q_block.device)
    _require(out, "out", q_block.dtype)
    need = attention_workspace_bytes(p)
    if need and workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=q_block.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    kidx = keep_idx if n_keep else None
    args = (ctypes.byref(p), _ptr(q_block), _ptr(q_suffix), _ptr(k_cache), _ptr(v_cache), _ptr(k_block), _ptr(v_block),
            _ptr(k_suffix), _ptr(v_suffix), _ptr(kidx), _ptr(out), _ptr(workspace), ws_bytes, _stream(stream))
    keep = (p, q_block, q_suffix, k_cache, v_cache, k_block, v_block, k_suffix, v_suffix, kidx, out, workspace)
    return BoundCall(load_library().sdllm_block_attention, args, keep, out)


# ---------------------------------------------------------------------------------------------
def unmask_params(dtype, B, K, V, ld, tau0, alpha, r_extra_masked=0, r_extra_total=0, eos_id=-1,
                  tau_eos=None) -> UnmaskParams:
    return UnmaskParams(dtype, B, K, V, ld, tau0, alpha, r_extra_masked, r_extra_total, eos_id,
                        tau0 if tau_eos is None else tau_eos)


def unmask_workspace_bytes(p: UnmaskParams) -> int:
    n = load_library().sdllm_unmask_workspace_bytes(ctypes.byref(p))
    if n == ctypes.c_size_t(-1).value:
        raise SdllmError(ERR_INVALID_ARG, load_library().sdllm_last_error().decode())
    return n


def confidence_unmask(*args, **kw):
    """sdllm_confidence_unmask.  logits [B,K,ld]; tokens int32 [B,K] and masked uint8 [B,K] are updated
    in place.  Returns (n_committed int32 [B], block_done uint8 [B]).  Signature: see bind_confidence_unmask."""
    return bind_confidence_unmask(*args, **kw)()


def bind_confidence_unmask(logits, tokens, masked, tau0: float, alpha: float, V: Optional[int] = None,
                           confidence=None, n_committed=None, block_done=None, eos_seen=None, eos_id: int = -1,
                           tau_eos: Optional[float] = None, r_extra_masked: int = 0, r_extra_total: int = 0,
                           workspace=None, stream=None) -> BoundCall:
    import torch
    B, K, ld = logits.shape
    V = ld if V is None else V
    _require(logits, "logits")
    _require(tokens, "tokens", torch.int32)
    _require(masked, "masked", torch.uint8)
    _require(confidence, "confidence", torch.float32)
    _require(eos_seen, "eos_seen", torch.uint8)
    if n_committed is None:
        n_committed = torch.empty((B,), dtype=torch.int32, device=logits.device)
    if block_done is None:
        block_done = torch.empty((B,), dtype=torch.uint8, device=logits.device)
    _require(n_committed, "n_committed", torch.int32)
    _require(block_done, "block_done", torch.uint8)
    p = unmask_params(_dtype_code(logits), B, K, V, ld, tau0, alpha, r_extra_masked, r_extra_total, eos_id, tau_eos)
    need = unmask_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=logits.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    args = (ctypes.byref(p), _ptr(logits), _ptr(tokens), _ptr(masked), _ptr(confidence), _ptr(n_committed),
            _ptr(block_done), _ptr(eos_seen), _ptr(workspace), ws_bytes, _stream(stream))
    keep = (p, logits, tokens, masked, confidence, n_committed, block_done, eos_seen, workspace)
    return BoundCall(load_library().sdllm_confidence_unmask, args, keep, (n_committed, block_done))


NOALLOC_SCRATCH_BYTES = 1 << 20


def confidence_unmask_noalloc(*args, **kw):
    """sdllm_confidence_unmask_noalloc: same operation and results as confidence_unmask; the partial results live in
    the library's own device-resident scratch (no workspace, nothing allocated by the call when n_committed and
    block_done are passed).  Signature: see bind_confidence_unmask_noalloc."""
    return bind_confidence_unmask_noalloc(*args, **kw)()


def bind_confidence_unmask_noalloc(logits, tokens, masked, tau0: float, alpha: float, V: Optional[int] = None,
                                   confidence=None, n_committed=None, block_done=None, eos_seen=None, eos_id: int = -1,
                                   tau_eos: Optional[float] = None, r_extra_masked: int = 0, r_extra_total: int = 0,
                                   stream=None) -> BoundCall:
    import torch
    B, K, ld = logits.shape
    V = ld if V is None else V
    _require(logits, "logits")
    _require(tokens, "tokens", torch.int32)
    _require(masked, "masked", torch.uint8)
    _require(confidence, "confidence", torch.float32)
    _require(eos_seen, "eos_seen", torch.uint8)
    if n_committed is None:
        n_committed = torch.empty((B,), dtype=torch.int32, device=logits.device)
    if block_done is None:
        block_done = torch.empty((B,), dtype=torch.uint8, device=logits.device)
    _require(n_committed, "n_committed", torch.int32)
    _require(block_done, "block_done", torch.uint8)
    p = unmask_params(_dtype_code(logits), B, K, V, ld, tau0, alpha, r_extra_masked, r_extra_total, eos_id, tau_eos)
    args = (ctypes.byref(p), _ptr(logits), _ptr(tokens), _ptr(masked), _ptr(confidence), _ptr(n_committed),
            _ptr(block_done), _ptr(eos_seen), _stream(stream))
    keep = (p, logits, tokens, masked, confidence, n_committed, block_done, eos_seen)
    return BoundCall(load_library().sdllm_confidence_unmask_noalloc, args, keep, (n_committed, block_done))


# ---------------------------------------------------------------------------------------------
def lm_head_params(B, K, V, Hd, ld_h, ld_w, tau0, alpha, r_extra_masked=0, r_extra_total=0, eos_id=-1,
                   tau_eos=None, weight_packed=0) -> LmHeadParams:
    return LmHeadParams(B, K, V, Hd, ld_h, ld_w, tau0, alpha, r_extra_masked, r_extra_total, eos_id,
                        tau0 if tau_eos is None else tau_eos, weight_packed)


class PackedLmWeight:
    """The image sdllm_lm_head_pack_weight wrote for a projection matrix [V, Hd]: `data` is a flat bf16 device
    tensor; pass the object as `weight` to lm_head_unmask / bind_lm_head_unmask."""

    def __init__(self, data, V: int, Hd: int):
        self.data, self.V, self.Hd = data, V, Hd


def lm_head_packed_weight_bytes(V: int, Hd: int) -> int:
    n = load_library().sdllm_lm_head_packed_weight_bytes(V, Hd)
    if n == ctypes.c_size_t(-1).value:
        raise SdllmError(ERR_INVALID_ARG, "lm_head_packed_weight_bytes: need V >= 1 and Hd a positive multiple of 32")
    return n


def lm_head_pack_weight(weight, stream=None) -> PackedLmWeight:
    """sdllm_lm_head_pack_weight: weight bf16 [V, Hd] (row stride ld_w) -> PackedLmWeight (a new device tensor)."""
    import torch
    if weight.dtype != torch.bfloat16 or not weight.is_cuda or weight.dim() != 2 or weight.stride(1) != 1:
        raise ValueError("lm_head_pack_weight: need a bfloat16 device tensor [V, Hd] with contiguous rows")
    V, Hd = weight.shape
    data = torch.empty((lm_head_packed_weight_bytes(V, Hd) // 2,), dtype=torch.bfloat16, device=weight.device)
    _check(load_library().sdllm_lm_head_pack_weight(V, Hd, weight.stride(0), _ptr(weight), _ptr(data), _stream(stream)))
    return PackedLmWeight(data, V, Hd)


def lm_head_unmask_workspace_bytes(p: LmHeadParams) -> int:
    n = load_library().sdllm_lm_head_unmask_workspace_bytes(ctypes.byref(p))
    if n == ctypes.c_size_t(-1).value:
        raise SdllmError(ERR_INVALID_ARG, load_library().sdllm_last_error().decode())
    return n


def plan_lm_head(p: LmHeadParams) -> LmHeadPlan:
    plan = LmHeadPlan()
    _check(load_library().sdllm_plan_lm_head(ctypes.byref(p), ctypes.byref(plan)))
    return plan


def lm_head_unmask(*args, **kw):
    """sdllm_lm_head_unmask.  hidden bf16 [B,K,Hd] (row stride ld_h), weight bf16 [V,Hd] (row stride ld_w) or
    a PackedLmWeight;
    tokens int32 [B,K] and masked uint8 [B,K] are updated in place.  Returns (n_committed int32 [B],
    block_done uint8 [B]).  Signature: see bind_lm_head_unmask."""
    return bind_lm_head_unmask(*args, **kw)()


def bind_lm_head_unmask(hidden, weight, tokens, masked, tau0: float, alpha: float, confidence=None,
                        n_committed=None, block_done=None, eos_seen=None, eos_id: int = -1,
                        tau_eos: Optional[float] = None, r_extra_masked: int = 0, r_extra_total: int = 0,
                        workspace=None, stream=None) -> BoundCall:
    import torch
    B, K, Hd = hidden.shape
    packed = isinstance(weight, PackedLmWeight)
    if packed:
        V, w_hd, ld_w, weight = weight.V, weight.Hd, weight.Hd, weight.data
    else:
        V, w_hd, ld_w = weight.shape[0], weight.shape[1], weight.stride(0)
        if weight.stride(1) != 1:
            raise ValueError("lm_head_unmask: weight [V,Hd] needs a contiguous last dimension")
    if hidden.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16:
        raise TypeError("lm_head_unmask: hidden and weight must be bfloat16")
    if w_hd != Hd or hidden.stride(2) != 1 or hidden.stride(0) != K * hidden.stride(1):
        raise ValueError("lm_head_unmask: need hidden [B,K,Hd] with contiguous last dimension and a weight of the same Hd")
    if not hidden.is_cuda or not weight.is_cuda:
        raise ValueError("lm_head_unmask: hidden and weight must be device tensors")
    _require(tokens, "tokens", torch.int32)
    _require(masked, "masked", torch.uint8)
    _require(confidence, "confidence", torch.float32)
    _require(eos_seen, "eos_seen", torch.uint8)
    if n_committed is None:
        n_committed = torch.empty((B,), dtype=torch.int32, device=hidden.device)
    if block_done is None:
        block_done = torch.empty((B,), dtype=torch.uint8, device=hidden.device)
    _require(n_committed, "n_committed", torch.int32)
    _require(block_done, "block_done", torch.uint8)
    p = lm_head_params(B, K, V, Hd, hidden.stride(1), ld_w, tau0, alpha, r_extra_masked, r_extra_total,
                       eos_id, tau_eos, 1 if packed else 0)
    need = lm_head_unmask_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=hidden.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    args = (ctypes.byref(p), _ptr(hidden), _ptr(weight), _ptr(tokens), _ptr(masked), _ptr(confidence),
            _ptr(n_committed), _ptr(block_done), _ptr(eos_seen), _ptr(workspace), ws_bytes, _stream(stream))
    keep = (p, hidden, weight, tokens, masked, confidence, n_committed, block_done, eos_seen, workspace)
    return BoundCall(load_library().sdllm_lm_head_unmask, args, keep, (n_committed, block_done))


# ---------------------------------------------------------------------------------------------
def kv_append(*args, **kw):
    """sdllm_kv_append.  caches [L,B,Hkv,cap,D] (updated in place), blocks [L,B,Hkv,K,D].
    Signature: see bind_kv_append."""
    return bind_kv_append(*args, **kw)()


def _require_layers(t, name, dtype):
    """A [L, ...] tensor whose layers are contiguous blocks a constant distance apart (stride(0) may exceed the
    dense size: layers padded or interleaved with other data)."""
    if not t.is_cuda:
        raise SdllmError(ERR_INVALID_ARG, f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise SdllmError(ERR_INVALID_ARG, f"{name} must have dtype {dtype}, has {t.dtype}")
    if not t[0].is_contiguous() or (t.shape[0] > 1 and t.stride(0) < t[0].numel()):
        raise SdllmError(ERR_INVALID_ARG, f"{name}: every layer must be contiguous and layers must not overlap")


def bind_kv_append(k_caches, v_caches, k_blocks, v_blocks, prefix_len: int, do_append=None, stream=None) -> BoundCall:
    import torch
    L, B, Hkv, cap, D = k_caches.shape
    K = k_blocks.shape[3]
    for name, t in (("k_caches", k_caches), ("v_caches", v_caches), ("k_blocks", k_blocks), ("v_blocks", v_blocks)):
        _require_layers(t, name, k_caches.dtype)
    _require(do_append, "do_append", torch.uint8)
    if L > 1 and (v_caches.stride(0) != k_caches.stride(0) or v_blocks.stride(0) != k_blocks.stride(0)):
        raise SdllmError(ERR_INVALID_ARG, "kv_append: K and V tensors must share their layer strides")
    cls = k_caches.stride(0) if L > 1 else 0           # 0 = dense (a single layer has no stride to speak of)
    bls = k_blocks.stride(0) if L > 1 else 0
    p = AppendParams(_dtype_code(k_caches), L, B, Hkv, D, K, prefix_len, cap, cls, bls)
    args = (ctypes.byref(p), _ptr(k_caches), _ptr(v_caches), _ptr(k_blocks), _ptr(v_blocks), _ptr(do_append),
            _stream(stream))
    keep = (p, k_caches, v_caches, k_blocks, v_blocks, do_append)
    return BoundCall(load_library().sdllm_kv_append, args, keep, None)


# ---------------------------------------------------------------------------------------------
def rope_gathered(*args, **kw):
    """sdllm_rope_gathered: see include/sdllm.h.  Returns (out_block, out_suffix)."""
    return bind_rope_gathered(*args, **kw)()


def bind_rope_gathered(x_block, x_suffix, keep_idx, pos0: int, theta_base: float, interleaved: bool = False,
                       out_block=None, out_suffix=None, stream=None) -> BoundCall:
    """Marshal once, call many times.  out_* default to the inputs (in place)."""
    import torch
    B, H, K, D = x_block.shape
    n_keep = 0 if keep_idx is None else int(keep_idx.shape[0])
    S = 0 if x_suffix is None else int(x_suffix.shape[2])
    out_block = x_block if out_block is None else out_block
    out_suffix = x_suffix if out_suffix is None else out_suffix
    for name, t in (("x_block", x_block), ("x_suffix", x_suffix), ("out_block", out_block), ("out_suffix", out_suffix)):
        _require(t, name, x_block.dtype)
    _require(keep_idx, "keep_idx", torch.int32)
    if x_suffix is not None and tuple(x_suffix.shape) != (B, H, S, D):
        raise SdllmError(ERR_INVALID_ARG, "x_suffix must be [B,H,S,D] with the B, H, D of x_block")
    if tuple(out_block.shape) != (B, H, K, D) or (out_suffix is not None and tuple(out_suffix.shape) != (B, H, S, D)):
        raise SdllmError(ERR_INVALID_ARG, "out_block / out_suffix must have the shapes of the inputs")
    p = RopeParams(_dtype_code(x_block), B, H, D, K, S, n_keep, int(pos0), float(theta_base), int(bool(interleaved)))
    args = (ctypes.byref(p), _ptr(x_block), _ptr(x_suffix), _ptr(keep_idx), _ptr(out_block), _ptr(out_suffix),
            _stream(stream))
    keep = (p, x_block, x_suffix, keep_idx, out_block, out_suffix)
    return BoundCall(load_library().sdllm_rope_gathered, args, keep, (out_block, out_suffix))


# ---------------------------------------------------------------------------------------------
def probe_read(src, sink, stream=None):
    """sdllm_probe_read over the whole of `src` (device tensor, byte size a multiple of 16)."""
    _require(src, "src"); _require(sink, "sink")
    _check(load_library().sdllm_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))


def probe_copy(dst, src, stream=None):
    """sdllm_probe_copy: dst <- src (device tensors of the same byte size, a multiple of 16)."""
    _require(src, "src"); _require(dst, "dst")
    if dst.numel() * dst.element_size() != src.numel() * src.element_size():
        raise SdllmError(ERR_INVALID_ARG, "probe_copy: dst and src differ in size")
    _check(load_library().sdllm_probe_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)))


def probe_mfma_bf16(iters: int, operand_kind: int, sink, stream=None) -> float:
    """sdllm_probe_mfma_bf16; returns the floating-point operations of the launch."""
    _require(sink, "sink")
    fl = ctypes.c_double(0.0)
    _check(load_library().sdllm_probe_mfma_bf16(iters, operand_kind, _ptr(sink), _stream(stream), ctypes.byref(fl)))
    return fl.value


def suffix_keep_indices(S: int, K: int, w_blocks: int, keep_trailing: bool = True):
    """sdllm_suffix_keep_indices (host helper, paper Eq. 7).  Returns a Python list of the kept suffix
    positions (relative to the start of the suffix, strictly increasing)."""
    cap = max(min(w_blocks * K, max(S, 0)) + 1, 1)
    buf = (ctypes.c_int32 * cap)()
    n = ctypes.c_int32(0)
    _check(load_library().sdllm_suffix_keep_indices(S, K, w_blocks, 1 if keep_trailing else 0, buf, cap, ctypes.byref(n)))
    return [buf[i] for i in range(n.value)]
