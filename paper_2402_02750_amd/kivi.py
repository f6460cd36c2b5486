"""Thin Python binding of the C ABI in include/kivi.h (argument marshalling only).

Every step of the path runs in the HIP library; PyTorch only provides device memory and the
stream.  There is no CPU fallback: if libkivi_hip.so is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libkivi_hip.so")

KIVI_OK = 0
KIVI_ERR_INVALID_ARG = -1
KIVI_ERR_UNSUPPORTED = -2
KIVI_ERR_WORKSPACE = -3
KIVI_ERR_HIP = -4
KIVI_FLUSH_WINDOW = 0
KIVI_FLUSH_ALG1 = 1
KIVI_DECODE_AUTO = 0
KIVI_DECODE_VALU = 1
KIVI_DECODE_MFMA = 2
KIVI_DECODE_MFMA_ONE = 3
KIVI_DECODE_MFMA_TWO = 4

EXPORTS = [
    "kivi_status_string", "kivi_cache_sizes", "kivi_decode_workspace_bytes", "kivi_decode_plan",
    "kivi_quantize_key_groups", "kivi_quantize_value_tokens", "kivi_prefill", "kivi_append_residual",
    "kivi_flush_residual", "kivi_decode_attention", "kivi_decode_step", "kivi_stream_read_probe",
    "kivi_batch_slice", "kivi_decode_step_ragged", "kivi_decode_attention_ragged",
    "kivi_decode_attention_static", "kivi_decode_launches_ragged",
]
KIVI_STATIC_WORKSPACE_BYTES = 8 << 20


class KiviError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class kivi_layout_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "bits", "group", "residual",
        "cap_q_tokens", "cap_r_tokens", "decode_path")]


class kivi_cache_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid")] + \
        [(n, ctypes.c_int32) for n in ("n_kq", "n_vq", "k_r_start", "n_kr", "v_r_start", "n_vr")]


class kivi_seq_state_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_kq", "n_vq", "k_r_start", "n_kr", "v_r_start", "n_vr")]


class kivi_decode_plan_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("family", "launches", "splits_quantised", "splits_fp16",
                                              "tiles_per_split_quantised", "tiles_per_split_fp16",
                                              "units_per_kv_head")]


class kivi_cache_sizes_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in (
        "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid")]


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """dlopen libkivi_hip.so (built in-tree by paper_2402_02750_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2402_02750_amd.build). "
            "There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    P, I32, I64, VP = ctypes.POINTER, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.kivi_status_string.restype = ctypes.c_char_p
    lib.kivi_status_string.argtypes = [ctypes.c_int]
    lib.kivi_cache_sizes.argtypes = [P(kivi_layout_t), P(kivi_cache_sizes_t)]
    lib.kivi_decode_workspace_bytes.argtypes = [P(kivi_layout_t), P(ctypes.c_size_t)]
    lib.kivi_decode_plan.argtypes = [P(kivi_layout_t), P(kivi_cache_t), P(kivi_decode_plan_t)]
    for name in ("kivi_quantize_key_groups", "kivi_quantize_value_tokens"):
        getattr(lib, name).argtypes = [P(kivi_layout_t), VP, I64, I64, I64, I32, P(kivi_cache_t), VP]
    lib.kivi_prefill.argtypes = [P(kivi_layout_t), VP, I64, I64, I64, VP, I64, I64, I64, I32, I32,
                                 P(kivi_cache_t), VP]
    lib.kivi_append_residual.argtypes = [P(kivi_layout_t), P(kivi_cache_t), VP, VP, VP]
    lib.kivi_flush_residual.argtypes = [P(kivi_layout_t), P(kivi_cache_t), I32, P(I32), P(I32), VP]
    lib.kivi_decode_attention.argtypes = [P(kivi_layout_t), P(kivi_cache_t), VP, ctypes.c_float,
                                          VP, VP, ctypes.c_size_t, VP]
    lib.kivi_decode_launches_ragged.argtypes = [P(kivi_layout_t), P(kivi_seq_state_t), P(I32)]
    lib.kivi_decode_attention_static.argtypes = [P(kivi_layout_t), P(kivi_cache_t), VP, ctypes.c_float, VP, VP]
    lib.kivi_decode_step.argtypes = [P(kivi_layout_t), P(kivi_cache_t), VP, VP, VP, ctypes.c_float, I32,
                                     VP, VP, ctypes.c_size_t, VP]
    lib.kivi_stream_read_probe.argtypes = [VP, ctypes.c_size_t, VP, VP]
    lib.kivi_batch_slice.argtypes = [P(kivi_layout_t), P(kivi_cache_t), I32, I32, P(kivi_seq_state_t),
                                     P(kivi_layout_t), P(kivi_cache_t)]
    lib.kivi_decode_step_ragged.argtypes = [P(kivi_layout_t), P(kivi_cache_t), P(kivi_seq_state_t), VP, VP, VP,
                                            ctypes.c_float, I32, VP, VP, ctypes.c_size_t, VP]
    lib.kivi_decode_attention_ragged.argtypes = [P(kivi_layout_t), P(kivi_cache_t), P(kivi_seq_state_t), VP,
                                                 ctypes.c_float, VP, VP, ctypes.c_size_t, VP]
    for name in EXPORTS[1:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().kivi_status_string(status).decode()


def _check(status: int, where: str):
    if status != KIVI_OK:
        raise KiviError(status, where)


def make_layout(batch, n_q_heads, n_kv_heads, bits, residual, cap_q_tokens, cap_r_tokens,
                head_dim=128, group=32, decode_path=KIVI_DECODE_AUTO) -> kivi_layout_t:
    return kivi_layout_t(batch, n_q_heads, n_kv_heads, head_dim, bits, group, residual,
                         cap_q_tokens, cap_r_tokens, decode_path)


def kivi_cache_sizes(layout: kivi_layout_t) -> kivi_cache_sizes_t:
    sizes = kivi_cache_sizes_t()
    _check(load_library().kivi_cache_sizes(ctypes.byref(layout), ctypes.byref(sizes)), "kivi_cache_sizes")
    return sizes


def kivi_decode_plan(layout: kivi_layout_t, cache) -> kivi_decode_plan_t:
    """How kivi_decode_attention would serve the cache's current state (`cache`: a Cache or kivi_cache_t)."""
    plan = kivi_decode_plan_t()
    c = cache.c if hasattr(cache, "c") else cache
    _check(load_library().kivi_decode_plan(ctypes.byref(layout), ctypes.byref(c), ctypes.byref(plan)), "kivi_decode_plan")
    return plan


def kivi_decode_workspace_bytes(layout: kivi_layout_t) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().kivi_decode_workspace_bytes(ctypes.byref(layout), ctypes.byref(n)),
           "kivi_decode_workspace_bytes")
    return n.value


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _strides_bht(x):
    assert x.dim() == 4 and x.stride(3) == 1, "expected [b, h, t, 128] with contiguous channels"
    return x.stride(0), x.stride(1), x.stride(2)


class Cache:
    """Device buffers (torch tensors) + the kivi_cache_t that points at them."""

    _NAMES = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid")

    # Optional byte offset between the starts of consecutive arrays inside their allocations (an
    # experiment knob: the decode kernel visits the chunks of different units in different order, so
    # its speed no longer depends on how the arrays are placed relative to each other).
    DEFAULT_SKEW = 0

    def __init__(self, layout: kivi_layout_t, device="cuda", skew=None):
        """`skew` (a multiple of 16 bytes, default DEFAULT_SKEW): the i-th array starts i * skew bytes
        into its allocation."""
        skew = self.DEFAULT_SKEW if skew is None else skew
        import torch
        assert skew % 16 == 0
        self.layout = layout
        sizes = kivi_cache_sizes(layout)
        self.buffers = {}
        self.c = kivi_cache_t()
        for i, name in enumerate(self._NAMES):
            nbytes = max(int(getattr(sizes, name)), 16)
            raw = torch.empty(nbytes + i * skew, dtype=torch.uint8, device=device)
            buf = raw[i * skew:]
            self.buffers[name] = buf
            setattr(self.c, name, buf.data_ptr())
        ws = kivi_decode_workspace_bytes(layout)
        # zero-filled once: the decode kernel keeps its split counters at zero between calls
        self.workspace = torch.zeros(max(ws, 16), dtype=torch.uint8, device=device)

    # convenience typed views (tests compare these against the oracle)
    def view(self, name):
        import torch
        l = self.layout
        units = (l.batch, l.n_kv_heads)
        tiles = l.cap_q_tokens // 32
        buf = self.buffers[name]
        if name in ("k_codes", "v_codes"):
            return buf.view(torch.int32).view(*units, tiles, 32 * 128 * l.bits // 32)
        if name in ("k_scale", "k_zero"):       # one row per group of G tokens
            return buf.view(torch.float16).view(*units, l.cap_q_tokens // l.group, 128)
        if name in ("v_scale", "v_zero"):       # one entry per group of G channels
            return buf.view(torch.float16).view(*units, l.cap_q_tokens, 128 // l.group)
        return buf.view(torch.float16).view(*units, l.cap_r_tokens, 128)


def kivi_quantize_key_groups(layout, k_fp16, n_tokens, cache: Cache, stream=None):
    """k_fp16: CUDA fp16 tensor [b, H_kv, >= n_tokens, 128] (any b/h/t strides)."""
    sb, sh, st = _strides_bht(k_fp16)
    _check(load_library().kivi_quantize_key_groups(
        ctypes.byref(layout), ctypes.c_void_p(k_fp16.data_ptr()), sb, sh, st, n_tokens,
        ctypes.byref(cache.c), _stream_handle(stream)), "kivi_quantize_key_groups")


def kivi_quantize_value_tokens(layout, v_fp16, n_tokens, cache: Cache, stream=None):
    sb, sh, st = _strides_bht(v_fp16)
    _check(load_library().kivi_quantize_value_tokens(
        ctypes.byref(layout), ctypes.c_void_p(v_fp16.data_ptr()), sb, sh, st, n_tokens,
        ctypes.byref(cache.c), _stream_handle(stream)), "kivi_quantize_value_tokens")


def kivi_prefill(layout, k_fp16, v_fp16, n_tokens, cache: Cache, policy=KIVI_FLUSH_WINDOW, stream=None):
    """k_fp16, v_fp16: CUDA fp16 tensors [b, H_kv, >= n_tokens, 128]."""
    ks, vs = _strides_bht(k_fp16), _strides_bht(v_fp16)
    _check(load_library().kivi_prefill(
        ctypes.byref(layout), ctypes.c_void_p(k_fp16.data_ptr()), *ks,
        ctypes.c_void_p(v_fp16.data_ptr()), *vs, n_tokens, policy, ctypes.byref(cache.c),
        _stream_handle(stream)), "kivi_prefill")


def kivi_append_residual(layout, cache: Cache, k_new, v_new, stream=None):
    """k_new, v_new: contiguous CUDA fp16 tensors [b, H_kv, 128]."""
    assert k_new.is_contiguous() and v_new.is_contiguous()
    _check(load_library().kivi_append_residual(
        ctypes.byref(layout), ctypes.byref(cache.c), ctypes.c_void_p(k_new.data_ptr()),
        ctypes.c_void_p(v_new.data_ptr()), _stream_handle(stream)), "kivi_append_residual")


def kivi_flush_residual(layout, cache: Cache, policy=KIVI_FLUSH_WINDOW, stream=None):
    nk, nv = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load_library().kivi_flush_residual(
        ctypes.byref(layout), ctypes.byref(cache.c), policy, ctypes.byref(nk), ctypes.byref(nv),
        _stream_handle(stream)), "kivi_flush_residual")
    return nk.value, nv.value


def kivi_decode_attention(layout, cache: Cache, q_fp16, softmax_scale, out_fp32, stream=None):
    """q_fp16: contiguous CUDA fp16 [b, H_q, 128]; out_fp32: contiguous CUDA fp32 [b, H_q, 128]."""
    assert q_fp16.is_contiguous() and out_fp32.is_contiguous()
    _check(load_library().kivi_decode_attention(
        ctypes.byref(layout), ctypes.byref(cache.c), ctypes.c_void_p(q_fp16.data_ptr()),
        ctypes.c_float(softmax_scale), ctypes.c_void_p(out_fp32.data_ptr()),
        ctypes.c_void_p(cache.workspace.data_ptr()), cache.workspace.numel(),
        _stream_handle(stream)), "kivi_decode_attention")
    return out_fp32


def kivi_decode_attention_static(layout, cache, q_fp16, softmax_scale, out_fp32, stream=None):
    """kivi_decode_attention on the library's static workspace (no allocation, no workspace argument)."""
    assert q_fp16.is_contiguous() and out_fp32.is_contiguous()
    _check(load_library().kivi_decode_attention_static(
        ctypes.byref(layout), ctypes.byref(cache.c), ctypes.c_void_p(q_fp16.data_ptr()),
        ctypes.c_float(softmax_scale), ctypes.c_void_p(out_fp32.data_ptr()), _stream_handle(stream)),
        "kivi_decode_attention_static")
    return out_fp32


def kivi_decode_step(layout, cache: Cache, k_new, v_new, q_fp16, softmax_scale, out_fp32,
                     policy=KIVI_FLUSH_WINDOW, stream=None):
    """Append + flush + attention of one decoding step.  k_new, v_new: contiguous CUDA fp16
    [b, H_kv, 128] (keep them alive until the launch has run); q_fp16 / out_fp32 as for
    kivi_decode_attention."""
    assert k_new.is_contiguous() and v_new.is_contiguous()
    assert q_fp16.is_contiguous() and out_fp32.is_contiguous()
    _check(load_library().kivi_decode_step(
        ctypes.byref(layout), ctypes.byref(cache.c), ctypes.c_void_p(k_new.data_ptr()),
        ctypes.c_void_p(v_new.data_ptr()), ctypes.c_void_p(q_fp16.data_ptr()),
        ctypes.c_float(softmax_scale), policy, ctypes.c_void_p(out_fp32.data_ptr()),
        ctypes.c_void_p(cache.workspace.data_ptr()), cache.workspace.numel(),
        _stream_handle(stream)), "kivi_decode_step")
    return out_fp32


def kivi_stream_read_probe(src, sink, stream=None):
    """Measurement helper: plain read-only stream over the CUDA tensor `src` (any dtype, contiguous,
    a multiple of 16 bytes); `sink`: CUDA tensor of at least 16 KiB."""
    assert src.is_contiguous() and sink.numel() * sink.element_size() >= 4096 * 4
    _check(load_library().kivi_stream_read_probe(
        ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(), ctypes.c_void_p(sink.data_ptr()),
        _stream_handle(stream)), "kivi_stream_read_probe")


class CacheSlice:
    """Batch entries [b0, b0 + nb) of a Cache as a cache of their own (kivi_batch_slice): `layout`
    and `c` can be passed to every entry point, e.g. to prefill one sequence of a ragged batch."""

    def __init__(self, cache: Cache, b0: int, nb: int, state=None):
        self.parent = cache
        self.layout = kivi_layout_t()
        self.c = kivi_cache_t()
        self.workspace = cache.workspace
        _check(load_library().kivi_batch_slice(
            ctypes.byref(cache.layout), ctypes.byref(cache.c), b0, nb,
            ctypes.byref(state) if state is not None else None,
            ctypes.byref(self.layout), ctypes.byref(self.c)), "kivi_batch_slice")

    def state(self) -> kivi_seq_state_t:
        return kivi_seq_state_t(self.c.n_kq, self.c.n_vq, self.c.k_r_start, self.c.n_kr, self.c.v_r_start, self.c.n_vr)


def make_states(batch: int):
    """Host array of per-sequence states (all empty) for the ragged entry points."""
    return (kivi_seq_state_t * batch)()


def kivi_decode_step_ragged(layout, cache: Cache, states, k_new, v_new, q_fp16, softmax_scale, out_fp32,
                            policy=KIVI_FLUSH_WINDOW, stream=None):
    """kivi_decode_step over a batch whose sequences differ in length; `states` from make_states."""
    assert k_new.is_contiguous() and v_new.is_contiguous() and q_fp16.is_contiguous() and out_fp32.is_contiguous()
    _check(load_library().kivi_decode_step_ragged(
        ctypes.byref(layout), ctypes.byref(cache.c), states, ctypes.c_void_p(k_new.data_ptr()),
        ctypes.c_void_p(v_new.data_ptr()), ctypes.c_void_p(q_fp16.data_ptr()), ctypes.c_float(softmax_scale),
        policy, ctypes.c_void_p(out_fp32.data_ptr()), ctypes.c_void_p(cache.workspace.data_ptr()),
        cache.workspace.numel(), _stream_handle(stream)), "kivi_decode_step_ragged")
    return out_fp32


def kivi_decode_launches_ragged(layout, states) -> int:
    """Kernel launches kivi_decode_attention_ragged would enqueue for these sequence states."""
    n = ctypes.c_int32(0)
    _check(load_library().kivi_decode_launches_ragged(ctypes.byref(layout), states, ctypes.byref(n)),
           "kivi_decode_launches_ragged")
    return n.value


def kivi_decode_attention_ragged(layout, cache: Cache, states, q_fp16, softmax_scale, out_fp32, stream=None):
    assert q_fp16.is_contiguous() and out_fp32.is_contiguous()
    _check(load_library().kivi_decode_attention_ragged(
        ctypes.byref(layout), ctypes.byref(cache.c), states, ctypes.c_void_p(q_fp16.data_ptr()),
        ctypes.c_float(softmax_scale), ctypes.c_void_p(out_fp32.data_ptr()),
        ctypes.c_void_p(cache.workspace.data_ptr()), cache.workspace.numel(), _stream_handle(stream)),
        "kivi_decode_attention_ragged")
    return out_fp32
