"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI binding and the
oracle on the same seeded inputs, and compare.  (No arithmetic of the method lives here.)"""
from __future__ import annotations

import numpy as np

from oracle import kivi_oracle as ko
from paper_2402_02750_amd import kivi, workloads

ABS_TOL = 2e-3   # gate: |gpu - ref| <= ABS_TOL + REL_TOL * |ref|, element-wise
REL_TOL = 1e-2


def require_gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU (run with -m gpu on the MI355X box)"
    kivi.load_library()     # raises if the HIP library was not built: no fallback
    return torch


def round_up(x, m):
    return (x + m - 1) // m * m


def gpu_prefill(w, k_np, v_np, policy, decode_path, extra_q_tokens=0):
    """Upload K, V ([b, h, l, 128] fp16 numpy) and run kivi_prefill.  Returns (layout, cache)."""
    import torch
    l = k_np.shape[2]
    cap_q = max(round_up(l + extra_q_tokens, w.group), w.group)
    cap_r = round_up(w.residual + w.group, 32) + 32
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, cap_q, cap_r,
                              decode_path=decode_path, group=w.group)
    cache = kivi.Cache(layout)
    kt = torch.from_numpy(k_np).cuda()
    vt = torch.from_numpy(v_np).cuda()
    kivi.kivi_prefill(layout, kt, vt, l, cache, policy)
    torch.cuda.synchronize()
    return layout, cache


def compare_quantized_state(cache, oc: ko.StreamingCache, heads=None):
    """Bit-exact comparison of packed codes, scales, zero-points and the fp16 residual parts.
    `oc` holds either all (b, h) or the listed `heads` as a pseudo-batch [len(heads), 1]."""
    import torch
    c = cache.c
    assert (c.n_kq, c.n_kr, c.n_vq, c.n_vr) == (oc.n_kq, oc.n_kr, oc.n_vq, oc.n_vr)
    bits = cache.layout.bits
    cap_r = cache.layout.cap_r_tokens

    def pick(t):
        if heads is None:
            return t.cpu().numpy()
        # slice on the device: at full sizes the arrays hold gigabytes
        return torch.stack([t[b, h] for b, h in heads])[:, None].cpu().numpy()

    nkt, nvt = oc.n_kq // 32, (oc.n_vq + 31) // 32
    # scales and zero-points: one per group (keys: a row per G tokens; values: 128 / G entries per token)
    nkg = oc.n_kq // cache.layout.group
    if nkt:
        got = pick(cache.view("k_codes")[:, :, :nkt]).view(np.uint32)
        assert np.array_equal(got, ko.pack_key_codes(oc.k_codes, bits)), "key codes differ"
        assert np.array_equal(pick(cache.view("k_scale")[:, :, :nkg]).view(np.uint16), oc.k_scale.view(np.uint16))
        assert np.array_equal(pick(cache.view("k_zero")[:, :, :nkg]).view(np.uint16), oc.k_zero.view(np.uint16))
    if oc.n_vq:
        got = pick(cache.view("v_codes")[:, :, :nvt]).view(np.uint32)
        pad = nvt * 32 - oc.n_vq
        codes = oc.v_codes
        if pad:   # a partly filled tile: compare only the bits of valid tokens
            codes = np.concatenate([codes, np.zeros(codes.shape[:2] + (pad, 128), np.uint16)], axis=2)
            valid = np.concatenate([np.full(oc.v_codes.shape, 2 ** bits - 1, np.uint16),
                                    np.zeros(codes.shape[:2] + (pad, 128), np.uint16)], axis=2)
            got = got & ko.pack_value_codes(valid, bits)
        assert np.array_equal(got, ko.pack_value_codes(codes, bits)), "value codes differ"
        assert np.array_equal(pick(cache.view("v_scale")[:, :, :oc.n_vq]).view(np.uint16), oc.v_scale.view(np.uint16))
        assert np.array_equal(pick(cache.view("v_zero")[:, :, :oc.n_vq]).view(np.uint16), oc.v_zero.view(np.uint16))
    for name, start, n, ref in (("k_resid", c.k_r_start, c.n_kr, oc.k_resid),
                                ("v_resid", c.v_r_start, c.n_vr, oc.v_resid)):
        if n:
            slots = (start + np.arange(n)) % cap_r
            got = pick(cache.view(name))[:, :, slots]
            assert np.array_equal(got.view(np.uint16), ref.view(np.uint16)), name


def check_close(got: np.ndarray, ref: np.ndarray, what=""):
    err = np.abs(got.astype(np.float64) - ref)
    tol = ABS_TOL + REL_TOL * np.abs(ref)
    worst = float((err - tol).max())
    assert worst <= 0, f"{what}: max abs err {err.max():.3e}, tolerance exceeded by {worst:.3e}"
    return float(err.max())


def oracle_cache_for_heads(w, k_np, v_np, heads, policy):
    """Oracle cache over the listed (b, h) pairs, laid out as a pseudo-batch [len(heads), 1]."""
    oc = ko.StreamingCache(len(heads), 1, w.head_dim, w.bits, w.group, w.residual, policy)
    ks = np.stack([k_np[b, h] for b, h in heads])[:, None]
    vs = np.stack([v_np[b, h] for b, h in heads])[:, None]
    oc.prefill(ks, vs)
    return oc


def oracle_attention_for_heads(w, oc, q_np, heads):
    """fp64 outputs [len(heads), rep, 128] for the query heads that read the listed kv-heads."""
    rep = w.q_per_kv
    qs = np.stack([q_np[b, h * rep:(h + 1) * rep] for b, h in heads])       # [n, rep, 128]
    return oc.attention(qs, w.softmax_scale)


def gpu_attention(layout, cache, q_np, scale):
    import torch
    qt = torch.from_numpy(q_np).cuda()
    out = torch.empty(q_np.shape, dtype=torch.float32, device="cuda")
    kivi.kivi_decode_attention(layout, cache, qt, scale, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def pick_heads(out_np, w, heads):
    rep = w.q_per_kv
    return np.stack([out_np[b, h * rep:(h + 1) * rep] for b, h in heads])
