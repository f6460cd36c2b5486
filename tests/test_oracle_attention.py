"""Pins for the oracle's decode attention (KIVI Equations 1 and 4, Algorithm 1 Decoding)."""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import kivi_oracle as ko


def _textbook(q, k, v, scale, rep):
    """softmax(scale * q K^T) V with library routines, fp64, grouped-query aware."""
    b, hq, d = q.shape
    out = np.empty((b, hq, d))
    for bi in range(b):
        for j in range(hq):
            kk = k[bi, j // rep].astype(np.float64)
            vv = v[bi, j // rep].astype(np.float64)
            p = scipy_softmax(scale * kk @ q[bi, j].astype(np.float64))
            out[bi, j] = p @ vv
    return out


def _empty_quant(b, h, d, g):
    return ((np.zeros((b, h, 0, d), np.uint16), np.zeros((b, h, 0, d), np.float16),
             np.zeros((b, h, 0, d), np.float16)),
            (np.zeros((b, h, 0, d), np.uint16), np.zeros((b, h, 0, d // g), np.float16),
             np.zeros((b, h, 0, d // g), np.float16)))


def test_all_residual_is_textbook_attention():
    """With nothing quantised (l < R) the method is Equation 1 itself."""
    rng = np.random.default_rng(0)
    b, hq, hkv, d, n = 2, 4, 2, 128, 77
    q = rng.standard_normal((b, hq, d)).astype(np.float16)
    k = rng.standard_normal((b, hkv, n, d)).astype(np.float16)
    v = rng.standard_normal((b, hkv, n, d)).astype(np.float16)
    kq, vq = _empty_quant(b, hkv, d, 32)
    out = ko.decode_attention(q, kq, k, vq, v, 32, 0.3)
    ref = _textbook(q, k, v, 0.3, hq // hkv)
    assert np.abs(out - ref).max() < 1e-12


def _lossless_kv(rng, n, d, g, bits):
    """K and V that the quantiser represents exactly: every group is z + code * s with a
    power-of-two s, and contains both the lowest and the highest code."""
    levels = 2 ** bits - 1
    def make(groups_shape, glen):
        s = 2.0 ** rng.integers(-4, 2, size=groups_shape)
        z = rng.integers(-16, 16, size=groups_shape) * 0.125
        codes = rng.integers(0, levels + 1, size=groups_shape + (glen,))
        codes[..., 0] = 0
        codes[..., 1] = levels
        codes = rng.permuted(codes, axis=-1)
        return z[..., None] + codes * s[..., None]
    k = make((n // g, d), g)                   # [n/G, D, G] -> tokens inside a group last
    k = np.swapaxes(k, -1, -2).reshape(n, d)
    v = make((n, d // g), g).reshape(n, d)
    return k.astype(np.float16), v.astype(np.float16)


@pytest.mark.parametrize("bits", [2, 4])
def test_lossless_cache_equals_textbook_attention(bits):
    """If every group is exactly representable the quantised cache *is* the cache, so the whole
    mixed-precision path (per-channel key groups, per-token value groups, residual part, softmax
    over the concatenation, grouped-query mapping) must equal Equation 1 on the raw tensors."""
    rng = np.random.default_rng(21 + bits)
    b, hq, hkv, d, g = 2, 4, 2, 128, 32
    n_q, n_r = 96, 40
    ks, vs = [], []
    for _ in range(b * hkv):
        k, v = _lossless_kv(rng, n_q, d, g, bits)
        ks.append(k); vs.append(v)
    kq_raw = np.stack(ks).reshape(b, hkv, n_q, d)
    vq_raw = np.stack(vs).reshape(b, hkv, n_q, d)
    kr = rng.standard_normal((b, hkv, n_r, d)).astype(np.float16)
    vr = rng.standard_normal((b, hkv, n_r, d)).astype(np.float16)
    q = (rng.standard_normal((b, hq, d)) * 0.3).astype(np.float16)
    kq = ko.quantize_key(kq_raw, bits, g)
    vq = ko.quantize_value(vq_raw, bits, g)
    assert (ko.dequantize_key(*kq, g) == kq_raw).all()
    assert (ko.dequantize_value(*vq, g) == vq_raw).all()
    out = ko.decode_attention(q, kq, kr, vq, vr, g, 0.09)
    ref = _textbook(q, np.concatenate([kq_raw, kr], 2), np.concatenate([vq_raw, vr], 2), 0.09,
                    hq // hkv)
    assert np.abs(out - ref).max() < 1e-12


def test_16bit_no_residual_reproduces_bruteforce_fp32_attention():
    """B = 16, R = 0 (oracle-only mode, fp32 scale): the cache is nearly lossless and the result
    must match brute-force fp32 attention on the unquantised tensors."""
    rng = np.random.default_rng(4)
    b, h, d, n, g = 1, 2, 128, 64, 32
    q = rng.standard_normal((b, h, d)).astype(np.float16)
    k = rng.standard_normal((b, h, n, d)).astype(np.float16)
    v = rng.standard_normal((b, h, n, d)).astype(np.float16)
    kq = ko.quantize_key(k, 16, g, scale_dtype=np.float32)
    vq = ko.quantize_value(v, 16, g, scale_dtype=np.float32)
    empty = np.zeros((b, h, 0, d), np.float16)
    out = ko.decode_attention(q, kq, empty, vq, empty, g, 1 / np.sqrt(d))
    # brute force, scalar fp32 loops
    f = np.float32
    ref = np.zeros((b, h, d), f)
    for bi in range(b):
        for hi in range(h):
            logits = np.zeros(n, f)
            for t in range(n):
                acc = f(0)
                for c in range(d):
                    acc = f(acc + f(q[bi, hi, c]) * f(k[bi, hi, t, c]))
                logits[t] = acc * f(1 / np.sqrt(d))
            m = logits.max()
            e = np.exp(logits - m).astype(f)
            p = e / e.sum(dtype=f)
            for c in range(d):
                acc = f(0)
                for t in range(n):
                    acc = f(acc + p[t] * f(v[bi, hi, t, c]))
                ref[bi, hi, c] = acc
    assert np.abs(out - ref).max() < 1e-4


def test_equal_keys_give_mean_of_values():
    """All keys equal -> uniform attention -> output is the mean of the (dequantised) values.
    Values are placed on an exactly representable grid so the mean is known in closed form."""
    rng = np.random.default_rng(8)
    b, h, d, g, n_q, n_r = 1, 1, 128, 32, 64, 32
    krow = rng.standard_normal(d).astype(np.float16)
    k = np.broadcast_to(krow, (b, h, n_q + n_r, d)).copy()
    _, v = _lossless_kv(rng, n_q + n_r, d, g, 2)
    v = v.reshape(b, h, n_q + n_r, d)
    q = rng.standard_normal((b, h, d)).astype(np.float16)
    out = ko.decode_attention(q, ko.quantize_key(k[:, :, :n_q], 2, g), k[:, :, n_q:],
                              ko.quantize_value(v[:, :, :n_q], 2, g), v[:, :, n_q:], g, 0.1)
    assert np.abs(out[0, 0] - v[0, 0].astype(np.float64).mean(0)).max() < 1e-12


def test_dominant_logit_selects_its_value_row():
    rng = np.random.default_rng(12)
    b, h, d, g, n_q, n_r = 1, 1, 128, 32, 64, 32
    q = np.zeros((b, h, d), np.float16); q[0, 0, 5] = 8.0
    k = np.zeros((b, h, n_q + n_r, d), np.float16)
    k[0, 0, 37, 5] = 60.0                                    # token 37 (quantised part) dominates
    _, v = _lossless_kv(rng, n_q + n_r, d, g, 2)
    v = v.reshape(b, h, -1, d)
    out = ko.decode_attention(q, ko.quantize_key(k[:, :, :n_q], 2, g), k[:, :, n_q:],
                              ko.quantize_value(v[:, :, :n_q], 2, g), v[:, :, n_q:], g, 1.0)
    assert np.abs(out[0, 0] - v[0, 0, 37].astype(np.float64)).max() < 1e-9


def test_group_permutation_invariance_and_split_choice():
    """Attention is a sum over tokens: permuting whole token groups of (K, V) together, or moving
    the K/V split points independently (Algorithm 1 splits K and V differently), cannot change
    the output when the moved tokens are exactly representable."""
    rng = np.random.default_rng(31)
    d, g = 128, 32
    k, v = _lossless_kv(rng, 128, d, g, 2)
    q = (rng.standard_normal((1, 1, d)) * 0.2).astype(np.float16)
    K = k.reshape(1, 1, 128, d); V = v.reshape(1, 1, 128, d)

    def run(K, V, n_kq, n_vq):
        return ko.decode_attention(q, ko.quantize_key(K[:, :, :n_kq], 2, g), K[:, :, n_kq:],
                                   ko.quantize_value(V[:, :, :n_vq], 2, g), V[:, :, n_vq:], g, 0.1)
    base = run(K, V, 96, 96)
    perm = np.concatenate([np.arange(64, 96), np.arange(0, 32), np.arange(32, 64), np.arange(96, 128)])
    assert np.abs(run(K[:, :, perm], V[:, :, perm], 96, 96) - base).max() < 1e-12
    assert np.abs(run(K, V, 64, 96) - base).max() < 1e-12
    assert np.abs(run(K, V, 128, 33) - base).max() < 1e-12
    assert np.abs(run(K, V, 0, 0) - base).max() < 1e-12


def test_logits_concat_order():
    """Equation 4: A = Concat(A_g, A_r) -- quantised tokens first, residual tokens after."""
    rng = np.random.default_rng(2)
    d, g = 128, 32
    k, _ = _lossless_kv(rng, 64, d, g, 2)
    kr = rng.standard_normal((1, 1, 5, d)).astype(np.float16)
    q = rng.standard_normal((1, 1, d)).astype(np.float16)
    a = ko.attention_logits(q, ko.quantize_key(k.reshape(1, 1, 64, d), 2, g), kr, g, 0.5)
    ref = 0.5 * np.concatenate([k.astype(np.float64), kr[0, 0].astype(np.float64)]) @ q[0, 0].astype(np.float64)
    assert a.shape == (1, 1, 69) and np.abs(a[0, 0] - ref).max() < 1e-12
