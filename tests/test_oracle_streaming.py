"""Pins for the oracle's streaming cache (KIVI Algorithm 1; Section 3.3 "Analysis")."""
import numpy as np
import pytest

from oracle import kivi_oracle as ko


def _kv(rng, b, h, n, d=128):
    k = (rng.standard_normal((b, h, n, d)) * np.where(np.arange(d) % 37 == 0, 9.0, 1.0)).astype(np.float16)
    v = rng.standard_normal((b, h, n, d)).astype(np.float16)
    return k, v


@pytest.mark.parametrize("policy", ["window", "alg1"])
@pytest.mark.parametrize("bits", [2, 4])
def test_streaming_equals_batch(policy, bits):
    """Groups are independent, so the cache after any prefill + append sequence is bit-identical
    to quantising the same token ranges in one go, and the fp16 parts are the untouched tail."""
    rng = np.random.default_rng(17)
    b, h, G, R = 1, 2, 32, 64
    total = 300
    k, v = _kv(rng, b, h, total)
    for prompt in (0, 1, 63, 64, 65, 200):
        c = ko.StreamingCache(b, h, 128, bits, G, R, policy)
        c.prefill(k[:, :, :prompt], v[:, :, :prompt])
        for t in range(prompt, total):
            c.append(k[:, :, t], v[:, :, t])
            assert c.n_kq + c.n_kr == t + 1 == c.n_vq + c.n_vr
            assert c.n_kq % G == 0
        ck, sk, zk = ko.quantize_key(k[:, :, :c.n_kq], bits, G)
        cv, sv, zv = ko.quantize_value(v[:, :, :c.n_vq], bits, G)
        assert (c.k_codes == ck).all() and (c.k_scale == sk).all() and (c.k_zero == zk).all()
        assert (c.v_codes == cv).all() and (c.v_scale == sv).all() and (c.v_zero == zv).all()
        assert (c.k_resid == k[:, :, c.n_kq:]).all() and (c.v_resid == v[:, :, c.n_vq:]).all()


def test_window_policy_keeps_recent_R_tokens_fp16():
    rng = np.random.default_rng(1)
    G, R = 32, 128
    k, v = _kv(rng, 1, 1, 2048 + 256)
    c = ko.StreamingCache(1, 1, 128, 2, G, R, "window")
    c.prefill(k[:, :, :2048], v[:, :, :2048])
    assert (c.n_kq, c.n_kr) == (1920, 128)
    flush_steps = []
    for step in range(1, 257):
        t = 2048 + step - 1
        nk, nv = c.append(k[:, :, t], v[:, :, t])
        assert nk == nv
        if nk:
            assert nk == G
            flush_steps.append(step)
        assert R <= c.n_kr <= R + G - 1 and c.n_kr == c.n_vr
    assert flush_steps == [32, 64, 96, 128, 160, 192, 224, 256]
    assert (c.n_kq, c.n_kr) == (2176, 128)


def test_alg1_policy_window_sizes():
    """Algorithm 1: the key residual is flushed whole when it reaches R tokens (so it holds
    0..R-1 tokens, R/2 on average) and the value residual holds exactly R tokens once l >= R
    (Section 3.3 "Analysis")."""
    rng = np.random.default_rng(2)
    G, R = 32, 128
    k, v = _kv(rng, 1, 1, 200 + 1024)
    c = ko.StreamingCache(1, 1, 128, 2, G, R, "alg1")
    c.prefill(k[:, :, :200], v[:, :, :200])
    assert (c.n_kq, c.n_kr) == (128, 72)          # KeyQuant: r = l % R
    assert (c.n_vq, c.n_vr) == (72, 128)          # X_Vr = X_V[l-R:]
    sizes = []
    for t in range(200, 200 + 1024):
        nk, nv = c.append(k[:, :, t], v[:, :, t])
        assert nv == 1 and c.n_vr == R
        assert nk in (0, R) and 0 <= c.n_kr < R
        sizes.append(c.n_kr)
    assert abs(np.mean(sizes) - R / 2) <= 1.0


def test_attention_through_cache_matches_direct_call():
    rng = np.random.default_rng(6)
    k, v = _kv(rng, 2, 2, 200)
    q = rng.standard_normal((2, 4, 128)).astype(np.float16)
    c = ko.StreamingCache(2, 2, 128, 2, 32, 64, "window")
    c.prefill(k[:, :, :150], v[:, :, :150])
    for t in range(150, 200):
        c.append(k[:, :, t], v[:, :, t])
    out = c.attention(q, 0.088)
    nq = c.n_kq
    ref = ko.decode_attention(q, ko.quantize_key(k[:, :, :nq], 2, 32), k[:, :, nq:],
                              ko.quantize_value(v[:, :, :nq], 2, 32), v[:, :, nq:], 32, 0.088)
    assert (out == ref).all()
