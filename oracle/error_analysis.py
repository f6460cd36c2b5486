"""Error-analysis harness of the KIVI paper's Section 3.2 (Table 2) on synthetic data.
TEST INFRASTRUCTURE ONLY -- built on oracle/kivi_oracle.py, used by tests; the HIP library never
touches it.

The paper fake-quantises (quantise, then dequantise) the key and the value cache of one head in
the two grouping directions and reports, averaged over layers and heads of Llama-2-13B,
  * the relative key reconstruction error and the relative attention-score error with
    A' = Softmax(t_Q X_K'^T)                                  -- Section 3.2 "Analysis of Key Cache";
  * the relative value reconstruction error and Delta, the relative error of the attention output
    A X_V with the value cache replaced by its reconstruction -- "Analysis of Value Cache".
Its numbers need the model's activations: parity unpinned.  What can be reproduced is the
ORDERING, on inputs that carry the two structures the paper names: a few fixed key channels of
large magnitude (Figure 2), and sparse attention (the paper measures 84.3 % sparsity) over value
rows whose magnitudes differ from token to token, so that a per-channel value group mixes heavy
and light tokens.

Readings: the printed norm of an element-wise quotient is taken as ||X - X'||_F / ||X||_F (an
element-wise quotient is undefined where X has zeros); errors are fractions, not percent; "fake
quantisation" pads nothing here because the token count is a multiple of the group size.
"""
from __future__ import annotations

import numpy as np

from oracle import kivi_oracle as ko


def fake_quantize(x: np.ndarray, bits: int, group: int, direction: str) -> np.ndarray:
    """x: [tokens, channels] fp16.  direction 'channel': groups of `group` consecutive tokens per
    channel (the key cache's direction in KIVI); 'token': groups of `group` consecutive channels
    per token (the value cache's direction).  Returns the fp64 reconstruction."""
    x4 = x[None, None]
    if direction == "channel":
        return ko.dequantize_key(*ko.quantize_key(x4, bits, group), group)[0, 0]
    if direction == "token":
        return ko.dequantize_value(*ko.quantize_value(x4, bits, group), group)[0, 0]
    raise ValueError(direction)


def relative_error(ref: np.ndarray, approx: np.ndarray) -> float:
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(ref - approx) / np.linalg.norm(ref))


def attention_sparsity(a: np.ndarray, threshold: float = 0.01) -> float:
    """Share of attention probabilities below `threshold` times the row maximum."""
    a = np.atleast_2d(a)
    return float((a < threshold * a.max(axis=-1, keepdims=True)).mean())


def analyze_head(q: np.ndarray, k: np.ndarray, v: np.ndarray, bits: int, group: int, scale: float) -> dict:
    """q: [n_queries, channels], k, v: [tokens, channels], all fp16.  Returns the four error
    statistics of Table 2 for both grouping directions of K and of V, plus the sparsity."""
    q64, k64, v64 = (np.asarray(t, np.float64) for t in (q, k, v))
    a = ko.softmax(scale * (q64 @ k64.T))
    out = {"sparsity": attention_sparsity(a)}
    for direction in ("token", "channel"):
        kq = fake_quantize(k, bits, group, direction)
        vq = fake_quantize(v, bits, group, direction)
        out[f"k_{direction}"] = {
            "reconstruction": relative_error(k64, kq),
            "attention_score": relative_error(a, ko.softmax(scale * (q64 @ kq.T))),
        }
        out[f"v_{direction}"] = {
            "reconstruction": relative_error(v64, vq),
            "attention_output": relative_error(a @ v64, a @ vq),
        }
    return out


def synthetic_head(seed: int, tokens: int = 1024, channels: int = 128, n_queries: int = 16,
                   n_outlier_channels: int = 4, outlier_gain: float = 12.0, token_scale_sigma: float = 1.0,
                   peak: float = 8.0, noise: float = 0.3):
    """One head's (q, k, v) with the structures named above.  Keys: N(0,1) with a few fixed
    channels scaled up.  Values: N(0,1) rows times a log-normal per-token magnitude.  Queries:
    each gives one light token the logit `peak` and all tokens Gaussian noise logits, which makes
    the softmax sparse and puts its mass on tokens whose value rows are small next to the range
    of their per-channel group."""
    rng = np.random.default_rng(seed)
    gain = np.ones(channels)
    gain[rng.choice(channels, n_outlier_channels, replace=False)] = outlier_gain
    k = (rng.standard_normal((tokens, channels)) * gain).astype(np.float16)
    tok_scale = np.exp(token_scale_sigma * rng.standard_normal(tokens))
    v = (rng.standard_normal((tokens, channels)) * tok_scale[:, None]).astype(np.float16)
    light = np.argsort(tok_scale)[: tokens // 4]
    targets = rng.choice(light, n_queries, replace=False)
    kn = k[targets].astype(np.float64) / gain                     # the targets' keys without the channel gains
    # scale * q . k_target = peak for scale = 1/sqrt(channels); other tokens see peak * cos-like terms
    q_sig = peak * np.sqrt(channels) * kn / (kn * kn).sum(axis=1, keepdims=True) / gain
    q = (q_sig + noise * rng.standard_normal((n_queries, channels))).astype(np.float16)
    return q, k, v
