"""Seeded synthetic workloads for the KIVI decode-attention path.

This module only *describes* workloads and draws random tensors.  It holds none of the
method's arithmetic (no quantisation, no packing, no attention): both the CPU oracle's tests
and the HIP path's tests/bench read their inputs from here, and nothing else is shared
between the two.

The tensors stand in for the key/value activations of the Llama-2-7B / Llama-2-13B /
Mistral-7B layers the paper evaluates (Section 4.1; Appendix D for the grouped-query models):
keys carry a few fixed large-magnitude channels, values have no outlier pattern (Section 3.2,
Figure 2).  The real activations need model weights and datasets, which are not available.

Recipe (one kv-head at a time, so a test can regenerate any single head):
  rng   = numpy Generator(PCG64) seeded with [seed, stream, b, h]   (stream: 0 = K, 1 = V, 2 = q)
  K     = fp16( N(0,1) fp32 * channel_gain[h] )    gain = 1 except `n_outlier` channels per kv-head
  V, q  = fp16( N(0,1) fp32 )
  channel_gain[h] is drawn from Generator([seed, 3, h]): the outlier channel indices (without
  replacement) and their factors (a constant, or U(lo, hi)); it is shared by all batch entries
  and all tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int          # tokens in the cache when decode attention runs (single-step configs)
    bits: int
    group: int
    residual: int
    n_outlier: int
    outlier_lo: float
    outlier_hi: float
    seed: int
    # streaming workload only
    prompt: int = 0       # prefill tokens (0: single-step workload)
    decode_steps: int = 0

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def q_per_kv(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def split_single_step(self) -> Tuple[int, int]:
        """(n_q, n_r) for a single decode step: the most recent `residual` tokens stay fp16."""
        n_r = min(self.residual, self.context)
        n_q = self.context - n_r
        assert n_q % self.group == 0
        return n_q, n_r

    def packed_bytes_per_token_head(self) -> int:
        """Codes + scale + zero-point of one cached token of one kv-head, K and V together."""
        d, g, b = self.head_dim, self.group, self.bits
        return 2 * (d * b // 8 + (d // g) * 4)

    def algorithmic_bytes(self, n_q: int, n_r: int) -> dict:
        """Bytes one decode-attention call must move (per call, all heads)."""
        units = self.batch * self.n_kv_heads
        packed = units * n_q * self.packed_bytes_per_token_head()
        resid = units * n_r * self.head_dim * 2 * 2
        qo = self.batch * self.n_q_heads * self.head_dim * (2 + 4)
        return {"packed": packed, "residual": resid, "q_out": qo, "all": packed + resid + qo}


_BASE_SEED = 20240202

CONFIGS = {
    # benchmark configuration 1: tiny single decode step
    "tiny": Workload("tiny", 1, 4, 4, 128, 1024, 2, 32, 32, 4, 10.0, 10.0, _BASE_SEED + 1),
    # benchmark configuration 2: Llama-2-7B-shaped layer (the configuration the metric is quoted on)
    "llama7b": Workload("llama7b", 16, 32, 32, 128, 4096, 2, 32, 128, 6, 8.0, 15.0, _BASE_SEED + 2),
    # benchmark configuration 3: streaming, batch 64, prompt 2048 + 256 decode steps
    "stream": Workload("stream", 64, 32, 32, 128, 2048, 2, 32, 128, 6, 8.0, 15.0, _BASE_SEED + 3,
                       prompt=2048, decode_steps=256),
    # benchmark configuration 4: 4-bit on a Llama-2-13B-shaped layer
    "llama13b_4bit": Workload("llama13b_4bit", 8, 40, 40, 128, 8192, 4, 32, 128, 8, 8.0, 15.0,
                              _BASE_SEED + 4),
    # benchmark configuration 5: grouped-query long context, Mistral-7B-shaped
    "mistral_gqa": Workload("mistral_gqa", 4, 32, 8, 128, 32768, 2, 32, 128, 6, 8.0, 15.0,
                            _BASE_SEED + 5),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller/larger variant of a workload (for parity cases the oracle finishes quickly)."""
    return replace(w, **kw)


def channel_gain(w: Workload, h: int) -> np.ndarray:
    """fp32 [head_dim] per-channel gain of kv-head h: 1 except the outlier channels."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 3, h]))
    gain = np.ones(w.head_dim, dtype=np.float32)
    idx = rng.choice(w.head_dim, size=w.n_outlier, replace=False)
    if w.outlier_lo == w.outlier_hi:
        fac = np.full(w.n_outlier, w.outlier_lo, dtype=np.float32)
    else:
        fac = rng.uniform(w.outlier_lo, w.outlier_hi, size=w.n_outlier).astype(np.float32)
    gain[idx] = fac
    return gain


def keys_head(w: Workload, b: int, h: int, n_tokens: int) -> np.ndarray:
    """fp16 [n_tokens, head_dim] keys of batch entry b, kv-head h (token-major)."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 0, b, h]))
    x = rng.standard_normal((n_tokens, w.head_dim), dtype=np.float32)
    x *= channel_gain(w, h)[None, :]
    return x.astype(np.float16)


def values_head(w: Workload, b: int, h: int, n_tokens: int) -> np.ndarray:
    """fp16 [n_tokens, head_dim] values of batch entry b, kv-head h."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 1, b, h]))
    return rng.standard_normal((n_tokens, w.head_dim), dtype=np.float32).astype(np.float16)


def query_head(w: Workload, b: int, hq: int, step: int = 0) -> np.ndarray:
    """fp16 [head_dim] query of batch entry b, query head hq, at decode step `step`."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 2, b, hq, step]))
    return rng.standard_normal(w.head_dim, dtype=np.float32).astype(np.float16)


def keys(w: Workload, n_tokens: int) -> np.ndarray:
    """fp16 [batch, n_kv_heads, n_tokens, head_dim]."""
    out = np.empty((w.batch, w.n_kv_heads, n_tokens, w.head_dim), dtype=np.float16)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            out[b, h] = keys_head(w, b, h, n_tokens)
    return out


def values(w: Workload, n_tokens: int) -> np.ndarray:
    out = np.empty((w.batch, w.n_kv_heads, n_tokens, w.head_dim), dtype=np.float16)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            out[b, h] = values_head(w, b, h, n_tokens)
    return out


def queries(w: Workload, step: int = 0) -> np.ndarray:
    """fp16 [batch, n_q_heads, head_dim]."""
    out = np.empty((w.batch, w.n_q_heads, w.head_dim), dtype=np.float16)
    for b in range(w.batch):
        for hq in range(w.n_q_heads):
            out[b, hq] = query_head(w, b, hq, step)
    return out


ADVERSARIAL_KINDS = ("normal", "offset", "lattice", "lattice_offset", "tiny", "half_integers", "wide")


def adversarial_values(kind: str, seed: int, shape) -> np.ndarray:
    """fp16 inputs that stress a group-wise quantiser: plain normal data; a large offset with a small
    spread (|min / scale| large); values on coarse lattices, which put many quotients exactly on or
    next to rounding ties; ranges so small that the fp16 scale is subnormal; ranges near the top of
    fp16.  Seeded; no arithmetic of the method in here."""
    rng = np.random.Generator(np.random.PCG64([seed, ADVERSARIAL_KINDS.index(kind)]))
    if kind == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
    elif kind == "offset":
        x = 100.0 + 0.05 * rng.standard_normal(shape, dtype=np.float32)
    elif kind == "lattice":
        x = rng.integers(-12, 13, size=shape).astype(np.float32) / 8.0
    elif kind == "lattice_offset":
        x = 3.0 + rng.integers(0, 7, size=shape).astype(np.float32) / 2.0
    elif kind == "tiny":
        x = rng.integers(0, 9, size=shape).astype(np.float32) * np.float32(2.0 ** -24)
    elif kind == "half_integers":
        x = rng.integers(0, 31, size=shape).astype(np.float32) * 0.5
    elif kind == "wide":
        x = rng.standard_normal(shape, dtype=np.float32) * 3000.0
    else:
        raise ValueError(kind)
    return x.astype(np.float16)
