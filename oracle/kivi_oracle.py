"""CPU oracle for the KIVI decode-attention path.  TEST INFRASTRUCTURE ONLY.

This file is a plain, slow, deliberately unoptimised statement of what the path computes,
written from the paper (KIVI, arXiv 2402.02750).  Only tests, the smoke check and the
benchmark's `cpu_baseline` leg may import it.  It shares no code with the HIP library and
the HIP library never calls it.

What follows the paper, and where:
  * round-to-nearest asymmetric B-bit quantisation, zero-point = min, scale = (max-min)/(2^B-1)
    -- Section 3.1 (unnumbered equation) and the sentence after Table 1;
  * key cache grouped per channel over G consecutive tokens, value cache per token over G
    consecutive channels -- Section 3.3 "Algorithm", Algorithm 1 (KeyQuant, GroupQuant calls);
  * the grouped (quantised) / residual (fp16) split of the cache and the tiled logits
    A = Concat(t_Q Q(X_Kg)^T, t_Q X_Kr^T) -- Section 3.3, Equation 4;
  * softmax over the concatenated logits, output A_g Q(X_Vg) + A_r X_Vr -- Equation 1 and
    Algorithm 1 (Decoding);
  * Prefill / Decoding / KeyQuant cache updates -- Algorithm 1 (policy "alg1").

Readings taken where the paper is silent (all of them are part of the contract both this
oracle and the HIP library implement independently):
  * the rounding is round-half-to-even; scale and zero-point are stored as fp16, and the
    *stored* (rounded) scale is the one used to encode;
  * (x - z) / s is evaluated in IEEE fp32 (subtract, then a true division); codes are clamped
    to [0, 2^B-1]; a group whose stored scale is 0 gets all-zero codes (so x' = z);
  * a softmax scale (1/sqrt(head_dim) in the workloads) multiplies the logits; the paper's
    equations drop it together with the head structure;
  * grouped-query attention: query head j reads kv-head j // (n_q_heads // n_kv_heads);
  * policy "window" (what the benchmark configurations describe): after an append, while the
    fp16 window holds at least R+G tokens its oldest G tokens are quantised (one key group,
    G value tokens), so the most recent R tokens are always fp16;
  * the physical packing of the codes is not the paper's business; `code_slot` below states
    the layout the library's ABI fixes.

All floating-point work is fp64 except the quantiser's (x - z) / s, which is fp32 by contract.

Parity pins (tests/test_oracle_*.py): closed-form worked examples and tie cases, the s/2 error
bound, exactness on constant groups, nearest-level optimality checked in exact rational
arithmetic, hand-derived packed bytes, reduction to textbook softmax attention when nothing is
quantised, convergence to brute-force fp32 attention at B=16/R=0, uniform / one-hot special
cases, permutation invariance, streaming == batch.  The paper's accuracy tables depend on
model weights and datasets: parity unpinned for those (only the ordering of Table 2's
per-channel vs per-token errors is checked on synthetic outlier data).
"""
from __future__ import annotations

import numpy as np

TILE_TOKENS = 32  # tokens per packed code tile (the ABI packs 32 x 128 codes per tile for every group size G)
HEAD_DIM = 128    # channels per packed code tile


# --------------------------------------------------------------------------------------
# Section 3.1: B-bit round-to-nearest quantisation of one group
# --------------------------------------------------------------------------------------
def quantize_groups(x: np.ndarray, bits: int, scale_dtype=np.float16):
    """Quantise every last-axis vector of fp16 array `x` as one group.

    Q(X) = round((X - z) / s),  z = min X,  s = (max X - min X) / (2^B - 1)   (Section 3.1).
    Returns (codes uint16 [..., G], scale `scale_dtype` [...], zero fp16 [...]).
    """
    assert x.dtype == np.float16
    x32 = x.astype(np.float32)
    lo = x32.min(axis=-1)
    hi = x32.max(axis=-1)
    levels = np.float32(2 ** bits - 1)
    s_stored = ((hi - lo) / levels).astype(scale_dtype)          # fp32 arithmetic, then stored
    z_stored = lo.astype(np.float16)                             # exact: lo is an fp16 value
    s32 = s_stored.astype(np.float32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = (x32 - lo[..., None]) / s32                      # fp32 subtract, fp32 divide
    codes = np.clip(np.rint(ratio), 0.0, levels)                 # rint = round-half-to-even
    codes = np.where(s32 == 0.0, 0.0, codes)
    return codes.astype(np.uint16), s_stored, z_stored


def dequantize_groups(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """X' = Q(X) * s + z  (Section 3.1), in fp64."""
    return codes.astype(np.float64) * scale.astype(np.float64)[..., None] \
        + zero.astype(np.float64)[..., None]


# --------------------------------------------------------------------------------------
# Section 3.3: key cache per channel (groups of G tokens), value cache per token
# --------------------------------------------------------------------------------------
def quantize_key(k: np.ndarray, bits: int, group: int, scale_dtype=np.float16):
    """k fp16 [..., n, D], n % G == 0.  Each (group of G tokens, channel) is one quantisation
    group (Algorithm 1, KeyQuant: GroupQuant(X_Kg, dim=channel)).

    Returns codes uint16 [..., n, D], scale/zero [..., n/G, D].
    """
    n, d = k.shape[-2:]
    assert n % group == 0
    lead = k.shape[:-2]
    kg = k.reshape(*lead, n // group, group, d)
    kg = np.swapaxes(kg, -1, -2)                                  # [..., n/G, D, G]
    codes, s, z = quantize_groups(np.ascontiguousarray(kg), bits, scale_dtype)
    codes = np.swapaxes(codes, -1, -2).reshape(*lead, n, d)
    return codes, s, z


def quantize_value(v: np.ndarray, bits: int, group: int, scale_dtype=np.float16):
    """v fp16 [..., n, D].  Each (token, group of G channels) is one quantisation group
    (Algorithm 1: GroupQuant(X_Vg, dim=token, numGroup=d//G)).

    Returns codes uint16 [..., n, D], scale/zero [..., n, D/G].
    """
    n, d = v.shape[-2:]
    assert d % group == 0
    lead = v.shape[:-2]
    vg = v.reshape(*lead, n, d // group, group)
    codes, s, z = quantize_groups(vg, bits, scale_dtype)
    return codes.reshape(*lead, n, d), s, z


def dequantize_key(codes, scale, zero, group: int) -> np.ndarray:
    """fp64 [..., n, D] from key codes [..., n, D] and scale/zero [..., n/G, D]."""
    s = np.repeat(scale.astype(np.float64), group, axis=-2)
    z = np.repeat(zero.astype(np.float64), group, axis=-2)
    return codes.astype(np.float64) * s + z


def dequantize_value(codes, scale, zero, group: int) -> np.ndarray:
    """fp64 [..., n, D] from value codes [..., n, D] and scale/zero [..., n, D/G]."""
    s = np.repeat(scale.astype(np.float64), group, axis=-1)
    z = np.repeat(zero.astype(np.float64), group, axis=-1)
    return codes.astype(np.float64) * s + z


# --------------------------------------------------------------------------------------
# ABI layout of the packed codes (ours to define; the paper only asks for a
# "hardware-friendly implementation", Section 3.3 "System Support")
# --------------------------------------------------------------------------------------
def code_slot(u, lane, e, bits: int):
    """(word index, bit offset) inside one 32-token x 128-channel code tile.

    A tile is addressed by u in [0,8), lane in [0,64), e in [0,8):
      key tile   : token   = (u & 1) * 16 + (lane & 15),  channel = (u >> 1) * 32 + (lane >> 4) * 8 + e
      value tile : channel = u * 16 + (lane & 15),        token   = (lane >> 4) * 8 + e
    B = 2 (256 words):  word = lane*4 + (u >> 1)
                        bit  = (e & 1)*16 + 2*((u & 1)*4 + (e >> 1))
    B = 4 (512 words):  i    = (u >> 1)*2 + (e >> 2)
                        word = (i >> 2)*256 + lane*4 + (i & 3)
                        bit  = (e & 1)*16 + 4*((u & 1)*2 + ((e >> 1) & 1))
    Words are little-endian uint32.
    """
    if bits == 2:
        word = lane * 4 + (u >> 1)
        bit = (e & 1) * 16 + 2 * ((u & 1) * 4 + (e >> 1))
    elif bits == 4:
        i = (u >> 1) * 2 + (e >> 2)
        word = (i >> 2) * 256 + lane * 4 + (i & 3)
        bit = (e & 1) * 16 + 4 * ((u & 1) * 2 + ((e >> 1) & 1))
    else:
        raise ValueError("packed layout is defined for 2 and 4 bits")
    return word, bit


def _key_ule(t, c):
    u = (c >> 5) * 2 + (t >> 4)
    lane = ((c >> 3) & 3) * 16 + (t & 15)
    e = c & 7
    return u, lane, e


def _value_ule(t, c):
    u = c >> 4
    lane = (t >> 3) * 16 + (c & 15)
    e = t & 7
    return u, lane, e


def _pack_tiles(codes: np.ndarray, bits: int, ule) -> np.ndarray:
    n, d = codes.shape[-2:]
    assert d == HEAD_DIM and n % TILE_TOKENS == 0
    lead = codes.shape[:-2]
    words_per_tile = TILE_TOKENS * HEAD_DIM * bits // 32
    tiles = codes.reshape(-1, n // TILE_TOKENS, TILE_TOKENS, d).astype(np.uint32)
    out = np.zeros((tiles.shape[0], tiles.shape[1], words_per_tile), dtype=np.uint32)
    for t in range(TILE_TOKENS):
        for c in range(d):
            word, bit = code_slot(*ule(t, c), bits)
            out[:, :, word] |= tiles[:, :, t, c] << np.uint32(bit)
    return out.reshape(*lead, n // TILE_TOKENS, words_per_tile)


def _unpack_tiles(words: np.ndarray, bits: int, ule) -> np.ndarray:
    lead = words.shape[:-2]
    n_tiles = words.shape[-2]
    w = words.reshape(-1, n_tiles, words.shape[-1])
    out = np.zeros((w.shape[0], n_tiles, TILE_TOKENS, HEAD_DIM), dtype=np.uint16)
    mask = np.uint32(2 ** bits - 1)
    for t in range(TILE_TOKENS):
        for c in range(HEAD_DIM):
            word, bit = code_slot(*ule(t, c), bits)
            out[:, :, t, c] = (w[:, :, word] >> np.uint32(bit)) & mask
    return out.reshape(*lead, n_tiles * TILE_TOKENS, HEAD_DIM)


def pack_key_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes [..., n, 128] -> uint32 [..., n/32, 32*128*B/32] in the key-tile layout."""
    return _pack_tiles(codes, bits, _key_ule)


def unpack_key_codes(words: np.ndarray, bits: int) -> np.ndarray:
    return _unpack_tiles(words, bits, _key_ule)


def pack_value_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes [..., n, 128] -> uint32 [..., n/32, 32*128*B/32] in the value-tile layout."""
    return _pack_tiles(codes, bits, _value_ule)


def unpack_value_codes(words: np.ndarray, bits: int) -> np.ndarray:
    return _unpack_tiles(words, bits, _value_ule)


# --------------------------------------------------------------------------------------
# Equations 1 and 4, Algorithm 1 (Decoding): attention over the mixed-precision cache
# --------------------------------------------------------------------------------------
def softmax(a: np.ndarray) -> np.ndarray:
    """Max-subtracted softmax over the last axis, fp64."""
    a = a - a.max(axis=-1, keepdims=True)
    e = np.exp(a)
    return e / e.sum(axis=-1, keepdims=True)


def decode_attention(q, k_quant, k_resid, v_quant, v_resid, group: int, softmax_scale: float):
    """One decode step's attention output, fp64 [b, H_q, D].

    q        fp16 [b, H_q, D]
    k_quant  (codes [b, H_kv, n_kq, D], scale [b, H_kv, n_kq/G, D], zero same)   -- Q(X_Kg)
    k_resid  fp16 [b, H_kv, n_kr, D]                                              -- X_Kr
    v_quant  (codes [b, H_kv, n_vq, D], scale [b, H_kv, n_vq, D/G], zero same)   -- Q(X_Vg)
    v_resid  fp16 [b, H_kv, n_vr, D]                                              -- X_Vr
    with n_kq + n_kr == n_vq + n_vr (the K and V splits may differ, Algorithm 1).

    A   = Concat(t_Q Q(X_Kg)^T, t_Q X_Kr^T) * softmax_scale            (Equation 4)
    t_O = Softmax(A)[:n_vq] Q(X_Vg) + Softmax(A)[n_vq:] X_Vr            (Algorithm 1, Decoding)
    """
    b, hq, d = q.shape
    hkv = k_resid.shape[1]
    rep = hq // hkv
    out = np.empty((b, hq, d), dtype=np.float64)
    for bi in range(b):
        for h in range(hkv):                       # one kv-head at a time keeps the fp64 copy small
            kq = dequantize_key(*(x[bi, h] for x in k_quant), group)
            vq = dequantize_value(*(x[bi, h] for x in v_quant), group)
            k_all = np.concatenate([kq, k_resid[bi, h].astype(np.float64)], axis=0)   # [L, D]
            v_all = np.concatenate([vq, v_resid[bi, h].astype(np.float64)], axis=0)
            assert k_all.shape[0] == v_all.shape[0]
            for j in range(h * rep, (h + 1) * rep):
                a = softmax_scale * (k_all @ q[bi, j].astype(np.float64))
                p = softmax(a)
                out[bi, j] = p @ v_all
    return out


def attention_logits(q, k_quant, k_resid, group: int, softmax_scale: float) -> np.ndarray:
    """The scaled logits A of Equation 4, fp64 [b, H_q, L] (exposed for tests)."""
    b, hq, d = q.shape
    hkv = k_resid.shape[1]
    rep = hq // hkv
    kq = dequantize_key(*k_quant, group)
    k_all = np.concatenate([kq, k_resid.astype(np.float64)], axis=-2)
    out = np.empty((b, hq, k_all.shape[-2]), dtype=np.float64)
    for bi in range(b):
        for j in range(hq):
            out[bi, j] = softmax_scale * (k_all[bi, j // rep] @ q[bi, j].astype(np.float64))
    return out


# --------------------------------------------------------------------------------------
# Algorithm 1: the streaming cache (Prefill / Decoding / KeyQuant)
# --------------------------------------------------------------------------------------
class StreamingCache:
    """The 4-tuple cache (Q(X_Kg), X_Kr, Q(X_Vg), X_Vr) of Algorithm 1 for a [b, H_kv] batch.

    policy "alg1"   -- Algorithm 1 literally: prefill keeps l % R key tokens and R value tokens
                       in fp16; a decode step quantises the whole key residual when it reaches
                       R tokens, and the oldest value tokens once more than R are held.
    policy "window" -- K and V split alike; the oldest G residual tokens are quantised whenever
                       the window holds >= R + G tokens (the most recent R tokens stay fp16).
    """

    def __init__(self, batch, n_kv_heads, head_dim, bits, group, residual, policy="window",
                 scale_dtype=np.float16):
        assert residual % group == 0, "R must be divisible by G (Section 3.3)"
        assert policy in ("window", "alg1")
        self.bits, self.group, self.residual, self.policy = bits, group, residual, policy
        self.scale_dtype = scale_dtype
        lead = (batch, n_kv_heads)
        d = head_dim
        self.k_codes = np.zeros(lead + (0, d), np.uint16)
        self.k_scale = np.zeros(lead + (0, d), scale_dtype)
        self.k_zero = np.zeros(lead + (0, d), np.float16)
        self.v_codes = np.zeros(lead + (0, d), np.uint16)
        self.v_scale = np.zeros(lead + (0, d // group), scale_dtype)
        self.v_zero = np.zeros(lead + (0, d // group), np.float16)
        self.k_resid = np.zeros(lead + (0, d), np.float16)
        self.v_resid = np.zeros(lead + (0, d), np.float16)

    # sizes
    @property
    def n_kq(self): return self.k_codes.shape[2]
    @property
    def n_vq(self): return self.v_codes.shape[2]
    @property
    def n_kr(self): return self.k_resid.shape[2]
    @property
    def n_vr(self): return self.v_resid.shape[2]
    @property
    def length(self): return self.n_kq + self.n_kr

    def _quantize_oldest_keys(self, n):
        if n == 0:
            return
        c, s, z = quantize_key(self.k_resid[:, :, :n], self.bits, self.group, self.scale_dtype)
        self.k_codes = np.concatenate([self.k_codes, c], axis=2)
        self.k_scale = np.concatenate([self.k_scale, s], axis=2)
        self.k_zero = np.concatenate([self.k_zero, z], axis=2)
        self.k_resid = self.k_resid[:, :, n:]

    def _quantize_oldest_values(self, n):
        if n == 0:
            return
        c, s, z = quantize_value(self.v_resid[:, :, :n], self.bits, self.group, self.scale_dtype)
        self.v_codes = np.concatenate([self.v_codes, c], axis=2)
        self.v_scale = np.concatenate([self.v_scale, s], axis=2)
        self.v_zero = np.concatenate([self.v_zero, z], axis=2)
        self.v_resid = self.v_resid[:, :, n:]

    def prefill(self, k, v):
        """Algorithm 1, Prefill (the projections X W_K, X W_V are the caller's)."""
        assert self.length == 0
        l = k.shape[2]
        self.k_resid = np.array(k, dtype=np.float16)
        self.v_resid = np.array(v, dtype=np.float16)
        G, R = self.group, self.residual
        if self.policy == "alg1":
            self._quantize_oldest_values(max(l - R, 0))      # X_Vg = X_V[:l-R]
            self._quantize_oldest_keys(l - l % R)            # KeyQuant: r = l % R
        else:
            n = max(l - R, 0) // G * G
            self._quantize_oldest_keys(n)
            self._quantize_oldest_values(n)

    def append(self, k_new, v_new):
        """Algorithm 1, Decoding: concatenate t_K, t_V to the residual parts, then flush."""
        self.k_resid = np.concatenate([self.k_resid, k_new[:, :, None, :]], axis=2)
        self.v_resid = np.concatenate([self.v_resid, v_new[:, :, None, :]], axis=2)
        return self.flush()

    def flush(self):
        """Returns (key tokens quantised, value tokens quantised) by this call."""
        G, R = self.group, self.residual
        nk = nv = 0
        if self.policy == "alg1":
            if self.n_kr == R:
                nk = R
            if self.n_vr > R:
                nv = self.n_vr - R
        else:
            while self.n_kr - nk >= R + G:
                nk += G
            nv = nk
        self._quantize_oldest_keys(nk)
        self._quantize_oldest_values(nv)
        return nk, nv

    def attention(self, q, softmax_scale):
        return decode_attention(q, (self.k_codes, self.k_scale, self.k_zero), self.k_resid,
                                (self.v_codes, self.v_scale, self.v_zero), self.v_resid,
                                self.group, softmax_scale)
