"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2402_02750_amd import kivi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kivi.LIB_PATH):
        from paper_2402_02750_amd.build import build_library
        build_library(verbose=False)
    return kivi.load_library()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "kivi.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(kivi_\w+)\s*\(", header, flags=re.M))
    assert declared == set(kivi.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert kivi.status_string(0) == "KIVI_OK"
    assert kivi.status_string(-1) == "KIVI_ERR_INVALID_ARG"
    assert kivi.status_string(-2) == "KIVI_ERR_UNSUPPORTED"
    assert kivi.status_string(-3) == "KIVI_ERR_WORKSPACE"
    assert kivi.status_string(-4) == "KIVI_ERR_HIP"
    assert kivi.status_string(-99) == "KIVI_ERR_UNKNOWN"


def _layout(**kw):
    base = dict(batch=2, n_q_heads=4, n_kv_heads=2, bits=2, residual=64, cap_q_tokens=256, cap_r_tokens=96)
    base.update(kw)
    return kivi.make_layout(**base)


def test_cache_sizes_and_workspace(lib):
    l = _layout()
    s = kivi.kivi_cache_sizes(l)
    units = 4
    assert s.k_codes == s.v_codes == units * 8 * 1024
    assert s.k_scale == s.k_zero == units * 8 * 128 * 2
    assert s.v_scale == s.v_zero == units * 256 * 4 * 2
    assert s.k_resid == s.v_resid == units * 96 * 128 * 2
    # one scale / zero-point pair per group: G = 128 stores a quarter of what G = 32 does
    s128 = kivi.kivi_cache_sizes(kivi.make_layout(2, 4, 2, 2, 128, 256, 384, group=128))
    assert s128.k_scale == s128.k_zero == units * 2 * 128 * 2
    assert s128.v_scale == s128.v_zero == units * 256 * 1 * 2
    assert s128.k_codes == s.k_codes
    l4 = _layout(bits=4)
    assert kivi.kivi_cache_sizes(l4).k_codes == units * 8 * 2048
    assert kivi.kivi_decode_workspace_bytes(l) >= 2 * 4 * 3 * 130 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=64), kivi.KIVI_ERR_UNSUPPORTED),
    (dict(bits=3), kivi.KIVI_ERR_UNSUPPORTED),
    (dict(group=48), kivi.KIVI_ERR_UNSUPPORTED),
    (dict(group=128, residual=64), kivi.KIVI_ERR_INVALID_ARG),  # G must divide R
    (dict(group=64, cap_q_tokens=288), kivi.KIVI_ERR_INVALID_ARG),   # capacity in whole groups
    (dict(n_q_heads=3), kivi.KIVI_ERR_INVALID_ARG),
    (dict(n_q_heads=258), kivi.KIVI_ERR_UNSUPPORTED),             # 129 query heads per kv-head (limit 128)
    (dict(residual=48), kivi.KIVI_ERR_INVALID_ARG),           # R must be divisible by G
    (dict(cap_q_tokens=100), kivi.KIVI_ERR_INVALID_ARG),
    (dict(cap_r_tokens=64), kivi.KIVI_ERR_INVALID_ARG),       # needs R + G
    (dict(batch=0), kivi.KIVI_ERR_INVALID_ARG),
    (dict(decode_path=7), kivi.KIVI_ERR_INVALID_ARG),
])
def test_bad_layouts(lib, kw, status):
    l = _layout(**kw)
    sizes = kivi.kivi_cache_sizes_t()
    assert lib.kivi_cache_sizes(ctypes.byref(l), ctypes.byref(sizes)) == status


def _fake_cache(**kw):
    """A cache whose pointers are aligned but never dereferenced (validation fails first)."""
    c = kivi.kivi_cache_t()
    for name in kivi.Cache._NAMES:
        setattr(c, name, 0x1000)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_entry_points_validate_before_launch(lib):
    l = _layout()
    good_ptr = ctypes.c_void_p(0x2000)
    out = ctypes.c_void_p(0x3000)
    # null / misaligned cache pointer
    c = _fake_cache(k_codes=0)
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, good_ptr, 1 << 30, None) \
        == kivi.KIVI_ERR_INVALID_ARG
    c = _fake_cache(v_resid=0x1004)
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, good_ptr, 1 << 30, None) \
        == kivi.KIVI_ERR_INVALID_ARG
    # empty cache, inconsistent K/V lengths
    c = _fake_cache()
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, good_ptr, 1 << 30, None) \
        == kivi.KIVI_ERR_INVALID_ARG
    c = _fake_cache(n_kq=64, n_kr=3, n_vq=64, n_vr=4)
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, good_ptr, 1 << 30, None) \
        == kivi.KIVI_ERR_INVALID_ARG
    # workspace missing / too small
    c = _fake_cache(n_kq=64, n_kr=3, n_vq=64, n_vr=3)
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, None, 0, None) \
        == kivi.KIVI_ERR_WORKSPACE
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), good_ptr, 0.1, out, good_ptr, 64, None) \
        == kivi.KIVI_ERR_WORKSPACE
    # null q
    assert lib.kivi_decode_attention(ctypes.byref(l), ctypes.byref(c), None, 0.1, out, good_ptr, 1 << 30, None) \
        == kivi.KIVI_ERR_INVALID_ARG
    # quantise: token count not a multiple of G, capacity exceeded, bad strides
    c = _fake_cache()
    f = lib.kivi_quantize_key_groups
    assert f(ctypes.byref(l), good_ptr, 128 * 64 * 2, 128 * 64, 128, 33, ctypes.byref(c), None) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), good_ptr, 128 * 64 * 2, 128 * 64, 128, 288, ctypes.byref(c), None) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), good_ptr, 128 * 64 * 2, 128 * 64, 100, 32, ctypes.byref(c), None) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), None, 128 * 64 * 2, 128 * 64, 128, 32, ctypes.byref(c), None) == kivi.KIVI_ERR_INVALID_ARG
    assert c.n_kq == 0                                   # nothing advanced on error
    g = lib.kivi_quantize_value_tokens
    assert g(ctypes.byref(l), good_ptr, 128 * 64 * 2, 128 * 64, 128, 257, ctypes.byref(c), None) == kivi.KIVI_ERR_INVALID_ARG
    # append into a full ring, unknown flush policy
    c = _fake_cache(n_kr=96, n_vr=96)
    assert lib.kivi_append_residual(ctypes.byref(l), ctypes.byref(c), good_ptr, good_ptr, None) == kivi.KIVI_ERR_INVALID_ARG
    c = _fake_cache()
    assert lib.kivi_flush_residual(ctypes.byref(l), ctypes.byref(c), 5, None, None, None) == kivi.KIVI_ERR_INVALID_ARG
    # nothing to flush: OK without any launch
    nk, nv = ctypes.c_int32(-1), ctypes.c_int32(-1)
    c = _fake_cache(n_kr=70, n_vr=70)
    assert lib.kivi_flush_residual(ctypes.byref(l), ctypes.byref(c), kivi.KIVI_FLUSH_WINDOW,
                                   ctypes.byref(nk), ctypes.byref(nv), None) == kivi.KIVI_OK
    assert (nk.value, nv.value) == (0, 0) and c.n_kr == 70


def test_decode_step_validates_before_launch(lib):
    l = _layout()
    good_ptr = ctypes.c_void_p(0x2000)
    out = ctypes.c_void_p(0x3000)
    f = lib.kivi_decode_step

    def call(c, k_new=good_ptr, v_new=good_ptr, q=good_ptr, policy=kivi.KIVI_FLUSH_WINDOW, ws=good_ptr, ws_bytes=1 << 30):
        before = bytes(c)
        st = f(ctypes.byref(l), ctypes.byref(c), k_new, v_new, q, 0.1, policy, out, ws, ws_bytes, None)
        assert bytes(c) == before, "the cache must be unchanged on an error"
        return st

    c = _fake_cache(n_kq=64, n_kr=3, n_vq=64, n_vr=3)
    assert call(c, k_new=None) == kivi.KIVI_ERR_INVALID_ARG
    assert call(c, v_new=ctypes.c_void_p(0x2004)) == kivi.KIVI_ERR_INVALID_ARG
    assert call(c, q=None) == kivi.KIVI_ERR_INVALID_ARG
    assert call(c, policy=7) == kivi.KIVI_ERR_INVALID_ARG
    assert call(c, ws=None, ws_bytes=0) == kivi.KIVI_ERR_WORKSPACE
    assert call(c, ws_bytes=64) == kivi.KIVI_ERR_WORKSPACE
    # full ring
    assert call(_fake_cache(n_kq=64, n_kr=96, n_vq=64, n_vr=96)) == kivi.KIVI_ERR_INVALID_ARG
    # the flush that this step triggers does not fit the quantised capacity (256 tokens)
    assert call(_fake_cache(n_kq=256, n_kr=95, n_vq=256, n_vr=95)) == kivi.KIVI_ERR_INVALID_ARG
    # WINDOW policy needs the symmetric split
    assert call(_fake_cache(n_kq=64, n_kr=10, n_vq=32, n_vr=42)) == kivi.KIVI_ERR_INVALID_ARG


def test_stream_probe_validates(lib):
    good = ctypes.c_void_p(0x4000)
    assert lib.kivi_stream_read_probe(None, 1024, good, None) == kivi.KIVI_ERR_INVALID_ARG
    assert lib.kivi_stream_read_probe(good, 1024, None, None) == kivi.KIVI_ERR_INVALID_ARG
    assert lib.kivi_stream_read_probe(ctypes.c_void_p(0x4008), 1024, good, None) == kivi.KIVI_ERR_INVALID_ARG
    assert lib.kivi_stream_read_probe(good, 1000, good, None) == kivi.KIVI_ERR_INVALID_ARG
    assert lib.kivi_stream_read_probe(good, 0, good, None) == kivi.KIVI_OK          # nothing to read, no launch


def test_batch_slice_and_ragged_validate(lib):
    l = _layout()
    c = _fake_cache(n_kq=64, n_kr=3, n_vq=64, n_vr=3)
    sl, sc = kivi.kivi_layout_t(), kivi.kivi_cache_t()
    f = lib.kivi_batch_slice
    assert f(ctypes.byref(l), ctypes.byref(c), -1, 1, None, ctypes.byref(sl), ctypes.byref(sc)) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), ctypes.byref(c), 0, 0, None, ctypes.byref(sl), ctypes.byref(sc)) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), ctypes.byref(c), l.batch - 1, 2, None, ctypes.byref(sl), ctypes.byref(sc)) == kivi.KIVI_ERR_INVALID_ARG
    assert f(ctypes.byref(l), ctypes.byref(c), 0, 1, None, None, ctypes.byref(sc)) == kivi.KIVI_ERR_INVALID_ARG
    # a state that does not fit the layout is refused
    bad = kivi.kivi_seq_state_t(n_kq=33, n_vq=32, n_kr=1, n_vr=2)
    assert f(ctypes.byref(l), ctypes.byref(c), 0, 1, ctypes.byref(bad), ctypes.byref(sl), ctypes.byref(sc)) == kivi.KIVI_ERR_INVALID_ARG
    # the slice: same geometry, batch nb, every array moved by b0 sequences, counters from `state`
    sizes = kivi.kivi_cache_sizes_t()
    assert lib.kivi_cache_sizes(ctypes.byref(l), ctypes.byref(sizes)) == kivi.KIVI_OK
    st = kivi.kivi_seq_state_t(n_kq=32, n_vq=32, k_r_start=5, n_kr=7, v_r_start=5, n_vr=7)
    b0 = l.batch - 1
    assert f(ctypes.byref(l), ctypes.byref(c), b0, 1, ctypes.byref(st), ctypes.byref(sl), ctypes.byref(sc)) == kivi.KIVI_OK
    assert (sl.batch, sl.n_kv_heads, sl.bits, sl.cap_q_tokens, sl.cap_r_tokens) == (
        1, l.n_kv_heads, l.bits, l.cap_q_tokens, l.cap_r_tokens)
    for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid"):
        assert getattr(sc, name) - getattr(c, name) == getattr(sizes, name) // l.batch * b0, name
    assert (sc.n_kq, sc.n_vq, sc.k_r_start, sc.n_kr, sc.v_r_start, sc.n_vr) == (32, 32, 5, 7, 5, 7)

    good = ctypes.c_void_p(0x2000)
    out = ctypes.c_void_p(0x3000)
    states = kivi.make_states(l.batch)
    step, att = lib.kivi_decode_step_ragged, lib.kivi_decode_attention_ragged
    assert step(ctypes.byref(l), ctypes.byref(c), None, good, good, good, 0.1, 0, out, good, 1 << 30, None) == kivi.KIVI_ERR_INVALID_ARG
    assert step(ctypes.byref(l), ctypes.byref(c), states, None, good, good, 0.1, 0, out, good, 1 << 30, None) == kivi.KIVI_ERR_INVALID_ARG
    assert att(ctypes.byref(l), ctypes.byref(c), None, good, 0.1, out, good, 1 << 30, None) == kivi.KIVI_ERR_INVALID_ARG
    assert att(ctypes.byref(l), ctypes.byref(c), states, None, 0.1, out, good, 1 << 30, None) == kivi.KIVI_ERR_INVALID_ARG
    # all slots empty: nothing to attend to, no launch
    assert att(ctypes.byref(l), ctypes.byref(c), states, good, 0.1, out, good, 1 << 30, None) == kivi.KIVI_OK
    # a full ring in one sequence is refused before anything is launched, states unchanged
    for b in range(l.batch):
        states[b] = kivi.kivi_seq_state_t(n_kq=64, n_vq=64, n_kr=96, n_vr=96)
    before = bytes(states)
    assert step(ctypes.byref(l), ctypes.byref(c), states, good, good, good, 0.1, 0, out, good, 1 << 30, None) == kivi.KIVI_ERR_INVALID_ARG
    assert bytes(states) == before


def test_decode_plan(lib):
    """kivi_decode_plan: family, launches and splits for a cache state, without any launch."""
    def plan(batch, hq, hkv, bits, n_q, n_r, path=kivi.KIVI_DECODE_AUTO, n_vq=None, n_vr=None):
        l = kivi.make_layout(batch, hq, hkv, bits, 128, max(n_q, 32) + 64, 192, decode_path=path)
        c = _fake_cache(n_kq=n_q, n_kr=n_r, n_vq=n_q if n_vq is None else n_vq, n_vr=n_r if n_vr is None else n_vr)
        return kivi.kivi_decode_plan(l, c)

    # one (batch, kv-head) unit per resident workgroup: the single launch, 16-tile chunks, one fp16-row chunk
    p = plan(16, 32, 32, 2, 3968, 128)
    assert (p.family, p.launches) == (kivi.KIVI_DECODE_MFMA, 1)
    assert (p.splits_quantised, p.tiles_per_split_quantised, p.splits_fp16, p.tiles_per_split_fp16) == (8, 16, 1, 4)
    # four units per workgroup: fp16 rows in a launch of their own, one part per unit
    p = plan(64, 32, 32, 2, 1920, 150)
    assert (p.family, p.launches, p.splits_fp16, p.tiles_per_split_fp16) == (kivi.KIVI_DECODE_MFMA, 2, 1, 5)
    assert plan(64, 32, 32, 2, 1920, 150, path=kivi.KIVI_DECODE_MFMA_ONE).launches == 1
    assert plan(16, 32, 32, 2, 3968, 128, path=kivi.KIVI_DECODE_MFMA_TWO).launches == 2
    # 6 or 8 query heads per kv-head and few chunks per workgroup: the halves of every group as units of their own
    assert plan(1, 64, 8, 2, 3968, 128).units_per_kv_head == 4      # 8 units x 12 chunks, 2 bits: quarters
    assert plan(4, 64, 8, 2, 3968, 128).units_per_kv_head == 2      # 32 units: halves
    assert plan(1, 64, 8, 4, 3968, 128).units_per_kv_head == 2      # 4 bits: halves
    assert plan(1, 48, 8, 4, 3968, 128).units_per_kv_head == 2
    assert plan(1, 56, 8, 2, 3968, 128).units_per_kv_head == 1      # 7 heads do not halve
    assert plan(1, 32, 8, 2, 3968, 128).units_per_kv_head == 2      # 4 heads at 2 bits: 2 + 2
    assert plan(1, 32, 8, 4, 3968, 128).units_per_kv_head == 1      # ... not at 4 bits
    assert plan(16, 32, 8, 2, 992, 128).units_per_kv_head == 1      # ... not from 128 units on
    assert plan(1, 16, 8, 2, 3968, 128).units_per_kv_head == 1      # 2 heads: nothing to split
    assert plan(16, 64, 8, 2, 16256, 128).units_per_kv_head == 1    # 128 units x 36 chunks: too many at 2 bits
    assert plan(32, 64, 8, 2, 3968, 128, path=kivi.KIVI_DECODE_MFMA_TWO).units_per_kv_head == 1
    assert plan(1, 64, 8, 2, 3968, 128, path=kivi.KIVI_DECODE_VALU).units_per_kv_head == 1
    # two launches need both parts and K and V split at the same token
    assert plan(64, 32, 32, 2, 0, 100, path=kivi.KIVI_DECODE_MFMA_TWO).launches == 1
    assert plan(64, 32, 32, 2, 1920, 0, path=kivi.KIVI_DECODE_MFMA_TWO).launches == 1
    assert plan(64, 32, 32, 2, 1920, 150, n_vq=1984, n_vr=86).launches == 1
    # 4 or more query heads per kv-head, fewer units than workgroups: two launches once there is
    # enough work overall and enough fp16 rows, one launch below that and for a one-tile window
    assert plan(16, 64, 8, 4, 4096, 128).launches == 2       # 128 units x 132 tiles, 512 fp16 tiles
    assert plan(8, 64, 8, 4, 4096, 128).launches == 1        # 64 units: 256 fp16 tiles are too few
    assert plan(1, 64, 8, 4, 4096, 128).launches == 1        # 8 units: too little work
    assert plan(32, 64, 8, 2, 3968, 128).launches == 2       # 2-bit, 8 heads: 256 units x 4 fp16 tiles
    assert plan(8, 64, 8, 2, 3968, 128).launches == 1        # ... 64 units x 4 fp16 tiles: one launch
    assert plan(32, 64, 8, 2, 4064, 32).launches == 1        # a single tile of fp16 rows
    assert plan(8, 32, 8, 2, 3968, 128).launches == 1        # 2-bit, 4 heads: 64 units x 128 tiles is little work
    assert plan(48, 32, 8, 2, 3968, 128).launches == 2
    # 1 head per kv-head: only by units per workgroup -- more than one, or between a half and one
    # (workgroups straddle two units) in a launch long enough to carry a second one
    assert plan(32, 8, 8, 2, 3968, 128).launches == 1        # 256 units: two workgroups per unit
    assert plan(48, 8, 8, 2, 3968, 128).launches == 2        # 384 units x 128 tiles
    assert plan(48, 8, 8, 2, 992, 128).launches == 1         # 384 units x 35 tiles: too short
    assert plan(2, 64, 8, 2, 4096, 128).launches == 1
    # vector-ALU family: decode + merge
    p = plan(16, 32, 32, 2, 3968, 128, path=kivi.KIVI_DECODE_VALU)
    assert (p.family, p.launches) == (kivi.KIVI_DECODE_VALU, 2)
    # more than 8 query heads per kv-head (multi-query attention): runs of 4 heads as units of one
    # launch in the single-launch form; one pass per 8 heads in the two-launch form and the vector-ALU family
    p = plan(16, 71, 1, 2, 3968, 128)
    assert (p.launches, p.units_per_kv_head) == (1, 18)
    p = plan(4, 128, 8, 4, 3968, 128)
    assert (p.launches, p.units_per_kv_head) == (1, 4)
    p = plan(16, 71, 1, 2, 3968, 128, path=kivi.KIVI_DECODE_MFMA_TWO)
    assert (p.launches, p.units_per_kv_head) == (18, 1)
    p = plan(16, 71, 1, 2, 3968, 128, path=kivi.KIVI_DECODE_VALU)
    assert (p.launches, p.units_per_kv_head) == (10, 1)
    bad = kivi.kivi_decode_plan_t()
    l = _layout()
    assert lib.kivi_decode_plan(ctypes.byref(l), None, ctypes.byref(bad)) == kivi.KIVI_ERR_INVALID_ARG
    assert lib.kivi_decode_plan(ctypes.byref(l), ctypes.byref(_fake_cache()), None) == kivi.KIVI_ERR_INVALID_ARG


def test_decode_launches_ragged(lib):
    """kivi_decode_launches_ragged: a batch of different lengths goes through one pair of launches when
    every sequence splits K and V alike and has fp16 rows; run by run otherwise."""
    l = kivi.make_layout(4, 8, 2, 2, 128, 4096, 192)
    st = kivi.make_states(4)
    for b, (nq, nr) in enumerate([(0, 50), (992, 130), (2048, 159), (64, 128)]):
        st[b] = kivi.kivi_seq_state_t(nq, nq, 0, nr, 0, nr)
    assert kivi.kivi_decode_launches_ragged(l, st) == 2
    # 16 query heads per kv-head: two groups of 8, a pair of launches each
    l16 = kivi.make_layout(4, 32, 2, 2, 128, 4096, 192)
    assert kivi.kivi_decode_launches_ragged(l16, st) == 4
    # an empty slot, or K and V split differently (Algorithm 1's policy): run by run
    st[0] = kivi.kivi_seq_state_t()
    assert kivi.kivi_decode_launches_ragged(l, st) >= 3
    st[0] = kivi.kivi_seq_state_t(128, 100, 0, 10, 0, 38)
    assert kivi.kivi_decode_launches_ragged(l, st) >= 4
    # the vector-ALU family: decode + merge per run
    lv = kivi.make_layout(4, 8, 2, 2, 128, 4096, 192, decode_path=kivi.KIVI_DECODE_VALU)
    st[0] = kivi.kivi_seq_state_t(0, 0, 0, 50, 0, 50)
    assert kivi.kivi_decode_launches_ragged(lv, st) == 8
    bad = kivi.make_states(4)
    bad[1] = kivi.kivi_seq_state_t(32, 0, 0, 5, 0, 5)
    n = ctypes.c_int32(0)
    assert lib.kivi_decode_launches_ragged(ctypes.byref(l), bad, ctypes.byref(n)) == kivi.KIVI_ERR_INVALID_ARG
