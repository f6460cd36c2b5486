"""Pins for the oracle's packer against the written ABI layout (hand-evaluated slots)."""
import os

import numpy as np
import pytest

from oracle import kivi_oracle as ko


def _rows(golden_dir):
    out = []
    with open(os.path.join(golden_dir, "layout_golden.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split("|")
            kind, bits, t, c, code = lhs.split()
            widx, wval = rhs.split()
            out.append((kind, int(bits), int(t), int(c), int(code), int(widx), int(wval, 16)))
    return out


def test_hand_evaluated_slots(golden_dir):
    rows = _rows(golden_dir)
    assert len(rows) >= 12
    for kind, bits, t, c, code, widx, wval in rows:
        codes = np.zeros((32, 128), np.uint16)
        codes[t, c] = code
        pack = ko.pack_key_codes if kind == "key" else ko.pack_value_codes
        words = pack(codes, bits)
        assert words.shape == (1, 32 * 128 * bits // 32)
        nz = np.nonzero(words[0])[0]
        assert nz.tolist() == [widx], (kind, bits, t, c)
        assert int(words[0, widx]) == wval, (kind, bits, t, c)


@pytest.mark.parametrize("bits", [2, 4])
def test_slots_are_a_bijection(bits):
    """Every (token, channel) gets its own B bits: packing all-ones codes fills every bit, and
    packing any single code never collides with another."""
    full = np.full((32, 128), 2 ** bits - 1, np.uint16)
    for pack in (ko.pack_key_codes, ko.pack_value_codes):
        w = pack(full, bits)
        assert (w == 0xFFFFFFFF).all()
    seen_k, seen_v = set(), set()
    for t in range(32):
        for c in range(128):
            seen_k.add(ko.code_slot(*ko._key_ule(t, c), bits))
            seen_v.add(ko.code_slot(*ko._value_ule(t, c), bits))
    assert len(seen_k) == len(seen_v) == 32 * 128


@pytest.mark.parametrize("bits", [2, 4])
def test_round_trip(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2 ** bits, size=(2, 3, 96, 128)).astype(np.uint16)
    wk = ko.pack_key_codes(codes, bits)
    wv = ko.pack_value_codes(codes, bits)
    assert wk.shape == (2, 3, 3, 32 * 128 * bits // 32) and wk.dtype == np.uint32
    assert (ko.unpack_key_codes(wk, bits) == codes).all()
    assert (ko.unpack_value_codes(wv, bits) == codes).all()
    assert not (wk == wv).all()          # the two tile layouts differ


def test_lane_fragment_property_2bit():
    """What the layout is for: the 16 bytes lane l owns in a 2-bit key tile hold, in word ks,
    the codes of tokens {l%16, l%16+16} x channels ks*32 + (l/16)*8 + [0,8); masking the word
    with 0x00030003 << 2j (after >> 8 for the second token) leaves channel pair (2j, 2j+1) in
    the low/high half-words."""
    rng = np.random.default_rng(9)
    codes = rng.integers(0, 4, size=(32, 128)).astype(np.uint16)
    w = ko.pack_key_codes(codes, 2)[0]
    for lane in (0, 5, 16, 37, 63):
        r, kq = lane % 16, lane // 16
        for ks in range(4):
            word = int(w[lane * 4 + ks])
            for mt in range(2):
                sh = word >> (8 * mt)
                for j in range(4):
                    m = sh & (0x00030003 << (2 * j))
                    lo = (m & 0xFFFF) >> (2 * j)
                    hi = (m >> 16) >> (2 * j)
                    c0 = ks * 32 + kq * 8 + 2 * j
                    assert lo == codes[mt * 16 + r, c0] and hi == codes[mt * 16 + r, c0 + 1]
    wv = ko.pack_value_codes(codes, 2)[0]
    for lane in (0, 21, 63):
        r, kq = lane % 16, lane // 16
        for u in range(8):
            word = int(wv[lane * 4 + (u >> 1)]) >> (8 * (u & 1))
            for j in range(4):
                m = word & (0x00030003 << (2 * j))
                lo = (m & 0xFFFF) >> (2 * j)
                hi = (m >> 16) >> (2 * j)
                assert lo == codes[kq * 8 + 2 * j, u * 16 + r]
                assert hi == codes[kq * 8 + 2 * j + 1, u * 16 + r]
