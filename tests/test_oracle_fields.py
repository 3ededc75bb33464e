"""Pins for the oracle's field split, rebuild and histogram (paper Sec. 3.1, 3.2, 3.4)."""
import os

import numpy as np
import pytest

from oracle import zc_oracle as o

GOLD = os.path.join(os.path.dirname(__file__), "golden")
FMT = {"bf16": o.BF16, "e4m3": o.FP8_E4M3, "e2m1": o.FP4_E2M1_MX}


def _rows(name):
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line


def test_hand_worked_splits():
    n = 0
    for row in _rows("field_split.txt"):
        fmt, _, pat, e, sm = row.split()
        f, x = FMT[fmt], int(pat, 16)
        assert o.lib().zco_exponent_of(f, x) == int(e, 16), row
        assert o.lib().zco_signmant_of(f, x) == int(sm, 16), row
        assert o.lib().zco_rebuild(f, int(e, 16), int(sm, 16)) == x, row
        n += 1
    assert n >= 12


@pytest.mark.parametrize("fmt,bits", [(o.BF16, 16), (o.FP8_E4M3, 8), (o.FP4_E2M1_MX, 4)])
def test_split_rebuild_identity_exhaustive(fmt, bits):
    # every bit pattern survives split -> rebuild, and the two symbols together use
    # every bit exactly once (their widths add up to the element width)
    L = o.lib()
    eb = {16: 8, 8: 4, 4: 2}[bits]
    seen = set()
    for x in range(1 << bits):
        e, sm = L.zco_exponent_of(fmt, x), L.zco_signmant_of(fmt, x)
        assert e < (1 << eb) and sm < (1 << (bits - eb))
        assert L.zco_rebuild(fmt, e, sm) == x
        seen.add((e, sm))
    assert len(seen) == 1 << bits


def test_exponent_is_the_ieee_exponent_field():
    # independent of the shifts in the oracle: numpy's frexp gives the unbiased exponent
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(4096) * np.exp2(rng.integers(-20, 20, 4096))).astype(np.float32)
    bits16 = (x.view(np.uint32) >> 16).astype(np.uint16)            # truncation is exact bf16
    xt = (bits16.astype(np.uint32) << 16).view(np.float32)
    e, sm = o.split(o.BF16, bits16, len(bits16))
    _, ex = np.frexp(xt)                                            # xt = m * 2^ex, m in [0.5,1)
    assert np.array_equal(e.astype(int), ex - 1 + 127)
    assert np.array_equal(sm >> 7, (xt < 0).astype(np.uint8))
    frac = np.abs(xt) / np.exp2((ex - 1).astype(np.float32)) - 1.0
    assert np.array_equal(sm & 0x7F, np.round(frac * 128).astype(np.uint8))


def test_fp4_nibble_order_and_array_split():
    # byte 0xF7: element 0 is the low nibble 0x7 (= 6.0), element 1 the high nibble 0xF (= -6.0)
    e, sm = o.split(o.FP4_E2M1_MX, np.array([0xF7, 0x1A], np.uint8), 4)
    assert e.tolist() == [3, 3, 1, 0] and sm.tolist() == [1, 3, 2, 1]
    assert o.join(o.FP4_E2M1_MX, e, sm).tolist() == [0xF7, 0x1A]


def test_xor_delta_split():
    # Sec. 3.1 / 4.1: the delta is the bitwise XOR of the two BF16 patterns
    a = np.array([0x3F80, 0xBFC0, 0x3CA4, 0x0001], np.uint16)
    b = np.array([0x3F80, 0x3FC0, 0x3CA5, 0x8000], np.uint16)
    e, sm = o.split(o.BF16, a, 4, base=b)
    e2, sm2 = o.split(o.BF16, a ^ b, 4)
    assert np.array_equal(e, e2) and np.array_equal(sm, sm2)
    assert e.tolist() == [0, 0, 0, 0] and sm.tolist() == [0, 0x80, 1, 0x81]
    assert np.array_equal(o.join(o.BF16, e, sm, base=b).view(np.uint16), a)


def test_histogram_matches_bincount():
    rng = np.random.default_rng(2)
    for n in (0, 1, 257, 100000):
        s = rng.integers(0, 256, n).astype(np.uint8)
        h = o.histogram(s)
        assert int(h.sum()) == n
        assert np.array_equal(h, np.bincount(s, minlength=256).astype(np.uint64))


def test_e5m2_fields():
    # Sec. 3.2, the other FP8 variant: s eeeee mm.  Exhaustive identity, and the fields against torch's own
    # decoding of the byte (value = (-1)^s * 2^(e-15) * (1 + m/4) for normal numbers)
    import torch
    L = o.lib()
    seen = set()
    for x in range(256):
        e, sm = L.zco_exponent_of(o.FP8_E5M2, x), L.zco_signmant_of(o.FP8_E5M2, x)
        assert e < 32 and sm < 8 and L.zco_rebuild(o.FP8_E5M2, e, sm) == x
        seen.add((e, sm))
    assert len(seen) == 256
    codes = torch.arange(256, dtype=torch.uint8)
    vals = codes.view(torch.float8_e5m2).to(torch.float32).numpy()
    e, sm = o.split(o.FP8_E5M2, codes.numpy(), 256)
    normal = (e > 0) & (e < 31)
    _, ex = np.frexp(vals[normal])
    assert np.array_equal(e[normal].astype(int), ex - 1 + 15)
    assert np.array_equal(sm[normal] >> 2, (np.signbit(vals[normal])).astype(np.uint8))
    frac = np.abs(vals[normal]) / np.exp2((ex - 1).astype(np.float32)) - 1.0
    assert np.array_equal(sm[normal] & 3, np.round(frac * 4).astype(np.uint8))
    # hand-worked: 0x3C = 0 01111 00 = 1.0; 0xC5 = 1 10001 01 = -(1.25 * 4) = -5.0
    assert (L.zco_exponent_of(o.FP8_E5M2, 0x3C), L.zco_signmant_of(o.FP8_E5M2, 0x3C)) == (15, 0)
    assert (L.zco_exponent_of(o.FP8_E5M2, 0xC5), L.zco_signmant_of(o.FP8_E5M2, 0xC5)) == (17, 5)
    assert float(torch.tensor([0xC5], dtype=torch.uint8).view(torch.float8_e5m2).to(torch.float32)) == -5.0
    # symbols are held in 8 bits: 16 per 16-byte run in both fields
    assert o.lib().zco_sym_bits(o.FP8_E5M2, 0) == 8 and o.lib().zco_sym_bits(o.FP8_E5M2, 1) == 8 and o.lib().zco_num_fields(o.FP8_E5M2) == 2
