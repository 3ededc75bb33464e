"""Pins of the oracle's statistics (per-component breakdown of Sec. 4): entropy, mean code length,
payload bits and ratios against values fixed by arithmetic, not by the oracle itself.

A wrong logarithm base, a probability taken over the wrong total, a dropped term or a field
swapped with another each fail at least one of these."""
import math

import numpy as np

from oracle import zc_oracle as o
from paper_2508_19263_amd import workloads as wl


def shannon_bits(hist):
    """-sum p log2 p of a count vector, in float64, written independently of the oracle."""
    h = np.asarray(hist, np.float64)
    p = h[h > 0] / h.sum()
    return float(-(p * np.log2(p)).sum())


def bf16_from_fields(exp, sm):
    """BF16 bit patterns (little-endian bytes) with the given exponent and sign+mantissa symbols."""
    exp = np.asarray(exp, np.uint16)
    sm = np.asarray(sm, np.uint16)
    x = ((sm & 0x80) << 8) | (exp << 7) | (sm & 0x7F)
    return x.astype("<u2").view(np.uint8)


def test_entropy_of_hand_made_histograms_is_exact():
    # exponent field: a two-symbol 50/50 field, entropy exactly 1 bit;
    # sign+mantissa field: counts (8, 4, 2, 1, 1) x 64, a dyadic distribution, entropy exactly 1.875 bits
    reps = 64
    sm = np.repeat(np.array([3, 40, 77, 130, 255], np.uint8), np.array([8, 4, 2, 1, 1]) * reps)
    n = len(sm)
    exp = np.tile(np.array([0x7F, 0x80], np.uint8), n // 2)
    rng = np.random.default_rng(1)
    sm = rng.permutation(sm)
    x = bf16_from_fields(exp, sm)
    st = o.stats(x, n, o.params(o.BF16, 4096))
    assert st.n_fields == 2
    assert st.field[0].entropy_bits == 1.0
    assert abs(st.field[1].entropy_bits - 1.875) < 1e-15
    # dyadic histograms: the Huffman code reaches the entropy exactly
    assert st.field[0].mean_code_len == 1.0 and st.field[0].payload_bits == n
    assert abs(st.field[1].mean_code_len - 1.875) < 1e-15 and st.field[1].payload_bits == 30 * reps
    assert st.field[0].ratio_payload == 1.0 / 8 and abs(st.field[1].ratio_payload - 1.875 / 8) < 1e-15
    assert abs(st.ratio_payload_total - (n + 30 * reps) / (16.0 * n)) < 1e-15
    # a natural logarithm would have given ln 2 = 0.693 and 1.2997
    assert abs(st.field[0].entropy_bits - math.log(2)) > 0.3


def test_entropy_of_a_uniform_and_a_constant_field():
    # all 256 sign+mantissa bytes equally often: 8 bits; a single exponent: 0 bits (CONST, no payload)
    sm = np.tile(np.arange(256, dtype=np.uint8), 16)
    n = len(sm)
    x = bf16_from_fields(np.full(n, 0x7A, np.uint8), sm)
    st = o.stats(x, n, o.params(o.BF16, 4096))
    assert st.field[1].entropy_bits == 8.0 and st.field[1].mean_code_len == 8.0
    assert st.field[0].entropy_bits == 0.0 and st.field[0].mode == o.MODE_CONST and st.field[0].payload_bits == 0


def check_against_numpy(st, n_fields):
    for f in range(n_fields):
        fs = st.field[f]
        hist = np.array(fs.hist[:fs.alphabet], np.uint64)
        assert int(hist.sum()) == fs.n_symbols
        assert abs(fs.entropy_bits - shannon_bits(hist)) < 1e-12, (f, fs.entropy_bits, shannon_bits(hist))
        # payload bits and mean length from the histogram and the code lengths, recomputed here
        if fs.mode == o.MODE_HUFF:
            ln = np.array(fs.code_len[:fs.alphabet], np.uint64)
            assert int((hist * ln).sum()) == fs.payload_bits
            assert abs(fs.mean_code_len - fs.payload_bits / fs.n_symbols) < 1e-12
            assert fs.entropy_bits <= fs.mean_code_len + 1e-12


def test_entropy_matches_numpy_on_bf16_fp8_and_fp4():
    n = 1 << 18
    x = wl.bf16_weight(n, seed=0).numpy()
    st = o.stats(x, n, o.params(o.BF16, 65536))
    check_against_numpy(st, 2)
    # and the histograms themselves are those of the independently extracted fields
    u = np.ascontiguousarray(x).view(np.uint8).view("<u2")
    assert np.array_equal(np.bincount((u >> 7) & 0xFF, minlength=256), np.array(st.field[0].hist[:256], np.int64))
    assert np.array_equal(np.bincount(((u >> 8) & 0x80) | (u & 0x7F), minlength=256), np.array(st.field[1].hist[:256], np.int64))
    assert 2.0 < st.field[0].entropy_bits < 3.0                 # config 1: about 2.55 bits per exponent

    y = wl.fp8_weight(n, seed=1).numpy()
    st = o.stats(y, n, o.params(o.FP8_E4M3, 262144))
    check_against_numpy(st, 2)
    assert np.array_equal(np.bincount((y >> 3) & 0xF, minlength=16), np.array(st.field[0].hist[:16], np.int64))

    p, s = wl.mxfp4_weight(128, 4096, seed=2)
    st = o.stats(p.numpy(), 128 * 4096, o.params(o.FP4_E2M1_MX, 262144), scales=s.numpy())
    check_against_numpy(st, 3)
    assert np.array_equal(np.bincount(s.numpy(), minlength=256), np.array(st.field[2].hist[:256], np.int64))
    assert st.field[2].entropy_bits < 2.0 < st.field[2].alphabet   # the scale bytes are the compressible part (Sec. 3.4)

    pn, sn = wl.nvfp4_weight(128, 4096, seed=3)
    st = o.stats(pn.numpy(), 128 * 4096, o.params(o.FP4_E2M1_NV, 262144), scales=sn.numpy())
    check_against_numpy(st, 3)


def test_entropy_of_a_delta_is_taken_after_the_xor():
    n = 1 << 16
    w0, w1 = wl.bf16_checkpoint_pair(n, seed=4)
    st = o.stats(w1.numpy(), n, o.params(o.BF16, 65536), xor_base=w0.numpy())
    check_against_numpy(st, 2)
    d = (np.ascontiguousarray(w0.numpy()).view(np.uint8).view("<u2") ^ np.ascontiguousarray(w1.numpy()).view(np.uint8).view("<u2"))
    assert np.array_equal(np.bincount((d >> 7) & 0xFF, minlength=256), np.array(st.field[0].hist[:256], np.int64))
    assert st.field[0].entropy_bits < 0.5                        # Sec. 4.1: the delta's exponents are nearly all zero
