"""Pins for the oracle's lane-interleaved stream (the layout inside one chunk)."""
import os

import numpy as np
import pytest

from oracle import zc_oracle as o

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    for line in open(os.path.join(GOLD, "streams.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            S, G, ln, syms, hexbytes = [p.strip() for p in line.split("|")]
            yield (int(S), int(G), [int(v) for v in ln.split()], [int(v) for v in syms.split()],
                   bytes(int(b, 16) for b in hexbytes.split()))


def test_golden_streams():
    n = 0
    for S, G, ln, syms, want in _golden():
        got = o.encode_stream(np.array(syms, np.uint8), ln, G, S)
        assert got.tobytes() == want, (S, G)
        back, used = o.decode_stream(np.frombuffer(want, np.uint8), len(syms), ln, G, S)
        assert used == len(want) and back.tolist() == syms
        n += 1
    assert n >= 3


def lane_bits(syms, ln, codes, G, S, s):
    """The bit string of lane s: its symbols' codes, most significant bit first."""
    bits = []
    for j, v in enumerate(syms):
        if (j // G) % S == s:
            bits += [(int(codes[v]) >> b) & 1 for b in range(int(ln[v]) - 1, -1, -1)]
    return bits


def random_case(rng, A, n, skew):
    f = np.floor(np.exp2(rng.uniform(0, skew, A))).astype(np.int64) + 1
    p = f / f.sum()
    return rng.choice(A, size=n, p=p).astype(np.uint8), f


def test_single_lane_is_textbook_lsb_first_bitstream():
    # S=1: the stream is numpy.packbits(bitorder="little") of the concatenated codes,
    # plus look-ahead words of zeros and the 16-byte padding.
    rng = np.random.default_rng(7)
    for A, L in ((4, 3), (16, 8), (256, 16), (256, 9)):
        syms, f = random_case(rng, A, 3000, 14)
        ln = o.code_lengths(f.tolist(), L)
        codes = o.canonical_codes(ln)
        got = o.encode_stream(syms, ln, 16, 1)
        bits = lane_bits(syms, ln, codes, 16, 1, 0)
        packed = np.packbits(np.array(bits, np.uint8), bitorder="little")
        assert np.array_equal(got[:len(packed)], packed)
        assert not got[len(packed):].any()
        assert len(got) % 16 == 0
        # at most two look-ahead words plus alignment
        assert len(got) <= (len(bits) + 31) // 32 * 4 + 8 + 15


@pytest.mark.parametrize("S,G", [(1, 1), (2, 8), (4, 16), (64, 16), (64, 8), (8, 32), (16, 16), (32, 8)])
def test_stream_is_a_permutation_of_lane_words_and_round_trips(S, G):
    rng = np.random.default_rng(100 * S + G)
    for A, L, skew in ((16, 8, 10), (256, 16, 20), (4, 3, 3), (256, 8, 0.01), (16, 4, 6)):
        for n in (1, G * S - 1, G * S, G * S + 1, 5 * G * S + 3 * G + 1, 4000):
            syms, f = random_case(rng, A, n, skew)
            hist = np.bincount(syms, minlength=A)
            if (hist > 0).sum() < 2:
                continue
            ln = o.code_lengths(hist.tolist(), L)
            codes = o.canonical_codes(ln)
            stream = o.encode_stream(syms, ln, G, S)
            assert len(stream) % 16 == 0
            back, used = o.decode_stream(stream, n, ln, G, S)
            assert used == len(stream), "decoder must consume exactly what the encoder wrote"
            assert np.array_equal(back, syms)
            # multiset of words = every lane's packed bit string plus its zero look-ahead words
            words = sorted(stream.view("<u4").tolist())
            expect, total_bits = [], 0
            for s in range(S):
                bits = lane_bits(syms, ln, codes, G, S, s)
                total_bits += len(bits)
                if bits:
                    pk = np.packbits(np.array(bits + [0] * (-len(bits) % 32), np.uint8), bitorder="little")
                    expect += pk.view("<u4").tolist()
            expect.sort()
            nz = [w for w in words if w]
            assert nz == [w for w in expect if w]
            assert total_bits == int((hist * ln).sum())
            # overhead: at most 2 look-ahead words per lane + padding
            assert len(stream) <= 4 * len(expect) + 8 * S + 15


def test_truncated_or_wrong_table_is_rejected():
    rng = np.random.default_rng(8)
    syms, f = random_case(rng, 16, 5000, 8)
    ln = o.code_lengths(np.bincount(syms, minlength=16).tolist(), 8)
    stream = o.encode_stream(syms, ln, 16, 64)
    _, used = o.decode_stream(stream[:len(stream) // 2], 5000, ln, 16, 64)
    assert used == 0
    bad = ln.copy()
    bad[int(np.argmax(ln))] = 0                  # incomplete code (Kraft sum < 1)
    _, used = o.decode_stream(stream, 5000, bad, 16, 64)
    assert used == 0


def test_refill_period_changes_with_longest_code():
    # same symbols, two tables whose longest code differs (8 vs 4 bits with G=16): r = 4 vs 8.
    # Each must round-trip under its own table; the streams differ in word order only when
    # lanes run at different rates, but both obey the size bound.
    rng = np.random.default_rng(9)
    syms = rng.integers(0, 16, 64 * 16 * 7).astype(np.uint8)
    flat = [4] * 16
    s_flat = o.encode_stream(syms, flat, 16, 64)
    # flat code, r=8: every lane takes exactly one word every 8 symbols, so the stream is
    # rows of 64 words; lane 0's first word holds its first 8 symbols, code bits MSB first
    w0 = int(s_flat.view("<u4")[0])
    want = 0
    for t in range(8):
        v = int(syms[t])
        for b in range(4):
            want |= ((v >> (3 - b)) & 1) << (4 * t + b)
    assert w0 == want
    # number of words: 7 runs of 16 symbols -> 14 words per lane, +1 look-ahead? no: the last
    # check finds k = 32 exactly only after consuming, so the count is 14 + 1 request at step 8
    back, used = o.decode_stream(s_flat, len(syms), flat, 16, 64)
    assert used == len(s_flat) and np.array_equal(back, syms)


def test_stream_length_has_a_closed_form():
    # The decoder asks for a word at a refill step when it holds at most 32 unread bits, at most one word per step,
    # and r codes are at most 32 bits: by induction over the steps a lane with bits B before its last step has
    # taken min(steps, floor(B / 32) + 2) words when it ends.  So a stream's length follows from the lanes' bit
    # totals alone, without walking the steps (the size passes that work from symbol counts rely on this).
    rng = np.random.default_rng(20260317)
    cases = 0
    for A, L, G, S in ((16, 8, 16, 64), (16, 5, 16, 8), (256, 16, 8, 64), (256, 11, 8, 4), (256, 8, 16, 64), (32, 16, 16, 64),
                       (4, 3, 16, 2), (256, 9, 16, 1), (16, 4, 16, 64), (256, 13, 8, 32)):
        for n in (1, G - 1, G * S, G * S + 3, 5 * G * S - G - 1, 40 * G * S + G * (S // 2) + 2, 4096 + 17):
            syms, f = random_case(rng, A, n, 12)
            ln = np.asarray(o.code_lengths(f.tolist(), L))
            lmax = int(ln.max())
            r = 1
            while 2 * r * lmax <= 32:
                r *= 2
            r = min(r, G)
            words = 0
            lane_of = (np.arange(n) // G) % S
            for s in range(S):
                mine = ln[syms[lane_of == s]].astype(np.int64)
                if len(mine) == 0:
                    continue
                steps = -(-len(mine) // r)
                before_last_step = int(mine[:(steps - 1) * r].sum())
                words += min(steps, before_last_step // 32 + 2)
            got = o.encode_stream(syms, ln.tolist(), G, S)
            assert len(got) == 16 * (-(-words // 4)), (A, L, G, S, n)
            cases += 1
    assert cases == 70
