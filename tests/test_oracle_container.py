"""Pins for the oracle's container: exact round trips, chunk independence, modes, errors."""
import numpy as np
import pytest
import torch

from oracle import zc_oracle as o
from paper_2508_19263_amd import workloads as wl


def make_input(fmt, n, seed):
    """(element bytes, scale bytes or None) with a skewed, weight-like distribution."""
    if fmt == o.BF16:
        return wl.bf16_weight(n, seed=seed).numpy().view(np.uint8), None
    if fmt == o.FP8_E4M3:
        return (wl.fp8_weight(n, seed=seed).numpy() if n else np.zeros(0, np.uint8)), None
    p, s = wl.mxfp4_weight(1, n, seed=seed) if n else (torch.zeros(0, dtype=torch.uint8),) * 2
    return p.numpy(), s.numpy()


def roundtrip(fmt, n, chunk_bytes, S, policy=o.POLICY_HUFF_ALL, L=(0, 0, 0), base=None, data=None):
    src, sc = data if data is not None else make_input(fmt, n, seed=n + S)
    p = o.params(fmt, chunk_bytes, L, S, policy)
    comp = o.compress(src, n, p, xor_base=base, scales=sc)
    assert len(comp) <= o.compress_bound(n, p)
    rc, out, sco = o.decompress(comp, len(src), xor_base=base, n_scales=0 if sc is None else len(sc))
    assert rc == o.OK
    assert np.array_equal(out, src), "round trip must be bit exact (lossless: Sec. 1, 2.2)"
    if sc is not None and len(sc):
        assert np.array_equal(sco, sc)
    return comp, src, sc


@pytest.mark.parametrize("fmt,G", [(o.BF16, 8), (o.FP8_E4M3, 16)])
@pytest.mark.parametrize("S", [1, 4, 64])
def test_round_trip_sizes(fmt, G, S):
    chunk_bytes = 4096
    E = chunk_bytes * 8 // o.elem_bits(fmt)
    for n in (0, 1, G * S - 1, G * S, G * S + 1, E - 1, E, E + 1, 3 * E + 17 * G + 5):
        for policy in (o.POLICY_HUFF_ALL, o.POLICY_AUTO):
            roundtrip(fmt, n, chunk_bytes, S, policy)


@pytest.mark.parametrize("S", [1, 8, 64])
def test_round_trip_fp4(S):
    chunk_bytes = 1024                       # 2048 elements, 64 scales per chunk
    for n in (0, 32, 32 * 15, 32 * 16, 32 * 17, 2048 - 32, 2048, 2048 + 32, 3 * 2048 + 32 * 37):
        for policy in (o.POLICY_HUFF_ALL, o.POLICY_AUTO):
            roundtrip(o.FP4_E2M1_MX, n, chunk_bytes, S, policy)


def test_xor_delta_round_trip_and_gain():
    # Sec. 3.1/4.1: consecutive checkpoints differ little, so the XOR delta has a very
    # skewed exponent stream and compresses better than the tensor itself
    n = 50000
    w0, w1 = wl.bf16_checkpoint_pair(n, seed=3)
    w0, w1 = w0.numpy().view(np.uint8), w1.numpy().view(np.uint8)
    plain, _, _ = roundtrip(o.BF16, n, 16384, 64, data=(w1, None))
    delta, _, _ = roundtrip(o.BF16, n, 16384, 64, base=w0, data=(w1, None))
    assert delta[10] == 1 and plain[10] == 0
    assert len(delta) < 0.6 * len(plain)
    # decoding a delta container needs the base
    rc, _, _ = o.decompress(delta, len(w1))
    assert rc == o.ERR_ARG


def test_chunks_decode_independently():
    # Sec. 3.1: chunks support random access and parallel decoding
    for fmt, n, cb in ((o.FP8_E4M3, 10 * 2048 + 777, 2048), (o.BF16, 7 * 1024 + 5, 2048), (o.FP4_E2M1_MX, 9 * 1024 + 96, 512)):
        src, sc = make_input(fmt, n, 11)
        comp = o.compress(src, n, o.params(fmt, cb, streams=8), scales=sc)
        nc = (len(src) + cb - 1) // cb
        for c in (nc - 1, 0, nc // 2):
            lo, hi = c * cb, min(len(src), (c + 1) * cb)
            rc, out, sco = o.decompress_chunk(comp, c, cb, n_scales=0 if sc is None else cb // 16)
            assert rc == o.OK
            assert np.array_equal(out[:hi - lo], src[lo:hi])
            if sc is not None:
                ns = (hi - lo) // 16
                assert np.array_equal(sco[:ns], sc[c * (cb // 16):c * (cb // 16) + ns])
        # a chunk's bytes do not depend on the rest: compressing a prefix of whole chunks with
        # the same code would give the same streams; check the weaker, code-free form: damaging
        # chunk 0's stream leaves chunk 1 decodable
        hdr_payload = int(np.frombuffer(comp[56:64].tobytes(), "<u8")[0])
        bad = comp.copy()
        bad[hdr_payload:hdr_payload + 4] ^= 0xFF
        rc, out, _ = o.decompress_chunk(bad, 1, cb, n_scales=0 if sc is None else cb // 16)
        assert rc == o.OK and np.array_equal(out[:cb], src[cb:2 * cb])


def test_modes_const_raw_two_valued_uniform():
    n = 5000
    # all equal -> both fields CONST, no payload at all
    x = np.full(n, 0x38, np.uint8)
    comp, _, _ = roundtrip(o.FP8_E4M3, n, 1024, 64, data=(x, None))
    assert comp[32] == o.MODE_CONST and comp[36] == o.MODE_CONST
    assert comp[35] == 7 and comp[39] == 0
    assert len(comp) == int(np.frombuffer(comp[56:64].tobytes(), "<u8")[0])
    # two values: exponent has 2 symbols (1 bit each), sign+mantissa is CONST
    x = np.where(np.arange(n) % 3 == 0, 0x38, 0x40).astype(np.uint8)
    comp, _, _ = roundtrip(o.FP8_E4M3, n, 1024, 64, data=(x, None))
    assert comp[32] == o.MODE_HUFF and comp[34] == 1 and comp[36] == o.MODE_CONST
    # uniform random bytes: nothing to gain; still exact, AUTO stores both fields raw
    rng = np.random.default_rng(12)
    x = rng.integers(0, 256, n).astype(np.uint8)
    comp_h, _, _ = roundtrip(o.FP8_E4M3, n, 1024, 64, data=(x, None))
    comp_a, _, _ = roundtrip(o.FP8_E4M3, n, 1024, 64, policy=o.POLICY_AUTO, data=(x, None))
    assert comp_a[32] == o.MODE_RAW and comp_a[36] == o.MODE_RAW
    assert len(comp_a) <= len(comp_h) and len(comp_a) >= n
    # Sec. 3.1: the skewed exponent is Huffman coded, the flat mantissa stored as is
    x, _ = make_input(o.FP8_E4M3, 20000, 5)
    comp, _, _ = roundtrip(o.FP8_E4M3, 20000, 4096, 64, policy=o.POLICY_AUTO, data=(x, None))
    assert comp[32] == o.MODE_HUFF and comp[36] == o.MODE_RAW


def test_length_limit_binds_and_still_round_trips():
    # exponent histogram steep enough that unlimited Huffman would need > 8 bits
    rng = np.random.default_rng(13)
    p = np.exp2(-np.arange(1, 17, dtype=float)); p /= p.sum()
    e = rng.choice(16, size=60000, p=p).astype(np.uint8)
    x = (e << 3) | rng.integers(0, 8, 60000).astype(np.uint8)
    for L in (4, 5, 8, 15):
        comp, _, _ = roundtrip(o.FP8_E4M3, len(x), 8192, 64, L=(L, L, 0), data=(x, None))
        st = o.stats(x, len(x), o.params(o.FP8_E4M3, 8192, (L, L, 0), 64))
        assert st.field[0].max_len <= L
        assert comp[34] == st.field[0].max_len


def test_raw_stream_layout_hand_worked():
    # RAW: symbols in element order, sym_bits each, little-endian bit string.
    # 16 FP8 bytes with exponent i and sign+mantissa 15-i: every nibble value once per field,
    # so the code is flat and AUTO stores both fields raw: nibbles packed low nibble first.
    e = np.arange(16)
    sm = 15 - e
    x = (((sm >> 3) << 7) | (e << 3) | (sm & 7)).astype(np.uint8)
    comp = o.compress(x, 16, o.params(o.FP8_E4M3, 16, streams=1, policy=o.POLICY_AUTO))
    pay = int(np.frombuffer(comp[56:64].tobytes(), "<u8")[0])
    assert comp[32] == o.MODE_RAW and comp[36] == o.MODE_RAW
    assert comp[pay:pay + 16].tolist() == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE] + [0] * 8
    assert comp[pay + 16:pay + 32].tolist() == [0xEF, 0xCD, 0xAB, 0x89, 0x67, 0x45, 0x23, 0x01] + [0] * 8
    assert len(comp) == pay + 32
    rc, out, _ = o.decompress(comp, 16)
    assert rc == o.OK and np.array_equal(out, x)


def test_header_layout_and_index():
    n, cb = 10000, 4096
    x, _ = make_input(o.FP8_E4M3, n, 21)
    comp = o.compress(x, n, o.params(o.FP8_E4M3, cb, streams=16))
    assert comp[:4].tobytes() == b"ZC1\0"
    assert comp[4] == 1 and comp[6] == o.FP8_E4M3 and comp[8] == 16 and comp[9] == 2
    u32 = lambda off: int(np.frombuffer(comp[off:off + 4].tobytes(), "<u4")[0])
    u64 = lambda off: int(np.frombuffer(comp[off:off + 8].tobytes(), "<u8")[0])
    assert u32(12) == cb and u64(16) == n and u32(24) == 3 and u64(48) == len(comp)
    pay = u64(56)
    assert pay == 64 + 16 + 16 + 16 + 16          # 2 tables of 16 bytes, 2 indices of 4 u32
    idx0 = [u32(96 + 4 * i) for i in range(4)]
    idx1 = [u32(112 + 4 * i) for i in range(4)]
    assert idx0[0] == 0 and idx0 == sorted(idx0) and idx1 == sorted(idx1) and idx1[0] == idx0[3]
    assert pay + 16 * idx1[3] == len(comp)
    # the length table in the container is the code that the histogram gives
    e, sm = o.split(o.FP8_E4M3, x, n)
    assert comp[64:80].tolist() == o.code_lengths(np.bincount(e, minlength=16).tolist(), 8).tolist()
    assert comp[80:96].tolist() == o.code_lengths(np.bincount(sm, minlength=16).tolist(), 8).tolist()
    # each chunk stream is what encode_stream gives for the chunk's symbols
    ln = comp[64:80]
    for c in range(3):
        seg = e[c * cb:(c + 1) * cb]
        s = o.encode_stream(seg, ln, 16, 16)
        assert np.array_equal(comp[pay + 16 * idx0[c]:pay + 16 * idx0[c + 1]], s)


def test_reverse_payload_order():
    # the container with its fields in reverse order in the payload: the same tables, the same streams byte for byte
    # (each is what encode_stream / the raw packing gives for the chunk's symbols), only where they lie differs: the
    # last field's streams first, every index still counting 16-byte units from the payload start
    u32 = lambda c, off: int(np.frombuffer(c[off:off + 4].tobytes(), "<u4")[0])
    u64 = lambda c, off: int(np.frombuffer(c[off:off + 8].tobytes(), "<u8")[0])
    cases = [(o.FP8_E4M3, 5 * 2048 + 333, 2048, 8, o.POLICY_HUFF_ALL), (o.FP8_E4M3, 5 * 2048 + 333, 2048, 8, o.POLICY_AUTO),
             (o.BF16, 3 * 1024 + 77, 2048, 64, o.POLICY_HUFF_ALL), (o.FP4_E2M1_MX, 9 * 1024 + 96, 512, 16, o.POLICY_HUFF_ALL),
             (o.FP8_E4M3, 0, 2048, 8, o.POLICY_HUFF_ALL), (o.FP8_E4M3, 7, 2048, 8, o.POLICY_HUFF_ALL)]
    for fmt, n, cb, S, policy in cases:
        src, sc = make_input(fmt, n, 31)
        a = o.compress(src, n, o.params(fmt, cb, streams=S, policy=policy), scales=sc)
        b = o.compress(src, n, o.params(fmt, cb, streams=S, policy=policy, payload_order=1), scales=sc)
        nf = int(a[9])
        pay = u64(a, 56)
        assert len(a) == len(b) and u64(b, 56) == pay and a[10] == 0 and b[10] == 2
        nc = u32(a, 24)
        tab = 64 + sum(((1 << int(a[33 + 4 * f])) + 15) // 16 * 16 for f in range(nf))
        assert np.array_equal(a[11:tab], b[11:tab])                          # header fields and code-length tables
        ia = [[u32(a, tab + f * ((4 * (nc + 1) + 15) & ~15) + 4 * i) for i in range(nc + 1)] for f in range(nf)]
        ib = [[u32(b, tab + f * ((4 * (nc + 1) + 15) & ~15) + 4 * i) for i in range(nc + 1)] for f in range(nf)]
        for f in range(nf):
            for c in range(nc):
                sa = a[pay + 16 * ia[f][c]:pay + 16 * ia[f][c + 1]]
                sb = b[pay + 16 * ib[f][c]:pay + 16 * ib[f][c + 1]]
                assert np.array_equal(sa, sb), (fmt, f, c)
        # order: the last field starts the payload, each field starts where the one after it ended
        assert ib[nf - 1][0] == 0 and pay + 16 * ib[0][nc] == len(b)
        for f in range(nf - 1):
            assert ib[f][0] == ib[f + 1][nc]
        rc, out, sco = o.decompress(b, len(src), n_scales=0 if sc is None else len(sc))
        assert rc == o.OK and np.array_equal(out, src) and (sc is None or np.array_equal(sco, sc))
        if nc > 1:
            rc, out, _ = o.decompress_chunk(b, 1, cb, n_scales=0 if sc is None else cb // 16)
            assert rc == o.OK and np.array_equal(out[:cb], src[cb:2 * cb])
        # an index in the other order is damage: the flag and the offsets must agree
        if n > cb:
            bad = b.copy(); bad[10] = 0
            assert o.decompress(bad, len(src), n_scales=0 if sc is None else len(sc))[0] == o.ERR_CORRUPT
    # with one field of fixed stream size in front, the place of exponent stream c depends on the exponent streams
    # before it alone: FP8 pages whose sign+mantissa field is flat or raw
    src, _ = make_input(o.FP8_E4M3, 6 * 2048, 32)
    b = o.compress(src, len(src), o.params(o.FP8_E4M3, 2048, streams=8, policy=o.POLICY_AUTO, payload_order=1))
    assert b[36] == o.MODE_RAW
    tab = 64 + 32
    i1 = [u32(b, tab + 32 + 4 * i) for i in range(7)]
    assert i1 == [64 * i for i in range(7)]                                  # 2048 nibbles = 1 KiB = 64 units per page
    assert u32(b, tab) == 6 * 64


def test_corrupt_containers_are_rejected():
    x, _ = make_input(o.FP8_E4M3, 9000, 22)
    comp = o.compress(x, 9000, o.params(o.FP8_E4M3, 4096))

    def status(mutate):
        bad = comp.copy()
        mutate(bad)
        return o.decompress(bad, 9000)[0]

    assert status(lambda b: None) == o.OK
    assert status(lambda b: b.__setitem__(0, 0x5B)) == o.ERR_CORRUPT            # magic
    assert status(lambda b: b.__setitem__(6, 9)) == o.ERR_CORRUPT               # format
    assert status(lambda b: b.__setitem__(24, 7)) == o.ERR_CORRUPT              # chunk count
    assert status(lambda b: b.__setitem__(64, 0)) == o.ERR_CORRUPT              # Kraft sum != 1
    assert status(lambda b: b.__setitem__(slice(100, 104), [0xFF] * 4)) == o.ERR_CORRUPT  # offsets
    assert o.decompress(comp[:len(comp) - 16], 9000)[0] == o.ERR_CORRUPT        # truncated
    assert o.decompress(comp, 8999)[0] == o.ERR_SMALL


def test_bad_parameters():
    x = np.zeros(64, np.uint8)
    for p in (o.params(9, 4096), o.params(o.FP8_E4M3, 100), o.params(o.FP8_E4M3, 4096, streams=3),
              o.params(o.FP4_E2M1_MX, 128)):
        assert o.compress_bound(64, p) == 0
    with pytest.raises(ValueError):
        o.compress(x, 33, o.params(o.FP4_E2M1_MX, 256), scales=np.zeros(2, np.uint8))


def test_static_dictionary_training_and_use():
    # Sec. 3.3 / 5.2: a dictionary trained on representative data is applied to other tensors
    a, _ = make_input(o.FP8_E4M3, 150000, 31)
    b, _ = make_input(o.FP8_E4M3, 90001, 32)
    p = o.params(o.FP8_E4M3, 16384, streams=16)
    ln, md = o.train_code(a, len(a), p)
    e, sm = o.split(o.FP8_E4M3, a, len(a))
    # the training rule: histogram with every count raised by one, then the usual construction
    assert ln[0, :16].tolist() == o.code_lengths((np.bincount(e, minlength=16) + 1).tolist(), 8).tolist()
    assert ln[1, :16].tolist() == o.code_lengths((np.bincount(sm, minlength=16) + 1).tolist(), 8).tolist()
    assert md.tolist() == [o.MODE_HUFF, o.MODE_HUFF, 0] and ln[0, :16].min() >= 1
    comp = o.compress_with_code(b, len(b), p, ln, md)
    rc, out, _ = o.decompress(comp, len(b))
    assert rc == o.OK and np.array_equal(out, b)
    # the container carries the dictionary, not b's own code
    assert comp[64:80].tolist() == ln[0, :16].tolist() and comp[80:96].tolist() == ln[1, :16].tolist()
    own = o.compress(b, len(b), p)
    assert len(comp) >= len(own)
    # size: sum(hist_b * len_dict) payload bits plus at most the look-ahead and padding overhead
    eb, smb = o.split(o.FP8_E4M3, b, len(b))
    bits = int((np.bincount(eb, minlength=16) * ln[0, :16].astype(np.int64)).sum() + (np.bincount(smb, minlength=16) * ln[1, :16].astype(np.int64)).sum())
    pay = int(np.frombuffer(comp[56:64].tobytes(), "<u8")[0])
    n_chunks = (len(b) + 16383) // 16384
    assert bits / 8 <= len(comp) - pay <= bits / 8 + 2 * n_chunks * (16 * 12 + 16)
    # AUTO: the flat sign+mantissa field of the dictionary is raw
    ln2, md2 = o.train_code(a, len(a), o.params(o.FP8_E4M3, 16384, streams=16, policy=o.POLICY_AUTO))
    assert md2.tolist() == [o.MODE_HUFF, o.MODE_RAW, 0]
    comp2 = o.compress_with_code(b, len(b), p, ln2, md2)
    assert comp2[36] == o.MODE_RAW and np.array_equal(o.decompress(comp2, len(b))[1], b)
    # a dictionary that cannot code every symbol is rejected
    bad = ln.copy(); bad[0, 3] = 0
    with pytest.raises(ValueError):
        o.compress_with_code(b, len(b), p, bad, md)
    # BF16 delta with a dictionary trained on another delta
    w0, w1 = wl.bf16_checkpoint_pair(40000, seed=5)
    v0, v1 = wl.bf16_checkpoint_pair(30000, seed=6)
    pb = o.params(o.BF16, 8192)
    lnb, mdb = o.train_code(w1.numpy(), 40000, pb, xor_base=w0.numpy())
    cb = o.compress_with_code(v1.numpy(), 30000, pb, lnb, mdb, xor_base=v0.numpy())
    rc, out, _ = o.decompress(cb, 60000, xor_base=v0.numpy().view(np.uint8))
    assert rc == o.OK and np.array_equal(out, v1.numpy().view(np.uint8))


def test_byte_grouped_formats():
    # Sec. 3.2 (Fig. 7), 3.4: symbols are bytes of the packed field arrays
    x, _ = make_input(o.FP8_E4M3, 70001, 77)
    e, sm = o.split(o.FP8_E4M3, x, len(x))
    # grouping == bytes of the nibble-packed array (numpy), zero filled at the odd end
    ge = o.group_values(o.FP8_E4M3_BYTES, 0, e, len(e))
    pad = np.concatenate([e, np.zeros(1, np.uint8)])
    assert np.array_equal(ge, pad[0::2] | (pad[1::2] << 4)) and len(ge) == 35001
    assert np.array_equal(o.ungroup_symbols(o.FP8_E4M3_BYTES, 0, ge, len(e)), e)
    m, sc = make_input(o.FP4_E2M1_MX, 32 * 2000, 78)
    e4, sm4 = o.split(o.FP4_E2M1_MX, m, 32 * 2000)
    g4 = o.group_values(o.FP4_E2M1_MX_BYTES, 1, sm4, len(sm4))
    assert np.array_equal(g4, sm4[0::4] | (sm4[1::4] << 2) | (sm4[2::4] << 4) | (sm4[3::4] << 6))
    for fmt, plain, src, n, scales in ((o.FP8_E4M3_BYTES, o.FP8_E4M3, x, len(x), None), (o.FP4_E2M1_MX_BYTES, o.FP4_E2M1_MX, m, 32 * 2000, sc)):
        for S in (64, 4):
            p, pp = o.params(fmt, 4096, streams=S), o.params(plain, 4096, streams=S)
            comp = o.compress(src, n, p, scales=scales)
            rc, out, sco = o.decompress(comp, len(src.reshape(-1)), n_scales=0 if scales is None else n // 32)
            assert rc == o.OK and np.array_equal(out, src.reshape(-1))
            assert comp[6] == fmt and comp[33] == 8 and comp[37] == 8
            st, sp = o.stats(src, n, p, scales=scales), o.stats(src, n, pp, scales=scales)
            for f in range(2):
                # the product of the per-value code is one of the codes a group may get (and fits the limit
                # 16 = 2 x 8 = 4 x 4... of the per-value limits), so the optimal group code cannot cost more,
                # apart from the zero fill of one last group
                assert st.field[f].payload_bits <= sp.field[f].payload_bits + 16
                assert st.field[f].n_symbols == (n + o.group_of(fmt) - 1) // o.group_of(fmt)
                # the group histogram is the histogram of the packed bytes
                vals = o.split(plain, src, n)[f]
                assert list(st.field[f].hist) == np.bincount(o.group_values(fmt, f, vals, n), minlength=256).tolist()
            # every chunk alone
            E = 4096 * 8 // o.elem_bits(fmt)
            c = (n - 1) // E
            rc, oc, _ = o.decompress_chunk(comp, c, 4096, n_scales=0 if scales is None else E // 32)
            nb = (n - c * E) * o.elem_bits(fmt) // 8
            assert rc == o.OK and np.array_equal(oc[:nb], src.reshape(-1)[c * 4096:c * 4096 + nb])
        # raw storage packs the same bits in both readings of the field: identical payloads
        u = np.random.default_rng(5).integers(0, 256, len(src.reshape(-1)), dtype=np.uint8)
        ca = o.compress(u, n, o.params(fmt, 4096, policy=o.POLICY_AUTO), scales=scales)
        cp = o.compress(u, n, o.params(plain, 4096, policy=o.POLICY_AUTO), scales=scales)
        assert ca[32] == o.MODE_RAW and cp[32] == o.MODE_RAW and ca[36] == o.MODE_RAW and cp[36] == o.MODE_RAW
        pa, pb = int(np.frombuffer(ca[56:64].tobytes(), "<u8")[0]), int(np.frombuffer(cp[56:64].tobytes(), "<u8")[0])
        ia, ib = int(np.frombuffer(ca[24:28].tobytes(), "<u4")[0]), int(np.frombuffer(cp[24:28].tobytes(), "<u4")[0])
        assert ia == ib
        if scales is None:
            assert np.array_equal(ca[pa:], cp[pb:])


def test_nvfp4_format():
    # Sec. 3.4: E2M1 elements with one FP8 scale byte per 16 elements
    n = 16 * 3000 + 16
    m, sc = wl.nvfp4_weight(1, n, seed=12)
    m, sc = m.numpy(), sc.numpy()
    assert len(sc) == n // 16
    p = o.params(o.FP4_E2M1_NV, 4096, streams=16)
    comp = o.compress(m, n, p, scales=sc)
    rc, out, so = o.decompress(comp, n // 2, n_scales=n // 16)
    assert rc == o.OK and np.array_equal(out, m) and np.array_equal(so, sc)
    st = o.stats(m, n, p, scales=sc)
    assert st.n_fields == 3 and st.field[2].n_symbols == n // 16 and st.raw_bytes == n // 2 + n // 16
    assert list(st.field[2].hist) == np.bincount(sc, minlength=256).tolist()
    # the element fields are those of the MX format on the same bytes
    mx = o.stats(m[:n // 64 * 32], n // 32 * 32, o.params(o.FP4_E2M1_MX, 4096, streams=16), scales=np.zeros(n // 32, np.uint8))
    assert list(mx.field[0].hist)[:4] == np.bincount(o.split(o.FP4_E2M1_NV, m, n // 32 * 32)[0], minlength=4).tolist()
    # a chunk alone returns its 8192/16 scale bytes
    rc, oc, s1 = o.decompress_chunk(comp, 1, 4096, n_scales=512)
    assert rc == o.OK and np.array_equal(oc, m[4096:8192]) and np.array_equal(s1, sc[512:1024])
    # element count must be a multiple of the scale block
    with pytest.raises(ValueError):
        o.compress(m, n - 8, p, scales=sc)


def test_e5m2_format():
    x = wl.fp8_e5m2_weight(90001, seed=21).numpy()
    for S in (64, 4):
        for policy in (o.POLICY_HUFF_ALL, o.POLICY_AUTO):
            p = o.params(o.FP8_E5M2, 4096, streams=S, policy=policy)
            comp = o.compress(x, len(x), p)
            rc, out, _ = o.decompress(comp, len(x))
            assert rc == o.OK and np.array_equal(out, x)
            assert comp[6] == o.FP8_E5M2 and comp[33] == 8 and comp[37] == 8 and comp[32] == o.MODE_HUFF
    st = o.stats(x, len(x), p)
    e, sm = o.split(o.FP8_E5M2, x, len(x))
    assert list(st.field[0].hist) == np.bincount(e, minlength=256).tolist() and st.field[0].distinct <= 32
    assert list(st.field[1].hist) == np.bincount(sm, minlength=256).tolist() and st.field[1].distinct <= 8
    # the 3-bit sign+mantissa values of Gaussian data are near uniform: 3 bits each; the exponent beats 5 bits
    assert 2.99 < st.field[1].mean_code_len <= 3.01 and st.field[0].mean_code_len < 3.2
    assert abs(st.ratio_payload_total - (st.field[0].mean_code_len + st.field[1].mean_code_len) / 8) < 1e-9
