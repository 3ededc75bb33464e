"""Container validation of the HIP library on host memory (zc_validate_container): no GPU involved.

The containers come from the oracle, so this is also a CPU check that the library reads the oracle's header,
tables and chunk index the way the oracle wrote them."""
import numpy as np
import pytest

from oracle import zc_oracle as o
from paper_2508_19263_amd import workloads as wl
from paper_2508_19263_amd import zc


def containers():
    n = 9 * 4096 + 100
    yield zc.FMT_FP8_E4M3, o.compress(wl.fp8_weight(n, seed=3).numpy(), n, o.params(o.FP8_E4M3, 4096))
    m = 5 * 2048 + 9
    yield zc.FMT_BF16, o.compress(wl.bf16_weight(m, seed=4).numpy(), m, o.params(o.BF16, 4096, streams=8, policy=o.POLICY_AUTO))
    p, s = wl.mxfp4_weight(8, 2048, seed=5)
    yield zc.FMT_FP4_E2M1_MX, o.compress(p.numpy(), 8 * 2048, o.params(o.FP4_E2M1_MX, 1024), scales=s.numpy())


def reversed_containers():
    n = 9 * 4096 + 100
    yield zc.FMT_FP8_E4M3, o.compress(wl.fp8_weight(n, seed=3).numpy(), n, o.params(o.FP8_E4M3, 4096, payload_order=1))
    p, s = wl.mxfp4_weight(8, 2048, seed=5)
    yield zc.FMT_FP4_E2M1_MX, o.compress(p.numpy(), 8 * 2048, o.params(o.FP4_E2M1_MX, 1024, payload_order=1), scales=s.numpy())


def test_payload_order_is_read_from_the_header_and_checked_against_the_index():
    for (fmt, c), (_, r) in zip([x for x in containers() if x[0] != zc.FMT_BF16], reversed_containers()):
        assert zc.validate_container(c).payload_order == 0
        info = zc.validate_container(r)
        assert info.payload_order == 1 and info.format == fmt and info.total_bytes == len(r) == len(c)
        # the flag and the index must agree
        for good, flag in ((c, 2), (r, 0)):
            bad = good.copy()
            bad[10] = flag
            with pytest.raises(zc.ZcError) as e:
                zc.validate_container(bad)
            assert e.value.status == zc.ERR_CORRUPT


def test_oracle_containers_validate_and_describe_themselves():
    for fmt, c in containers():
        info = zc.validate_container(c)
        assert info.format == fmt and info.total_bytes == len(c)
        assert info.n_fields == (3 if fmt == zc.FMT_FP4_E2M1_MX else 2)
        # the code-length tables are the container's bytes
        for f in range(info.n_fields):
            A = 1 << info.sym_bits[f]
            assert list(info.code_len[f][:A]) == c[info.table_offset[f]:info.table_offset[f] + A].tolist()
        # header only (the first KiB) validates too, without the index
        head = zc.validate_container(c[:1024], check_index=False, container_bytes=len(c))
        assert head.n_chunks == info.n_chunks and head.total_bytes == len(c)
        with pytest.raises(zc.ZcError) as e:
            zc.validate_container(c[:info.payload_offset - 16], check_index=True, container_bytes=len(c))
        assert e.value.status == zc.ERR_INVALID_ARG
    # an empty tensor is a header-only container
    c = o.compress(np.zeros(0, np.uint8), 0, o.params(o.FP8_E4M3, 4096))
    info = zc.validate_container(c)
    assert info.n_elems == 0 and info.n_chunks == 0 and info.total_bytes == info.payload_offset == len(c)


def corrupt(c, at, value):
    d = c.copy()
    d[at] = value
    return d


def test_corrupt_containers_are_rejected():
    for fmt, c in containers():
        info = zc.validate_container(c)
        t0, i0, pay = int(info.table_offset[0]), int(info.index_offset[0]), int(info.payload_offset)
        bad = {
            "magic": corrupt(c, 0, 0x5B),
            "version": corrupt(c, 4, 2),
            "format": corrupt(c, 6, 9),
            "streams not a power of two": corrupt(c, 8, 3),
            "field count": corrupt(c, 9, 1),
            "chunk size": corrupt(c, 12, c[12] ^ 8),
            # (a count changed within its last chunk cannot be told from the header; one that changes the chunk count can)
            "element count": corrupt(c, 18, c[18] ^ 1) if fmt != zc.FMT_FP4_E2M1_MX else corrupt(c, 16, c[16] ^ 1),
            "chunk count": corrupt(c, 24, c[24] + 1),
            "mode": corrupt(c, 32, 7),
            "symbol width": corrupt(c, 33, c[33] ^ 1),
            "longest length": corrupt(c, 34, c[34] + 1),
            "total size beyond the buffer": corrupt(c, 50, c[50] + 1),
            "total size not a multiple of 16": corrupt(c, 48, c[48] ^ 4),
            "payload offset": corrupt(c, 56, c[56] ^ 16),
        }
        lens = c[t0:t0 + (1 << info.sym_bits[0])]
        used = int(np.flatnonzero(lens)[0])
        bad["incomplete code"] = corrupt(c, t0 + used, 0)
        bad["length above 16"] = corrupt(c, t0 + used, 17)
        for what, d in bad.items():
            with pytest.raises(zc.ZcError) as e:
                zc.validate_container(d)
            assert e.value.status == zc.ERR_CORRUPT, (fmt, what)
        # the chunk index: out of order, not starting at 0, not ending at the container's size
        d = c.copy(); d[i0 + 4:i0 + 8] = 0xFF
        with pytest.raises(zc.ZcError):
            zc.validate_container(d)
        assert zc.validate_container(d, check_index=False).total_bytes == len(c)      # only the index is wrong
        d = c.copy(); d[i0] = 1
        with pytest.raises(zc.ZcError):
            zc.validate_container(d)
        last = int(info.index_offset[info.n_fields - 1]) + 4 * int(info.n_chunks)
        d = c.copy(); d[last] ^= 1
        with pytest.raises(zc.ZcError):
            zc.validate_container(d)
        # truncated: the header says more bytes than are there
        with pytest.raises(zc.ZcError):
            zc.validate_container(c[:len(c) - 16])
        with pytest.raises(zc.ZcError):
            zc.validate_container(c[:40])
        assert pay <= len(c)


def test_params_are_size_versioned():
    p = zc.params(zc.FMT_FP8_E4M3, 4096)
    full = zc.compress_bound(10000, p)
    assert full > 0
    p.struct_size = 32                      # the first layout, without `flags`
    assert zc.compress_bound(10000, p) == full
    p.struct_size = 28
    assert zc.compress_bound(10000, p) == 0
    p = zc.params(zc.FMT_FP8_E4M3, 4096, flags=4)
    assert zc.compress_bound(10000, p) == 0  # unknown flag
