"""Host-side checks of the HIP library that need no GPU: it loads, exports every symbol
of include/zc.h, and its code construction agrees with the oracle's."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import zc_oracle as o
from paper_2508_19263_amd import zc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "zc.h")).read()
    declared = set(re.findall(r"\b(zc_[a-z_]+)\s*\(", header))
    assert declared == set(zc.EXPORTS)
    L = zc.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_struct_sizes_match_the_header():
    # sizes computed from the header's field lists by hand: see include/zc.h
    assert C.sizeof(zc.Params) == 4 * 9                                      # 32 bytes of the first layout + flags
    assert C.sizeof(zc.Info) == 8 * 4 + 3 * 8 + 6 * 8 + 12 + 768 + 4      # +4: tail padding to 8
    assert C.sizeof(zc.FieldStats) == 16 + 8 + 2048 + 256 + 8 + 8 + 8 + 8 + 8
    assert C.sizeof(zc.Tensor) == 11 * 8 + C.sizeof(zc.Info)


def test_code_construction_matches_oracle_on_random_histograms():
    rng = np.random.default_rng(40)
    for trial in range(3000):
        A = [4, 16, 256][trial % 3]
        kind = (trial // 3) % 4
        if kind == 0:
            f = np.floor(np.exp2(rng.uniform(0, 30, A))).astype(np.uint64)
        elif kind == 1:
            f = rng.integers(0, 4, A).astype(np.uint64)                       # many ties and zeros
        elif kind == 2:
            f = (rng.integers(1, 100, A) * (rng.random(A) < 0.3)).astype(np.uint64)
        else:
            f = np.sort(np.floor(np.exp2(np.arange(A) * 40.0 / A)).astype(np.uint64))[::-1].copy()
        if (f > 0).sum() < 2:
            continue
        L = int(rng.integers(max(1, int(np.ceil(np.log2((f > 0).sum())))), 17))
        want = o.code_lengths(f.tolist(), L)
        ln, cd = zc.build_code(f.tolist(), L)
        assert ln == want.tolist(), (trial, L)
        assert cd == o.canonical_codes(want).tolist()


def test_code_construction_rejects_too_small_limit():
    with pytest.raises(zc.ZcError):
        zc.build_code([1] * 9, 3)


def test_bounds_and_workspace():
    for fmt, cb in ((zc.FMT_BF16, 65536), (zc.FMT_FP8_E4M3, 262144), (zc.FMT_FP4_E2M1_MX, 262144)):
        p = zc.params(fmt, cb)
        po = o.params(fmt, cb)
        for n in (0, 32, 1 << 20, (1 << 22) + 32 * 5):
            assert zc.compress_bound(n, p) >= 64
            assert zc.workspace_bytes([n], p) > 0
            assert zc.compress_bound(n, p) > 0 and o.compress_bound(n, po) > 0
    # the workspace grows with the tensors, and FP8 with 64 lanes and 256 KiB chunks reserves 2 KiB per chunk on top
    # (the exponent counts per chunk lane that its size pass works from)
    for fmt, cb in ((zc.FMT_BF16, 65536), (zc.FMT_FP8_E4M3, 262144), (zc.FMT_FP8_E4M3, 131072)):
        sizes = [zc.workspace_bytes([n], zc.params(fmt, cb)) for n in (1 << 20, 1 << 24, 1 << 26)]
        assert sizes[0] < sizes[1] < sizes[2]
        assert zc.workspace_bytes([1 << 24, 1 << 24], zc.params(fmt, cb)) > sizes[1]
    # The formats of 8-bit symbols (BF16, FP8 in byte symbols) reserve 64 KiB per chunk there: 256 counts per chunk lane
    # and field; FP8 E5M2 reserves 5 KiB (40 counts per lane).  The FP8 formats have the same element size, fields and
    # work lists, so they differ by the counts.
    n = 1 << 28
    e4 = zc.workspace_bytes([n], zc.params(zc.FMT_FP8_E4M3, 262144))
    e5 = zc.workspace_bytes([n], zc.params(zc.FMT_FP8_E5M2, 262144))
    e8 = zc.workspace_bytes([n], zc.params(zc.FMT_FP8_E4M3_BYTES, 262144))
    assert e5 - e4 == (n // 262144) * (5120 - 2048)
    assert e8 - e4 == (n // 262144) * (65536 - 2048)
    assert zc.workspace_bytes([n // 2], zc.params(zc.FMT_BF16, 262144)) == e8
    # other chunk sizes and lane counts reserve nothing of the kind
    assert zc.workspace_bytes([n], zc.params(zc.FMT_FP8_E5M2, 131072)) < e4
    assert zc.workspace_bytes([n], zc.params(zc.FMT_FP8_E5M2, 262144, streams=32)) < e4
    assert zc.compress_bound(100, zc.params(zc.FMT_FP8_E4M3, 100)) == 0       # chunk not a multiple of 16
    assert zc.compress_bound(100, zc.params(9, 4096)) == 0
    assert zc.compress_bound(33, zc.params(zc.FMT_FP4_E2M1_MX, 256)) == 0     # FP4 needs whole 32-blocks
    assert zc.compress_bound(64, zc.params(zc.FMT_FP8_E4M3, 4096, (3, 0, 0))) == 0   # 2^3 < 16 symbols
    assert zc.status_string(zc.ERR_CORRUPT) == "corrupt container"


def test_code_stale_arithmetic():
    # the refresh test of a static dictionary is host arithmetic on two container descriptions
    code, w = zc.Info(), zc.Info()
    code.format = w.format = zc.FMT_FP8_E4M3
    code.n_elems, code.total_bytes = 1000000, 800000          # training tensor: ratio 0.80
    w.n_elems, w.total_bytes = 500000, 410000                 # 0.82
    assert zc.code_stale(code, w, 0.03) is False
    assert zc.code_stale(code, w, 0.01) is True
    w.format = zc.FMT_BF16                                    # another format: refused
    with pytest.raises(zc.ZcError):
        zc.code_stale(code, w, 0.01)
    code.format = w.format = zc.FMT_FP4_E2M1_MX               # raw size counts the scale bytes: n/2 + n/32
    code.n_elems, code.total_bytes = 3200, 1700
    w.n_elems, w.total_bytes = 6400, 3400 + 33
    assert zc.code_stale(code, w, 0.01) is False              # 3433/3400 = 1.0097 against 1700/1700 = 1
    w.total_bytes = 3400 + 69
    assert zc.code_stale(code, w, 0.01) is True
