"""zc_compress_noalloc (the entry point for callers that cannot allocate) against zc_compress, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2508_19263_amd import workloads as wl
from paper_2508_19263_amd import zc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(fmt, src, n, cb, S, policy=zc.POLICY_HUFF_ALL, base=None, scales=None, tag=""):
    """The container zc_compress_noalloc leaves must be the one zc_compress writes, byte for byte."""
    print("noalloc case", tag, "fmt", fmt, "n", n, "chunk", cb, "S", S, "policy", policy, flush=True)
    p = zc.params(fmt, cb, streams=S, policy=policy)
    d = lambda t: None if t is None else t.to(DEV)
    want, info = zc.compress(d(src), n, p, xor_base=d(base), scales=d(scales))
    want = want.clone()
    dst = torch.full((max(zc.compress_bound(n, p), 16),), 0xA5, dtype=torch.uint8, device=DEV)
    zc.compress_noalloc(d(src), n, p, dst, xor_base=d(base), scales=d(scales))
    torch.cuda.synchronize()
    got_info = zc.read_info(dst, check_index=True)
    assert got_info.total_bytes == want.numel(), (got_info.total_bytes, want.numel())
    got = dst[:want.numel()]
    assert torch.equal(got, want), "first difference at byte %d" % int((got != want).nonzero()[0])
    out, sco = zc.decompress(dst, got_info, xor_base=d(base))
    torch.cuda.synchronize()
    assert torch.equal(out.cpu()[:src.numel() * src.element_size()], src.view(torch.uint8).reshape(-1))
    if scales is not None:
        assert torch.equal(sco.cpu()[:scales.numel()], scales)
    return want.numel()


def test_noalloc_matches_compress_on_two_calls_in_a_row_the_second_smaller():
    # FP8, 256 KiB chunks, 64 lanes (the benchmark's shape: histogram with lane counts, FP8 size pass and encoder), a
    # ragged tail for the generic kernels; then a smaller tensor through the same scratch array
    big = wl.fp8_weight(21 * 262144 + 1234, seed=71)
    both(zc.FMT_FP8_E4M3, big, big.numel(), 262144, 64, tag="fp8-big")
    small = wl.fp8_weight(2 * 262144 + 77, seed=72)
    both(zc.FMT_FP8_E4M3, small, small.numel(), 262144, 64, tag="fp8-small")
    # and the big one again: what the smaller call left in the array must not matter
    both(zc.FMT_FP8_E4M3, big, big.numel(), 262144, 64, tag="fp8-big-again")


def test_noalloc_other_shapes_share_the_array():
    # K/V pages (page kernels, XCD-ordered lists of several hundred items), BF16 with a base, MXFP4 with scales,
    # an empty tensor, a single element: one after the other through the same array
    kv = wl.fp8_weight(3000 * 2048, seed=73)
    both(zc.FMT_FP8_E4M3, kv, kv.numel(), 2048, 8, tag="pages")
    w0, w1 = wl.bf16_checkpoint_pair(9 * 32768 + 11, seed=74)
    both(zc.FMT_BF16, w1.view(torch.uint8).reshape(-1), w1.numel(), 65536, 64, base=w0.view(torch.uint8).reshape(-1), tag="bf16-delta")
    both(zc.FMT_BF16, w1.view(torch.uint8).reshape(-1), w1.numel(), 4096, 8, policy=zc.POLICY_AUTO, tag="bf16-pages")
    pk, sc = wl.mxfp4_weight(64, 4096, seed=75)
    both(zc.FMT_FP4_E2M1_MX, pk, 64 * 4096, 16384, 64, scales=sc, tag="mxfp4")
    one = wl.fp8_weight(1, seed=76)
    both(zc.FMT_FP8_E4M3, one, 1, 4096, 64, tag="one")
    p = zc.params(zc.FMT_FP8_E4M3, 4096)
    dst = torch.full((zc.compress_bound(0, p),), 0xA5, dtype=torch.uint8, device=DEV)
    zc.compress_noalloc(torch.zeros(16, dtype=torch.uint8, device=DEV), 0, p, dst)
    torch.cuda.synchronize()
    info = zc.read_info(dst)
    assert info.n_elems == 0 and info.total_bytes == info.payload_offset


def test_noalloc_limits_are_errors():
    p = zc.params(zc.FMT_FP8_E4M3, 2048, streams=8)
    n = 1 << 31                                              # a million pages: the workspace would need more than the array holds
    assert zc.workspace_bytes([n], p) > zc.NOALLOC_SCRATCH_BYTES
    src = torch.zeros(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(zc.ZcError) as e:
        st = zc.lib().zc_compress_noalloc(zc._ptr(src), n, p, None, None, zc._ptr(src), zc.compress_bound(n, p), zc._stream())
        zc._check(st, "zc_compress_noalloc")
    assert e.value.status == zc.ERR_BUFFER_TOO_SMALL
    x = wl.fp8_weight(50000, seed=77).to(DEV)
    small = torch.empty(zc.compress_bound(50000, p) - 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(zc.ZcError) as e:
        zc.compress_noalloc(x, 50000, p, small)
    assert e.value.status == zc.ERR_BUFFER_TOO_SMALL
    with pytest.raises(zc.ZcError) as e:
        zc.compress_noalloc(x, 50000, zc.params(zc.FMT_FP8_E4M3, 2048, streams=8, flags=zc.FLAG_HOST_CODES), torch.empty(zc.compress_bound(50000, p), dtype=torch.uint8, device=DEV))
    assert e.value.status == zc.ERR_INVALID_ARG
