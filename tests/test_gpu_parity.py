"""GPU parity: the HIP library against the CPU oracle, byte for byte, through the C ABI."""
from ctypes import byref as C_byref

import numpy as np
import pytest
import torch

from oracle import zc_oracle as o
from paper_2508_19263_amd import workloads as wl
from paper_2508_19263_amd import zc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_input(fmt, n, seed):
    if fmt == zc.FMT_BF16:
        return wl.bf16_weight(n, seed=seed).view(torch.uint8), None
    if fmt == zc.FMT_FP8_E5M2:
        return wl.fp8_e5m2_weight(n, seed=seed) if n else torch.zeros(0, dtype=torch.uint8), None
    if fmt in (zc.FMT_FP8_E4M3, zc.FMT_FP8_E4M3_BYTES):
        return wl.fp8_weight(n, seed=seed) if n else torch.zeros(0, dtype=torch.uint8), None
    if n == 0:
        return torch.zeros(0, dtype=torch.uint8), torch.zeros(0, dtype=torch.uint8)
    if fmt == zc.FMT_FP4_E2M1_NV:
        return wl.nvfp4_weight(1, n, seed=seed)
    return wl.mxfp4_weight(1, n, seed=seed)


def dev(t):
    if t is None:
        return None
    if t.numel() == 0:
        return torch.zeros(16, dtype=torch.uint8, device=DEV)[:0]
    return t.to(DEV)


def o_info(container):
    """mode and longest code length per field from a container's header (bytes 32..43)."""
    c = np.asarray(container)
    return {"mode": [int(c[32 + 4 * f]) for f in range(3)], "lmax": [int(c[34 + 4 * f]) for f in range(3)]}


def check_case(fmt, n, cb, S, policy=zc.POLICY_HUFF_ALL, L=(0, 0, 0), data=None, base=None, tag="", order=0):
    """compress on both sides -> identical containers; decode the oracle's container on the
    GPU -> original bytes; decode on the GPU from the header alone -> original bytes."""
    src, sc = data if data is not None else make_input(fmt, n, seed=n % 1000 + S)
    print("case", tag, "fmt", fmt, "n", n, "chunk", cb, "S", S, "policy", policy, "L", L, "order", order, flush=True)
    p, po = zc.params(fmt, cb, L, S, policy, flags=zc.FLAG_REVERSE_FIELDS if order else 0), o.params(fmt, cb, L, S, policy, payload_order=order)
    want = o.compress(src.numpy(), n, po, xor_base=None if base is None else base.numpy(),
                      scales=None if sc is None else sc.numpy())
    comp, info = zc.compress(dev(src), n, p, xor_base=dev(base), scales=dev(sc))
    got = comp.cpu().numpy()
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.array_equal(got, want), "first difference at byte %d" % int(np.argmax(got != want))
    assert info.total_bytes == len(want)
    # decoder fed by the oracle's bytes, header parsed by the library
    oc = torch.from_numpy(want).to(DEV)
    info2 = zc.read_info(oc, check_index=True)
    out, sco = zc.decompress(oc, info2, xor_base=dev(base))
    torch.cuda.synchronize()
    assert torch.equal(out.cpu()[:src.numel()], src.view(torch.uint8).reshape(-1))
    if sc is not None and sc.numel():
        assert torch.equal(sco.cpu()[:sc.numel()], sc)
    return want, src, sc


@pytest.mark.parametrize("fmt,G", [(zc.FMT_BF16, 8), (zc.FMT_FP8_E4M3, 16)])
@pytest.mark.parametrize("S", [64, 8, 1])
def test_sizes_and_tails(fmt, G, S):
    cb = 4096
    E = cb * 8 // zc.elem_bits(fmt)
    for n in (1, G * S - 1, G * S, G * S + 1, E - 1, E, E + 1, 3 * E + 17 * G + 5, 40 * E + 3):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(fmt, n, cb, S, policy)


@pytest.mark.parametrize("S", [64, 16, 2])
def test_fp4_sizes(S):
    for n in (32, 32 * 15, 32 * 17, 2048 - 32, 2048, 2048 + 32, 3 * 2048 + 32 * 37, 70 * 2048):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP4_E2M1_MX, n, 1024, S, policy)


def test_empty_tensor():
    for fmt in (zc.FMT_BF16, zc.FMT_FP8_E4M3, zc.FMT_FP4_E2M1_MX):
        p = zc.params(fmt, 4096)
        src = torch.zeros(16, dtype=torch.uint8, device=DEV)
        comp, info = zc.compress(src, 0, p, scales=src if fmt == zc.FMT_FP4_E2M1_MX else None)
        want = o.compress(np.zeros(0, np.uint8), 0, o.params(fmt, 4096), scales=np.zeros(0, np.uint8))
        assert np.array_equal(comp.cpu().numpy(), want)
        out, _ = zc.decompress(comp, info, out=torch.zeros(16, dtype=torch.uint8, device=DEV),
                               scales_out=torch.zeros(16, dtype=torch.uint8, device=DEV))


def test_config1_bf16_full():
    # configuration 1: 1,048,576 BF16 values N(0, 0.02), seed 0, max length 16, 64 KiB chunks
    n = 1 << 20
    x = wl.bf16_weight(n, seed=0).view(torch.uint8)
    want, _, _ = check_case(zc.FMT_BF16, n, 65536, 64, L=(16, 16, 0), data=(x, None), tag="config1")
    assert want[34] > 11          # the code has words longer than the lookup table: slow path exercised
    st = zc.stats(x.to(DEV), n, zc.params(zc.FMT_BF16, 65536, (16, 16, 0)))
    so = o.stats(x.numpy(), n, o.params(o.BF16, 65536, (16, 16, 0)))
    compare_stats(st, so)


def compare_stats(st, so):
    assert st.n_fields == so.n_fields and st.raw_bytes == so.raw_bytes and st.container_bytes == so.container_bytes
    assert st.ratio_payload_total == so.ratio_payload_total and st.ratio_container_total == so.ratio_container_total
    for f in range(st.n_fields):
        a, b = st.field[f], so.field[f]
        assert list(a.hist) == list(b.hist) and list(a.code_len) == list(b.code_len)
        for k in ("alphabet", "distinct", "mode", "max_len", "n_symbols", "payload_bits", "stream_bytes"):
            assert getattr(a, k) == getattr(b, k), (f, k)
        assert abs(a.entropy_bits - b.entropy_bits) < 1e-12 and a.mean_code_len == b.mean_code_len
        assert a.ratio_payload == b.ratio_payload


def test_stats_all_formats():
    for fmt, n, cb in ((zc.FMT_FP8_E4M3, 300000, 65536), (zc.FMT_BF16, 200001, 16384), (zc.FMT_FP4_E2M1_MX, 32 * 9001, 8192)):
        src, sc = make_input(fmt, n, 77)
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            st = zc.stats(dev(src), n, zc.params(fmt, cb, policy=policy), scales=dev(sc))
            so = o.stats(src.numpy(), n, o.params(fmt, cb, policy=policy), scales=None if sc is None else sc.numpy())
            compare_stats(st, so)


def test_config2_fp8_layer_shapes_reduced():
    # one decoder layer of config 2 with both matrix dimensions / 8, 256 KiB chunks, S = 64
    for i, (name, r, c) in enumerate(wl.LAYER_8B):
        n = (r // 8) * (c // 8)
        x = wl.fp8_weight(n, seed=1000 + i)
        check_case(zc.FMT_FP8_E4M3, n, 262144, 64, data=(x, None), tag=name)


def test_config3_mxfp4_reduced():
    p, s = wl.mxfp4_weight(512, 3584, seed=3)
    want, _, _ = check_case(zc.FMT_FP4_E2M1_MX, 512 * 3584, 262144, 64, data=(p, s), tag="config3")
    check_case(zc.FMT_FP4_E2M1_MX, 512 * 3584, 262144, 64, policy=zc.POLICY_AUTO, data=(p, s), tag="config3-auto")


def test_config4_checkpoint_delta_reduced():
    n = 1 << 21
    w0, w1 = wl.bf16_checkpoint_pair(n, seed=4)
    w0, w1 = w0.view(torch.uint8), w1.view(torch.uint8)
    plain, _, _ = check_case(zc.FMT_BF16, n, 262144, 64, data=(w1, None), tag="config4-plain")
    delta, _, _ = check_case(zc.FMT_BF16, n, 262144, 64, data=(w1, None), base=w0, tag="config4-delta")
    assert len(delta) < 0.6 * len(plain)
    check_case(zc.FMT_BF16, n, 65536, 64, policy=zc.POLICY_AUTO, data=(w1, None), base=w0, tag="config4-delta-auto")


def test_stream_sizes_from_lane_counts_of_8_bit_symbols():
    # BF16 and FP8 in byte symbols with 64 lanes and chunks of 256 KiB: the histogram pass also counts both fields' symbols
    # per chunk lane, and the size pass of the tensors the 64-lane encoder takes works from those counts instead of reading
    # the source again.  Every refill period of the exponent field (codes of up to 16, 8 and 4 bits: 2, 4 and 8 symbols per step), a
    # sign+mantissa field that is flat, raw, table coded (a delta, periods 2 and 4) or constant, a short last chunk, a
    # tensor shorter than a chunk, and a batch whose tensors go different ways
    cb = 262144
    rng = np.random.default_rng(17)

    def bf16_of(n, n_exp, sm_bits):
        ex = (rng.integers(0, n_exp, n).astype(np.uint16) + 100) & 0xFF
        sm = rng.integers(0, 1 << sm_bits, n).astype(np.uint16)
        return torch.from_numpy((((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)).astype(np.uint16).view(np.uint8).copy())

    n = 5 * (cb // 2) + 12345
    for n_exp, L in ((40, (0, 0, 0)), (40, (8, 0, 0)), (12, (0, 0, 0)), (200, (0, 0, 0)), (3, (0, 0, 0))):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_BF16, n, cb, 64, policy, L=L, data=(bf16_of(n, n_exp, 8), None), tag="bf16-lane-counts")
    w0, w1 = wl.bf16_checkpoint_pair(n, seed=41)
    w0, w1 = w0.view(torch.uint8), w1.view(torch.uint8)
    for L in ((0, 0, 0), (16, 8, 0), (8, 8, 0), (11, 11, 0)):
        check_case(zc.FMT_BF16, n, cb, 64, L=L, data=(w1, None), base=w0, tag="bf16-lane-counts-delta")
    check_case(zc.FMT_BF16, n, cb, 64, data=(w1, None), base=w1, tag="bf16-lane-counts-constant")
    check_case(zc.FMT_BF16, n, cb, 64, data=(bf16_of(n, 1, 8), None), tag="bf16-lane-counts-one-exponent")
    check_case(zc.FMT_BF16, n, cb, 64, data=(bf16_of(n, 30, 0), None), tag="bf16-lane-counts-one-mantissa")
    check_case(zc.FMT_BF16, 3 * (cb // 2), cb, 64, data=(bf16_of(3 * (cb // 2), 30, 8), None), tag="bf16-lane-counts-whole")
    check_case(zc.FMT_BF16, 1000, cb, 64, data=(bf16_of(1000, 30, 8), None), tag="bf16-lane-counts-short")
    a = wl.fp8_weight(4 * cb + 777, seed=42)
    for L in ((0, 0, 0), (11, 0, 0), (8, 8, 0)):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E4M3_BYTES, a.numel(), cb, 64, policy, L=L, data=(a, None), tag="fp8-bytes-lane-counts")
    b = wl.fp8_weight(4 * cb + 777, seed=43)
    check_case(zc.FMT_FP8_E4M3_BYTES, a.numel(), cb, 64, data=(a, None), base=b, tag="fp8-bytes-lane-counts-delta")
    # FP8 E5M2: 16 symbols per run and field; exponent codes of every refill period (2, 4, 8 and, with four exponent values,
    # 16), a delta, a constant sign+mantissa field, a uniform tensor (every code 8 bits long)
    def e5m2_of(n, n_exp, geometric, n_sm=8):
        sm = rng.integers(0, n_sm, n).astype(np.uint8)
        ex = (np.minimum(rng.geometric(geometric, n) - 1, n_exp - 1) if geometric else rng.integers(0, n_exp, n)).astype(np.uint8)
        return torch.from_numpy(((sm >> 2) << 7 | (ex << 2) | (sm & 3)).astype(np.uint8))

    n5 = 4 * cb + 4321
    for x, L in ((e5m2_of(n5, 32, 0.45), (16, 0, 0)), (e5m2_of(n5, 32, 0.45), (11, 0, 0)), (e5m2_of(n5, 32, 0.45), (8, 8, 0)), (e5m2_of(n5, 6, 0), (0, 0, 0)),
                 (e5m2_of(n5, 4, 0), (0, 0, 0)), (e5m2_of(n5, 20, 0.3, n_sm=1), (0, 0, 0)), (wl.fp8_e5m2_weight(n5, seed=44), (0, 0, 0))):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E5M2, n5, cb, 64, policy, L=L, data=(x, None), tag="e5m2-lane-counts")
    check_case(zc.FMT_FP8_E5M2, n5, cb, 64, data=(e5m2_of(n5, 32, 0.45), None), base=e5m2_of(n5, 32, 0.3), tag="e5m2-lane-counts-delta")
    u8 = torch.from_numpy(rng.integers(0, 256, 3 * cb, dtype=np.uint8))
    check_case(zc.FMT_FP8_E5M2, u8.numel(), cb, 64, zc.POLICY_AUTO, data=(u8, None), tag="e5m2-lane-counts-uniform")
    check_case(zc.FMT_FP8_E5M2, 3 * cb, cb, 64, data=(torch.full((3 * cb,), 0x3C, dtype=torch.uint8), None), tag="e5m2-lane-counts-constant")
    # a batch: tensors with a table-coded, a raw and a constant second field, whole and ragged, queued without a wait too
    srcs = [bf16_of(2 * (cb // 2), 40, 8), w1, bf16_of(cb // 2 + 8, 1, 3), bf16_of(7 * (cb // 2), 9, 8)]
    bases = [torch.zeros_like(srcs[0]), w0, torch.zeros_like(srcs[2]), torch.zeros_like(srcs[3])]      # a batch has bases for all or none
    for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
        p, po = zc.params(zc.FMT_BF16, cb, policy=policy), o.params(o.BF16, cb, policy=policy)
        bt = zc.Batch([dev(x) for x in srcs], [x.numel() // 2 for x in srcs], p, xor_bases=[dev(x) for x in bases])
        sizes = bt.compress()
        for t, x in enumerate(srcs):
            want = o.compress(x.numpy(), x.numel() // 2, po, xor_base=bases[t].numpy())
            assert sizes[t] == len(want) and np.array_equal(bt.container(t).cpu().numpy(), want), (policy, t)
        bt.compress_async()
        assert bt.refresh_info() == sizes
        bt.decompress()
        torch.cuda.synchronize()
        for t, x in enumerate(srcs):
            assert torch.equal(bt.out[t].cpu()[:x.numel()], x), t


def test_config5_kv_pages_random_access():
    # pages of 16 tokens x 128 = 2 KiB are the chunks; decode a random 25% of the pages densely
    k, v = wl.fp8_kv_pair(batch=2, heads=4, tokens=1024, seed=5)
    for name, t in (("K", k), ("V", v)):
        flat = t.reshape(-1)
        n = flat.numel()
        for S in (8, 16, 4):
            want, _, _ = check_case(zc.FMT_FP8_E4M3, n, 2048, S, data=(flat, None), tag="config5-" + name)
            n_pages = n // 2048
            ids = wl.page_sample(n_pages, 0.25, seed=S)
            comp = torch.from_numpy(want).to(DEV)
            info = zc.read_info(comp)
            out, _ = zc.decompress_chunks(comp, info, ids.to(DEV))
            torch.cuda.synchronize()
            pages = flat.reshape(n_pages, 2048)[ids.long()]
            assert torch.equal(out.cpu().reshape(-1, 2048), pages)
            # the oracle decodes the same pages one by one
            for i in ids[:5].tolist():
                rc, pg, _ = o.decompress_chunk(want, i, 2048)
                assert rc == o.OK and np.array_equal(pg, pages[ids.tolist().index(i)].numpy())


def test_bf16_kv_pages_random_access():
    # the same cache in BF16: pages of 16 tokens x 128 values = 4 KiB; whole-tensor decode, a random quarter of the
    # pages decoded densely (also through the batch calls), a delta against the previous step's cache, ids out of range
    k, v = wl.bf16_kv_pair(batch=1, heads=4, tokens=1024, seed=15)
    for name, t in (("K", k), ("V", v)):
        flat = t.reshape(-1)
        n = flat.numel()
        raw = flat.view(torch.uint8).reshape(-1)
        for S in (8, 32, 4):
            for limit in ((0, 0, 0), (8, 0, 0)):              # longest exponent codes beyond and within 8 bits
                want, _, _ = check_case(zc.FMT_BF16, n, 4096, S, zc.POLICY_AUTO, limit, data=(raw, None), tag="bf16-pages-" + name)
            n_pages = n * 2 // 4096
            ids = wl.page_sample(n_pages, 0.25, seed=S)
            comp = torch.from_numpy(want).to(DEV)
            info = zc.read_info(comp)
            out, _ = zc.decompress_chunks(comp, info, ids.to(DEV))
            torch.cuda.synchronize()
            pages = raw.reshape(n_pages, 4096)[ids.long()]
            assert torch.equal(out.cpu().reshape(-1, 4096), pages)
            for i in ids[:3].tolist():
                rc, pg, _ = o.decompress_chunk(want, i, 4096)
                assert rc == o.OK and np.array_equal(pg, pages[ids.tolist().index(i)].numpy())
            # ids beyond the tensor leave their slots alone
            bad = torch.tensor([1, n_pages + 7, 0], dtype=torch.int32)
            outb = torch.full((3 * 4096,), 0x5A, dtype=torch.uint8, device=DEV)
            zc.decompress_chunks(comp, info, bad.to(DEV), out=outb)
            torch.cuda.synchronize()
            outb = outb.cpu().reshape(3, 4096)
            assert torch.equal(outb[0], raw[4096:8192]) and torch.equal(outb[2], raw[:4096]) and bool((outb[1] == 0x5A).all())
    # delta of V against K (any base will do), ragged length, page-sized chunks
    a, b = k.reshape(-1).view(torch.uint8).reshape(-1)[:41 * 4096 + 6], v.reshape(-1).view(torch.uint8).reshape(-1)[:41 * 4096 + 6]
    check_case(zc.FMT_BF16, a.numel() // 2, 4096, 16, data=(a, None), base=b, tag="bf16-pages-delta")
    # the batch calls with an id list per tensor
    srcs = [k.reshape(-1).view(torch.uint8).reshape(-1), v.reshape(-1).view(torch.uint8).reshape(-1)]
    bt = zc.Batch([dev(x) for x in srcs], [x.numel() // 2 for x in srcs], zc.params(zc.FMT_BF16, 4096, streams=8, policy=zc.POLICY_AUTO))
    bt.compress()
    idl = [wl.page_sample(x.numel() // 4096, 0.25, seed=40 + i) for i, x in enumerate(srcs)]
    bt.set_chunk_ids([dev(i) for i in idl])
    bt.plan_decompress()
    bt.run_decompress()
    torch.cuda.synchronize()
    for x, i, out in zip(srcs, idl, bt.out):
        assert torch.equal(out.cpu().reshape(-1, 4096), x.reshape(-1, 4096)[i.long()])


def test_random_access_with_short_last_chunk_and_bad_ids():
    n, cb = 10 * 4096 + 100, 4096
    x = wl.fp8_weight(n, seed=9)
    comp, info = zc.compress(x.to(DEV), n, zc.params(zc.FMT_FP8_E4M3, cb, streams=16))
    ids = torch.tensor([10, 0, 99, 3, 10], dtype=torch.int32)
    out = torch.full((5 * cb,), 0xA5, dtype=torch.uint8, device=DEV)
    zc.decompress_chunks(comp, info, ids.to(DEV), out=out)
    torch.cuda.synchronize()
    out = out.cpu().reshape(5, cb)
    assert torch.equal(out[0, :100], x[10 * cb:]) and bool((out[0, 100:] == 0xA5).all())
    assert torch.equal(out[1], x[:cb]) and torch.equal(out[3], x[3 * cb:4 * cb]) and torch.equal(out[4], out[0])
    assert bool((out[2] == 0xA5).all())          # id out of range: slot untouched


def test_modes_const_two_valued_uniform_and_binding_limit():
    n = 50000
    rng = np.random.default_rng(12)
    x = torch.full((n,), 0x38, dtype=torch.uint8)
    check_case(zc.FMT_FP8_E4M3, n, 4096, 64, data=(x, None), tag="const")
    x = torch.where(torch.arange(n) % 3 == 0, 0x38, 0x40).to(torch.uint8)
    check_case(zc.FMT_FP8_E4M3, n, 4096, 64, data=(x, None), tag="two-valued")
    x = torch.from_numpy(rng.integers(0, 256, n).astype(np.uint8))
    check_case(zc.FMT_FP8_E4M3, n, 4096, 64, data=(x, None), tag="uniform")
    check_case(zc.FMT_FP8_E4M3, n, 4096, 64, policy=zc.POLICY_AUTO, data=(x, None), tag="uniform-auto")
    check_case(zc.FMT_BF16, n // 2, 4096, 64, data=(x, None), tag="uniform-bf16")
    pr = np.exp2(-np.arange(1, 17, dtype=float)); pr /= pr.sum()
    e = rng.choice(16, size=n, p=pr).astype(np.uint8)
    x = torch.from_numpy(((e << 3) | rng.integers(0, 8, n).astype(np.uint8)).astype(np.uint8))
    for L in (4, 5, 6, 8, 15):
        check_case(zc.FMT_FP8_E4M3, n, 8192, 64, L=(L, L, 0), data=(x, None), tag="limit%d" % L)
    # 256-symbol alphabet with geometric weights: code lengths up to 16 on both BF16 fields
    pr = np.exp2(-np.minimum(np.arange(1, 257, dtype=float), 30) * 0.7); pr /= pr.sum()
    a = rng.choice(256, size=n, p=pr).astype(np.uint16)
    b = rng.choice(256, size=n, p=pr[::-1]).astype(np.uint16)
    w = (((b & 0x80) << 8) | (a << 7) | (b & 0x7F)).astype(np.uint16)
    x = torch.from_numpy(w.view(np.uint8).copy())
    for L in (16, 12, 9):
        check_case(zc.FMT_BF16, n, 16384, 64, L=(L, L, 0), data=(x, None), tag="bf16-limit%d" % L)


def test_batch_round_trip_and_parity():
    shapes = [70000, 1, 262144 * 2, 262144 + 5, 16, 300001]
    srcs = [wl.fp8_weight(n, seed=50 + i) for i, n in enumerate(shapes)]
    p = zc.params(zc.FMT_FP8_E4M3, 262144)
    b = zc.Batch([s.to(DEV) for s in srcs], shapes, p)
    sizes = b.compress()
    for i, n in enumerate(shapes):
        want = o.compress(srcs[i].numpy(), n, o.params(o.FP8_E4M3, 262144))
        assert sizes[i] == len(want)
        assert np.array_equal(b.container(i).cpu().numpy(), want), i
    outs = b.decompress()
    torch.cuda.synchronize()
    for i, n in enumerate(shapes):
        assert torch.equal(outs[i].cpu()[:n], srcs[i])
    # second pass reuses every buffer and gives the same bytes (no stale state in the workspace)
    for o_ in outs:
        o_.fill_(0xA5)
    sizes2 = b.compress()
    outs = b.decompress()
    torch.cuda.synchronize()
    assert sizes2 == sizes
    for i, n in enumerate(shapes):
        assert torch.equal(outs[i].cpu()[:n], srcs[i])


def test_batch_other_formats_and_mixed_tensors():
    # the batch calls on MXFP4 (chunks shared by four wavefronts in both directions), on BF16 with a delta, and on
    # a BF16 batch whose tensors take different kernels (compressible exponents, constant tensor, uniform noise,
    # a tensor shorter than a chunk): every container is the oracle's, every tensor comes back
    cb = 16384
    mats = [wl.mxfp4_weight(64, 512 * (3 + i), seed=60 + i) for i in range(3)]
    ns = [64 * 512 * (3 + i) for i in range(3)]
    p = zc.params(zc.FMT_FP4_E2M1_MX, cb, streams=64, policy=zc.POLICY_AUTO)
    po = o.params(o.FP4_E2M1_MX, cb, streams=64, policy=o.POLICY_AUTO)
    b = zc.Batch([dev(m[0]) for m in mats], ns, p, scales=[dev(m[1]) for m in mats])
    sizes = b.compress()
    for i, n in enumerate(ns):
        want = o.compress(mats[i][0].numpy(), n, po, scales=mats[i][1].numpy())
        assert sizes[i] == len(want) and np.array_equal(b.container(i).cpu().numpy(), want), i
    outs = b.decompress()
    torch.cuda.synchronize()
    for i, n in enumerate(ns):
        assert torch.equal(outs[i].cpu()[:n // 2], mats[i][0]) and torch.equal(b.scales_out[i].cpu()[:n // 32], mats[i][1])
    # BF16: a delta batch
    pairs = [wl.bf16_checkpoint_pair(40000 + 777 * i, seed=70 + i) for i in range(3)]
    raw = [[x.view(torch.uint8).reshape(-1) for x in pr] for pr in pairs]
    ns = [pr[0].numel() for pr in pairs]
    p, po = zc.params(zc.FMT_BF16, 8192), o.params(o.BF16, 8192)
    b = zc.Batch([dev(r[1]) for r in raw], ns, p, xor_bases=[dev(r[0]) for r in raw])
    sizes = b.compress()
    for i, n in enumerate(ns):
        want = o.compress(raw[i][1].numpy(), n, po, xor_base=raw[i][0].numpy())
        assert sizes[i] == len(want) and np.array_equal(b.container(i).cpu().numpy(), want), i
    outs = b.decompress()
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(outs[i].cpu()[:raw[i][1].numel()], raw[i][1])
    # BF16: tensors of different character in one batch
    rng = np.random.default_rng(8)
    srcs = [wl.bf16_weight(5 * 4096 + 11, seed=80).view(torch.uint8).reshape(-1),
            torch.full((3 * 4096 * 2,), 0x3C, dtype=torch.uint8),
            torch.from_numpy(rng.integers(0, 256, 4 * 4096 * 2, dtype=np.uint8)),
            wl.bf16_weight(100, seed=81).view(torch.uint8).reshape(-1)]
    ns = [s.numel() // 2 for s in srcs]
    for policy, opolicy in ((zc.POLICY_HUFF_ALL, o.POLICY_HUFF_ALL), (zc.POLICY_AUTO, o.POLICY_AUTO)):
        p, po = zc.params(zc.FMT_BF16, 8192, policy=policy), o.params(o.BF16, 8192, policy=opolicy)
        b = zc.Batch([dev(s) for s in srcs], ns, p)
        sizes = b.compress()
        for i, n in enumerate(ns):
            want = o.compress(srcs[i].numpy(), n, po)
            assert sizes[i] == len(want) and np.array_equal(b.container(i).cpu().numpy(), want), (policy, i)
        outs = b.decompress()
        torch.cuda.synchronize()
        for i in range(len(srcs)):
            assert torch.equal(outs[i].cpu()[:srcs[i].numel()], srcs[i]), (policy, i)


def test_errors():
    x = wl.fp8_weight(9000, seed=22).to(DEV)
    p = zc.params(zc.FMT_FP8_E4M3, 4096)
    comp, info = zc.compress(x, 9000, p)
    bad = comp.clone(); bad[0] = 0x5B
    with pytest.raises(zc.ZcError) as e:
        zc.read_info(bad)
    assert e.value.status == zc.ERR_CORRUPT
    bad = comp.clone(); bad[64] = 0            # incomplete code
    with pytest.raises(zc.ZcError):
        zc.read_info(bad)
    bad = comp.clone(); bad[100:104] = 0xFF    # chunk offsets out of order
    with pytest.raises(zc.ZcError):
        zc.read_info(bad, check_index=True)
    with pytest.raises(zc.ZcError) as e:
        zc.decompress(comp, info, out=torch.empty(8992, dtype=torch.uint8, device=DEV))
    assert e.value.status == zc.ERR_BUFFER_TOO_SMALL
    with pytest.raises(zc.ZcError) as e:
        zc.compress(x, 9000, p, dst=torch.empty(4096, dtype=torch.uint8, device=DEV))
    assert e.value.status == zc.ERR_BUFFER_TOO_SMALL
    with pytest.raises(zc.ZcError) as e:
        zc.compress(x[1:], 8000, p)              # misaligned source
    assert e.value.status == zc.ERR_INVALID_ARG
    # a delta container cannot be decoded without its base
    w0, w1 = wl.bf16_checkpoint_pair(5000, seed=1)
    comp, info = zc.compress(w1.to(DEV), 5000, zc.params(zc.FMT_BF16, 4096), xor_base=w0.to(DEV))
    with pytest.raises(zc.ZcError):
        zc.decompress(comp, info)


def test_decompress_reads_the_header_itself():
    # zc_decompress / zc_decompress_chunks without a zc_info: the library reads and validates the header first
    for fmt, n, cb, S in ((zc.FMT_FP8_E4M3, 5 * 4096 + 77, 4096, 64), (zc.FMT_BF16, 3 * 2048 + 5, 4096, 8),
                          (zc.FMT_FP4_E2M1_MX, 32 * 700, 1024, 64)):
        src, sc = make_input(fmt, n, 41)
        comp, info = zc.compress(dev(src), n, zc.params(fmt, cb, streams=S), scales=dev(sc))
        out, sco = zc.decompress(comp, read_header_in_call=True)
        torch.cuda.synchronize()
        assert torch.equal(out.cpu()[:src.numel()], src.view(torch.uint8).reshape(-1))
        if sc is not None:
            assert torch.equal(sco.cpu()[:sc.numel()], sc)
    bad = comp.clone(); bad[1] = 0x00
    with pytest.raises(zc.ZcError) as e:
        zc.decompress(bad, info, read_header_in_call=True)
    assert e.value.status == zc.ERR_CORRUPT


def test_container_description_that_was_never_filled_in_is_refused():
    # the *_async compress calls leave info.total_bytes at 0; a decode call handed that description must say so
    # instead of returning success with nothing decoded
    srcs = [wl.fp8_weight(6 * 2048, seed=61), wl.fp8_weight(9 * 2048, seed=62)]
    p = zc.params(zc.FMT_FP8_E4M3, 2048, streams=8)
    code = zc.train_code(dev(srcs[0]), srcs[0].numel(), p)
    bt = zc.Batch([dev(s) for s in srcs], [s.numel() for s in srcs], p)
    bt.compress(code=code)                                  # fills info
    bt.compress_async(code)                                 # leaves total_bytes 0
    torch.cuda.synchronize()
    assert bt.arr[0].info.total_bytes == 0
    bt.prepare_outputs()
    for o_ in bt.out:
        o_.fill_(0xEE)
    st = zc.lib().zc_decompress_batch(bt.arr, bt.n, zc._ptr(bt.ws), bt.ws.numel(), zc._stream())
    assert st == zc.ERR_INVALID_ARG
    plan = zc.BatchPlan()
    st = zc.lib().zc_decompress_batch_plan(bt.arr, bt.n, zc._ptr(bt.ws_plan), bt.ws_plan.numel(), C_byref(plan), zc._stream())
    assert st == zc.ERR_INVALID_ARG
    stale = bt.arr[0].info
    with pytest.raises(zc.ZcError) as e:
        zc.decompress(bt.comp[0], stale)
    assert e.value.status == zc.ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert all(bool((o_ == 0xEE).all()) for o_ in bt.out)
    # other descriptions that cannot belong to a container
    good = zc.read_info(bt.comp[0])
    for field, value in (("chunk_bytes", 0), ("chunk_bytes", 2040), ("n_chunks", good.n_chunks + 1), ("streams", 3),
                         ("payload_offset", 0), ("total_bytes", bt.comp[0].numel() + 16)):
        broken = zc.Info.from_buffer_copy(good)
        setattr(broken, field, value)
        with pytest.raises(zc.ZcError) as e:
            zc.decompress(bt.comp[0], broken)
        assert e.value.status == zc.ERR_INVALID_ARG, field
    # once the headers have been read back the same batch decodes
    bt.refresh_info()
    outs = bt.decompress()
    torch.cuda.synchronize()
    for out, s_ in zip(outs, srcs):
        assert torch.equal(out.cpu()[:s_.numel()], s_)


def test_determinism_and_poisoned_buffers():
    n = 500000
    x = wl.fp8_weight(n, seed=31).to(DEV)
    p = zc.params(zc.FMT_FP8_E4M3, 65536)
    ref = None
    for fill in (0x00, 0xA5, 0xFF):
        dst = torch.full((zc.compress_bound(n, p),), fill, dtype=torch.uint8, device=DEV)
        ws = torch.full((zc.workspace_bytes([n], p),), fill, dtype=torch.uint8, device=DEV)
        comp, info = zc.compress(x, n, p, dst=dst, ws=ws)
        out = torch.full((n,), fill, dtype=torch.uint8, device=DEV)
        zc.decompress(comp, info, out=out)
        torch.cuda.synchronize()
        assert torch.equal(out, x)
        if ref is None:
            ref = comp.clone()
        assert torch.equal(comp, ref)


def test_fp8_fast_path_variants():
    # the specialised FP8 kernel: single / pair lookups x flat / raw sign+mantissa x delta,
    # whole chunks through it and a short last chunk through the generic kernel
    n = 37 * 65536 + 12345
    x = wl.fp8_weight(n, seed=61)
    y = wl.fp8_weight(n, seed=62)
    for L in (8, 7, 6, 5):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E4M3, n, 65536, 64, policy, L=(L, 0, 0), data=(x, None), tag="fast-L%d" % L)
            check_case(zc.FMT_FP8_E4M3, n, 65536, 64, policy, L=(L, 0, 0), data=(x, None), base=y, tag="fast-xor-L%d" % L)
    # worst case for the window: every code 8 bits long for long stretches (16 equiprobable
    # exponents would be flat, so skew the histogram just enough to get lengths up to 8)
    rng = np.random.default_rng(63)
    pr = np.array([2.0 ** -min(k + 1, 8) for k in range(16)]); pr /= pr.sum()
    e = rng.choice(16, size=n, p=pr).astype(np.uint8)
    e[1000:200000] = 15                       # long runs of the rarest symbols
    e[300000:400000] = np.where(rng.random(100000) < 0.5, 14, 15)
    z = torch.from_numpy(((e << 3) | rng.integers(0, 8, n).astype(np.uint8)).astype(np.uint8))
    want, _, _ = check_case(zc.FMT_FP8_E4M3, n, 65536, 64, L=(8, 0, 0), data=(z, None), tag="fast-worst")


def test_config2_full_size_tensors_in_the_benchmark_launch_configuration():
    # One full layer of config 2 at its real sizes (q, o: 16 MiB; k, v: 4 MiB; gate, up, down: 56 MiB), generated
    # on the GPU exactly as bench.py does, compressed and decoded as one batch (the launch
    # configuration bench.py times).  The oracle compresses the same bytes: containers must be
    # identical; then sampled chunks of the oracle's container are decoded one by one on the CPU
    # and compared with the GPU output.
    shapes = [(name, r * c) for name, r, c in wl.LAYER_8B]
    dev_srcs = [wl.fp8_weight(n, device=DEV, seed=2000 + i) for i, (_, n) in enumerate(shapes)]
    counts = [n for _, n in shapes]
    p = zc.params(zc.FMT_FP8_E4M3, 262144, streams=64)
    b = zc.Batch(dev_srcs, counts, p)
    sizes = b.compress()
    outs = b.decompress()
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    for i, (name, n) in enumerate(shapes):
        print("full-size", name, n, flush=True)
        host = dev_srcs[i].cpu().numpy()
        want = o.compress(host, n, o.params(o.FP8_E4M3, 262144, streams=64))
        got = b.container(i).cpu().numpy()
        assert sizes[i] == len(want) and np.array_equal(got, want), name
        gpu_out = outs[i].cpu().numpy()
        assert np.array_equal(gpu_out[:n], host)
        n_chunks = n // 262144
        for c in sorted(set([0, n_chunks - 1] + rng.integers(0, n_chunks, 4).tolist())):
            rc, chunk, _ = o.decompress_chunk(want, c, 262144)
            assert rc == o.OK and np.array_equal(chunk, gpu_out[c * 262144:(c + 1) * 262144]), (name, c)


def test_configs_3_4_5_full_size_tensors_in_the_benchmark_launch_configuration():
    # One tensor each of configurations 3, 4 (W1 alone and the delta) and 5 at its real size, generated on the
    # GPU as bench.py does and compressed / decoded in a batch with the parameters bench.py times.  The
    # oracle compresses the same bytes: identical containers; sampled chunks of the oracle's container,
    # decoded one by one on the CPU, equal the GPU output; the K/V page list decodes to the sampled pages.
    rng = np.random.default_rng(8)

    def compare(tag, fmt, srcs, n, cb, S, limit, bases=None, scales=None, ids=None):
        p, po = zc.params(fmt, cb, limit, S), o.params(fmt, cb, limit, S)
        b = zc.Batch(srcs, [n] * len(srcs), p, xor_bases=bases, scales=scales)
        sizes = b.compress()
        b.plan_decompress()
        outs = b.run_decompress()
        torch.cuda.synchronize()
        print("full-size", tag, n, flush=True)
        host = srcs[0].view(torch.uint8).reshape(-1).cpu().numpy()
        hb = None if bases is None else bases[0].view(torch.uint8).reshape(-1).cpu().numpy()
        hs = None if scales is None else scales[0].cpu().numpy()
        want = o.compress(host, n, po, xor_base=hb, scales=hs)
        assert sizes[0] == len(want) and np.array_equal(b.container(0).cpu().numpy(), want), tag
        for i, s_ in enumerate(srcs):
            assert torch.equal(outs[i][:s_.numel() * s_.element_size()], s_.view(torch.uint8).reshape(-1)), (tag, i)
        gpu_out = outs[0].cpu().numpy()
        n_chunks = len(host) // cb
        n_sc = 0 if scales is None else cb * 8 // zc.elem_bits(fmt) // zc.scale_block(fmt)
        for c in sorted(set([0, n_chunks - 1] + rng.integers(0, n_chunks, 4).tolist())):
            rc, chunk, sc = o.decompress_chunk(want, c, cb, xor_base_chunk=None if hb is None else hb[c * cb:(c + 1) * cb], n_scales=n_sc)
            assert rc == o.OK and np.array_equal(chunk, gpu_out[c * cb:(c + 1) * cb]), (tag, c)
            if n_sc:
                assert np.array_equal(sc, b.scales_out[0].cpu().numpy()[c * n_sc:(c + 1) * n_sc]), (tag, c)
        if ids is not None:
            b.set_chunk_ids(ids)
            b.plan_decompress()
            outs = b.run_decompress()
            torch.cuda.synchronize()
            for i, s_ in enumerate(srcs):
                assert torch.equal(outs[i].view(-1, cb), s_.view(torch.uint8).view(-1, cb)[ids[i].long()]), (tag, "pages", i)

    m = [wl.mxfp4_weight(8192, 28672, device=DEV, seed=300 + i) for i in range(2)]
    compare("c3", zc.FMT_FP4_E2M1_MX, [x[0] for x in m], 8192 * 28672, 262144, 64, (0, 0, 0), scales=[x[1] for x in m])
    del m
    pairs = [wl.bf16_checkpoint_pair(4096 * 16384, device=DEV, seed=400 + i) for i in range(2)]
    w0, w1 = [q[0] for q in pairs], [q[1] for q in pairs]
    compare("c4-w1", zc.FMT_BF16, w1, 4096 * 16384, 262144, 64, (16, 16, 0))
    compare("c4-delta", zc.FMT_BF16, w1, 4096 * 16384, 262144, 64, (16, 16, 0), bases=w0)
    del pairs, w0, w1
    k, v = wl.fp8_kv_pair(device=DEV, seed=500)
    kv = [k.reshape(-1), v.reshape(-1)]
    n_pages = kv[0].numel() // 2048
    ids = [wl.page_sample(n_pages, 0.25, device=DEV, seed=600 + i) for i in range(2)]
    compare("c5", zc.FMT_FP8_E4M3, kv, kv[0].numel(), 2048, 8, (0, 0, 0), ids=ids)


def test_full_chunk_kernel_all_formats_and_kinds():
    # the 64-lane full-chunk decoder: every format, table-decoded / flat / raw / constant fields,
    # one or two LDS rings, delta, chunks that are whole multiples of its row size
    rng = np.random.default_rng(71)
    # FP4 with skewed element fields (mostly small magnitudes) so that exponent and sign+mantissa
    # get real Huffman codes, and few distinct scales
    n = 5 * 32768 + 32 * 77
    nib = rng.choice(16, size=n, p=np.array([40, 20, 8, 4, 2, 1, 1, 1, 10, 5, 3, 2, 1, 1, 0.5, 0.5]) / 100.0).astype(np.uint8)
    packed = torch.from_numpy((nib[0::2] | (nib[1::2] << 4)).astype(np.uint8))
    scales = torch.from_numpy(rng.choice([118, 119, 120, 121, 127], size=n // 32, p=[0.5, 0.3, 0.1, 0.05, 0.05]).astype(np.uint8))
    for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
        check_case(zc.FMT_FP4_E2M1_MX, n, 16384, 64, policy, data=(packed, scales), tag="fp4-skewed")
    flat_nib = rng.integers(0, 16, n).astype(np.uint8)
    packed2 = torch.from_numpy((flat_nib[0::2] | (flat_nib[1::2] << 4)).astype(np.uint8))
    const_scales = torch.full((n // 32,), 119, dtype=torch.uint8)
    check_case(zc.FMT_FP4_E2M1_MX, n, 16384, 64, data=(packed2, const_scales), tag="fp4-flat-constscale")
    check_case(zc.FMT_FP4_E2M1_MX, n, 32768, 64, zc.POLICY_AUTO, data=(packed2, scales), tag="fp4-raw")
    # BF16: plain weights (exponent table decoded, sign+mantissa flat) and a delta with both fields table decoded
    m = 9 * 8192 + 4097
    w0, w1 = wl.bf16_checkpoint_pair(m, seed=72)
    w0, w1 = w0.view(torch.uint8), w1.view(torch.uint8)
    for cb in (1024, 16384):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_BF16, m, cb, 64, policy, data=(w1, None), tag="bf16-plain")
            check_case(zc.FMT_BF16, m, cb, 64, policy, data=(w1, None), base=w0, tag="bf16-delta")
    # identical checkpoints: the delta is all zero, both fields constant
    check_case(zc.FMT_BF16, m, 16384, 64, data=(w1, None), base=w1, tag="bf16-zero-delta")
    # FP8 with exponent codes longer than 8 bits (not the specialised FP8 kernel) and both fields skewed
    pr = np.exp2(-np.arange(1, 17, dtype=float)); pr /= pr.sum()
    k = 20 * 4096 + 100
    e = rng.choice(16, size=k, p=pr).astype(np.uint8)
    sm = rng.choice(16, size=k, p=pr[::-1]).astype(np.uint8)
    x = torch.from_numpy((((sm >> 3) << 7) | (e << 3) | (sm & 7)).astype(np.uint8))
    for L in (15, 12, 9):
        check_case(zc.FMT_FP8_E4M3, k, 4096, 64, L=(L, L, 0), data=(x, None), tag="fp8-long-L%d" % L)


def test_fp8_short_exponent_codes_take_the_general_path():
    # longest exponent code below 5 bits -> refill period 8 or 16: not the period-4 FP8 kernels
    rng = np.random.default_rng(81)
    n = 11 * 4096 + 300
    for probs in ([0.6, 0.25, 0.1, 0.05], [0.9, 0.1], [0.3, 0.3, 0.2, 0.1, 0.05, 0.05]):
        e = rng.choice(len(probs), size=n, p=probs).astype(np.uint8) + 5
        x = torch.from_numpy(((e << 3) | rng.integers(0, 8, n).astype(np.uint8) | (rng.integers(0, 2, n).astype(np.uint8) << 7)).astype(np.uint8))
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E4M3, n, 4096, 64, policy, data=(x, None), tag="fp8-short-%d" % len(probs))


def test_batched_page_decode():
    # a whole (small) K/V cache: every tensor's page sample decoded densely in one launch
    tensors = []
    for layer in range(3):
        k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=512, seed=90 + layer)
        tensors += [k.reshape(-1), v.reshape(-1)]
    counts = [t.numel() for t in tensors]
    n_pages = counts[0] // 2048
    for S in (8, 16):
        b = zc.Batch([t.to(DEV) for t in tensors], counts, zc.params(zc.FMT_FP8_E4M3, 2048, streams=S))
        b.compress()
        ids = [wl.page_sample(n_pages, 0.25, seed=S * 100 + i) for i in range(len(tensors))]
        b.set_chunk_ids([i.to(DEV) for i in ids])
        outs = b.decompress()
        torch.cuda.synchronize()
        for i, t in enumerate(tensors):
            want = t.reshape(n_pages, 2048)[ids[i].long()]
            assert torch.equal(outs[i].cpu().reshape(-1, 2048), want), (S, i)
        # and back to whole tensors with the same batch object
        b.set_chunk_ids(None)
        outs = b.decompress()
        torch.cuda.synchronize()
        for i, t in enumerate(tensors):
            assert torch.equal(outs[i].cpu()[:counts[i]], t)


def test_odd_geometries():
    # chunk sizes that are not whole rows of any specialised kernel, every lane count, ragged sizes
    for fmt, cbs in ((zc.FMT_FP8_E4M3, (16, 1008, 48 * 1024 + 16)), (zc.FMT_BF16, (16, 2064)), (zc.FMT_FP4_E2M1_MX, (256, 768))):
        for cb in cbs:
            for S in (2, 4, 16, 32, 64):
                E = cb * 8 // zc.elem_bits(fmt)
                n = 5 * E + (E // 3 // 32) * 32 + (0 if fmt == zc.FMT_FP4_E2M1_MX else 7)
                check_case(fmt, n, cb, S, zc.POLICY_HUFF_ALL if S != 16 else zc.POLICY_AUTO, tag="odd")


def test_damaged_payload_and_index_do_not_escape_the_buffers():
    # The decoders' own range checks must turn a damaged stream into wrong output, never into an
    # access outside the container or the destination: canaries around both stay intact.
    rng = np.random.default_rng(91)
    H, A = zc.POLICY_HUFF_ALL, zc.POLICY_AUTO
    cases = [(zc.FMT_FP8_E4M3, 8 * 65536, 65536, 64, H, False), (zc.FMT_FP8_E4M3, 64 * 2048, 2048, 8, H, False),
             (zc.FMT_BF16, 6 * 8192, 16384, 64, H, False), (zc.FMT_FP8_E4M3, 9 * 4096 + 11, 4096, 16, H, False),
             # BF16 pages (the page decoder's BF16 kernel), a BF16 delta with both fields table decoded and long
             # codes (the paired decode), an FP8 page delta
             (zc.FMT_BF16, 24 * 2048, 4096, 8, A, False), (zc.FMT_BF16, 5 * 131072, 262144, 64, H, True),
             (zc.FMT_FP8_E4M3, 64 * 2048, 2048, 8, A, True),
             # the E5M2 kernel, and the BF16 64-lane kernel with a raw sign+mantissa field
             (zc.FMT_FP8_E5M2, 8 * 65536, 65536, 64, H, False), (zc.FMT_BF16, 6 * 8192, 16384, 64, A, False),
             # 64 lanes with a short last chunk, and with a chunk size that is not whole rows (the build for such chunks)
             (zc.FMT_FP8_E4M3, 5 * 65536 + 1234, 65536, 64, H, False), (zc.FMT_BF16, 3 * 12296 + 777, 24592, 64, H, False),
             (zc.FMT_FP8_E4M3_BYTES, 4 * 49168 + 50, 49168, 64, A, False)]
    for fmt, n, cb, S, policy, delta in cases:
        if delta and fmt == zc.FMT_BF16:
            w0, w1 = wl.bf16_checkpoint_pair(n, seed=23)
            src, base = w1.view(torch.uint8).reshape(-1), w0.view(torch.uint8).reshape(-1)
        else:
            src, _sc = make_input(fmt, n, 17)
            base = make_input(fmt, n, 18)[0] if delta else None
        comp, info = zc.compress(dev(src), n, zc.params(fmt, cb, streams=S, policy=policy), xor_base=dev(base))
        if fmt == zc.FMT_BF16 and delta:
            assert info.mode[0] == zc.MODE_HUFF and info.mode[1] == zc.MODE_HUFF and info.max_len[1] > 11
        raw = src.numel() * src.element_size()
        pay = int(info.payload_offset)
        for what in ("payload", "index"):
            guard = 4096
            buf = torch.full((guard + comp.numel() + guard,), 0x5A, dtype=torch.uint8, device=DEV)
            body = buf[guard:guard + comp.numel()]
            body.copy_(comp)
            if what == "payload":
                noise = torch.from_numpy(rng.integers(0, 256, comp.numel() - pay).astype(np.uint8)).to(DEV)
                body[pay:] = noise
            else:
                lo = int(info.index_offset[0])
                body[lo:pay] = torch.from_numpy(rng.integers(0, 256, pay - lo).astype(np.uint8)).to(DEV)
            out = torch.full((guard + raw + guard,), 0xC3, dtype=torch.uint8, device=DEV)
            print("damaged", what, "fmt", fmt, "n", n, "chunk", cb, "S", S, "policy", policy, "delta", delta, flush=True)
            zc.decompress(body, info, out=out[guard:guard + raw], xor_base=dev(base))
            torch.cuda.synchronize()
            assert bool((out[:guard] == 0xC3).all()) and bool((out[guard + raw:] == 0xC3).all())
            assert bool((buf[:guard] == 0x5A).all()) and bool((buf[guard + comp.numel():] == 0x5A).all())


def test_static_dictionary():
    # dictionary trained on one tensor, applied to others: same dictionary and same container bytes as the oracle
    for fmt, n_a, n_b, cb, S in ((zc.FMT_FP8_E4M3, 300000, 5 * 65536 + 777, 65536, 64), (zc.FMT_FP8_E4M3, 64 * 2048, 96 * 2048, 2048, 8),
                                 (zc.FMT_BF16, 100000, 70001, 16384, 64), (zc.FMT_FP4_E2M1_MX, 32 * 4000, 32 * 5001, 16384, 64)):
        a, sa = make_input(fmt, n_a, 41)
        b, sb_ = make_input(fmt, n_b, 42)
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            print("dictionary fmt", fmt, "policy", policy, flush=True)
            p, po = zc.params(fmt, cb, streams=S, policy=policy), o.params(fmt, cb, streams=S, policy=policy)
            code = zc.train_code(dev(a), n_a, p, scales=dev(sa))
            ln, md = o.train_code(a.numpy(), n_a, po, scales=None if sa is None else sa.numpy())
            for f in range(code.n_fields):
                assert list(code.code_len[f]) == ln[f].tolist() and code.mode[f] == md[f]
            # the dictionary records what its own training tensor costs under it
            assert code.n_elems == n_a and code.total_bytes == len(o.compress_with_code(a.numpy(), n_a, po, ln, md, scales=None if sa is None else sa.numpy()))
            want = o.compress_with_code(b.numpy(), n_b, po, ln, md, scales=None if sb_ is None else sb_.numpy())
            comp, info = zc.compress_with_code(dev(b), n_b, p, code, scales=dev(sb_))
            assert np.array_equal(comp.cpu().numpy(), want)
            out, sco = zc.decompress(comp, info)
            torch.cuda.synchronize()
            assert torch.equal(out.cpu()[:b.numel() * b.element_size()], b.view(torch.uint8).reshape(-1))
            assert not zc.code_stale(code, info, 0.02)      # same distribution: no refresh
    # refresh test: data of another distribution compresses worse under the dictionary than the training data did
    p = zc.params(zc.FMT_FP8_E4M3, 65536)
    a = wl.fp8_weight(1 << 20, seed=50)
    k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=4096, seed=51)
    code = zc.train_code(dev(a), a.numel(), p)
    _, info_k = zc.compress_with_code(dev(k.reshape(-1)), k.numel(), p, code)
    want_k = o.compress_with_code(k.reshape(-1).numpy(), k.numel(), o.params(o.FP8_E4M3, 65536), *o.train_code(a.numpy(), a.numel(), o.params(o.FP8_E4M3, 65536)))
    assert info_k.total_bytes == len(want_k)
    assert zc.code_stale(code, info_k, 0.02) == (len(want_k) / k.numel() > code.total_bytes / a.numel() + 0.02)
    assert zc.code_stale(code, info_k, 0.02)
    # a dictionary that cannot code every symbol is refused
    fmt, n_a, cb, S = zc.FMT_FP4_E2M1_MX, 32 * 4000, 16384, 64
    a, sa = make_input(fmt, n_a, 41)
    p = zc.params(fmt, cb, streams=S, policy=zc.POLICY_HUFF_ALL)
    code = zc.train_code(dev(a), n_a, p, scales=dev(sa))
    assert code.mode[0] == zc.MODE_HUFF
    code.code_len[0][2] = 0
    with pytest.raises(zc.ZcError):
        zc.compress_with_code(dev(b), n_b, p, code, scales=dev(sb_))


def test_dictionary_compress_of_few_pages_in_one_kernel():
    # dictionary calls over FP8 or BF16 tensors of at most 512 whole pages run size pass, scan and encoder as one kernel: at
    # and around that limit, every lane count of the page kernels, flat and raw sign+mantissa fields, a batch with
    # tensors of different lengths, a destination below the worst case
    for S in (4, 8, 16, 32):
        cb = 16 * S * 8
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=S, policy=policy), o.params(o.FP8_E4M3, cb, streams=S, policy=policy)
            a = wl.fp8_weight(200 * cb, seed=61)
            code = zc.train_code(dev(a), a.numel(), p)
            ln, md = o.train_code(a.numpy(), a.numel(), po)
            for pages in (1, 31, 512, 513):
                b = wl.fp8_weight(pages * cb, seed=62 + pages)
                print("few pages S", S, "policy", policy, "pages", pages, flush=True)
                want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md)
                comp, info = zc.compress_with_code(dev(b), b.numel(), p, code)
                assert np.array_equal(comp.cpu().numpy(), want) and info.total_bytes == len(want)
                out, _ = zc.decompress(comp, info)
                torch.cuda.synchronize()
                assert torch.equal(out.cpu(), b)
            # a batch, queued without a wait
            srcs = [wl.fp8_weight(k * cb, seed=70 + k) for k in (3, 512, 40, 1)]
            bt = zc.Batch([dev(x) for x in srcs], [x.numel() for x in srcs], p)
            bt.compress_async(code)
            sizes = bt.refresh_info()
            for t, x in enumerate(srcs):
                want = o.compress_with_code(x.numpy(), x.numel(), po, ln, md)
                assert sizes[t] == len(want) and np.array_equal(bt.container(t).cpu().numpy(), want)
            # a destination that holds the container but not the worst case is fine; one that does not hold it is refused
            b = wl.fp8_weight(64 * cb, seed=99)
            want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md)
            dst = torch.zeros(len(want), dtype=torch.uint8, device=DEV)
            comp, _ = zc.compress_with_code(dev(b), b.numel(), p, code, dst=dst)
            assert np.array_equal(comp.cpu().numpy(), want)
            with pytest.raises(zc.ZcError):
                zc.compress_with_code(dev(b), b.numel(), p, code, dst=torch.zeros(len(want) - 16, dtype=torch.uint8, device=DEV))
    # BF16 pages: the same kernel in its builds for an exponent refill period of 8, 4 and 2 (longest code up to 4, up to 8,
    # beyond), flat and raw sign+mantissa field, a delta; the dictionary with a 1-bit code next to long ones (last case)
    # is not this kernel's and takes the three-kernel way
    rng = np.random.default_rng(77)

    def bf16_pages(n, n_exp, skew):
        sm = rng.integers(0, 256, n).astype(np.uint16)
        pick = rng.integers(0, n_exp, n) if skew == 0 else np.minimum(rng.geometric(skew, n) - 1, 199)
        if n_exp == 201:
            pick = np.where(rng.random(n) < 0.6, 200, pick)
        ex = (pick.astype(np.uint16) * 3 + 60) & 0xFF
        return torch.from_numpy((((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)).astype(np.uint16).view(np.uint8).copy())

    for S in (4, 8, 16, 32):
        cb = 16 * S * 6
        for n_exp, skew in ((12, 0), (40, 0), (200, 0.08), (201, 0.08)):
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                p, po = zc.params(zc.FMT_BF16, cb, streams=S, policy=policy), o.params(o.BF16, cb, streams=S, policy=policy)
                a = bf16_pages(300 * cb // 2, n_exp, skew)
                code = zc.train_code(dev(a), a.numel() // 2, p)
                ln, md = o.train_code(a.numpy(), a.numel() // 2, po)
                for pages in (1, 37, 512, 513):
                    b = bf16_pages(pages * cb // 2, n_exp, skew)
                    print("few bf16 pages S", S, "exponents", n_exp, "policy", policy, "pages", pages, flush=True)
                    want = o.compress_with_code(b.numpy(), b.numel() // 2, po, ln, md)
                    comp, info = zc.compress_with_code(dev(b), b.numel() // 2, p, code)
                    assert np.array_equal(comp.cpu().numpy(), want) and info.total_bytes == len(want)
                    out, _ = zc.decompress(comp, info)
                    torch.cuda.synchronize()
                    assert torch.equal(out.cpu(), b)
                b = bf16_pages(20 * cb // 2, n_exp, skew)
                base = torch.from_numpy((rng.integers(0, 2, b.numel() // 2, dtype=np.uint16) << 15).view(np.uint8).copy())   # flips signs only
                want = o.compress_with_code(b.numpy(), b.numel() // 2, po, ln, md, xor_base=base.numpy())
                comp, info = zc.compress_with_code(dev(b), b.numel() // 2, p, code, xor_base=dev(base))
                assert np.array_equal(comp.cpu().numpy(), want)


def test_dictionary_compress_of_pages_in_one_pass():
    # containers with their fields in reverse order (ZC_FLAG_REVERSE_FIELDS): a dictionary call over whole pages sizes,
    # places and encodes them in one kernel whose workgroups hand the running sum of the exponent streams on to each
    # other.  Tensors of more pages than one workgroup takes (so that the chain has many links), around the item
    # size, several tensors per call, every lane count, flat and raw sign+mantissa fields, a delta, a call that
    # waits for nothing, a destination that is too small; BF16 pages at each refill period of the exponent field
    R = zc.FLAG_REVERSE_FIELDS
    for S in (4, 8, 16, 32):
        cb = 16 * S * 8
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=S, policy=policy, flags=R), o.params(o.FP8_E4M3, cb, streams=S, policy=policy, payload_order=1)
            a = wl.fp8_weight(200 * cb, seed=161)
            code = zc.train_code(dev(a), a.numel(), p)
            ln, md = o.train_code(a.numpy(), a.numel(), po)
            for pages in (513, 600, 1024, 4099):
                b = wl.fp8_weight(pages * cb, seed=162 + pages)
                print("one pass S", S, "policy", policy, "pages", pages, flush=True)
                want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md)
                comp, info = zc.compress_with_code(dev(b), b.numel(), p, code)
                got = comp.cpu().numpy()
                assert got.shape == want.shape and np.array_equal(got, want), int(np.argmax(got[:len(want)] != want[:len(got)]))
                assert info.total_bytes == len(want) and info.payload_order == 1
                out, _ = zc.decompress(comp, zc.read_info(comp, check_index=True))
                torch.cuda.synchronize()
                assert torch.equal(out.cpu(), b)
            # several tensors, queued without a wait; one of few pages keeps the call away from the one-workgroup kernel
            srcs = [wl.fp8_weight(k * cb, seed=170 + k) for k in (700, 3, 2048, 515, 1)]
            bt = zc.Batch([dev(x) for x in srcs], [x.numel() for x in srcs], p)
            bt.compress_async(code)
            sizes = bt.refresh_info()
            for t, x in enumerate(srcs):
                want = o.compress_with_code(x.numpy(), x.numel(), po, ln, md)
                assert sizes[t] == len(want) and np.array_equal(bt.container(t).cpu().numpy(), want), t
            bt.decompress()
            torch.cuda.synchronize()
            for t, x in enumerate(srcs):
                assert torch.equal(bt.out[t].cpu()[:x.numel()], x)
            # a delta
            b, base = wl.fp8_weight(900 * cb, seed=180), torch.from_numpy((np.random.default_rng(S).integers(0, 2, 900 * cb, dtype=np.uint8) << 7))
            want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md, xor_base=base.numpy())
            comp, _ = zc.compress_with_code(dev(b), b.numel(), p, code, xor_base=dev(base))
            assert np.array_equal(comp.cpu().numpy(), want)
            # a destination that holds the container but not the worst case is fine; one that does not hold it is refused
            b = wl.fp8_weight(640 * cb, seed=199)
            want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md)
            comp, _ = zc.compress_with_code(dev(b), b.numel(), p, code, dst=torch.zeros(len(want), dtype=torch.uint8, device=DEV))
            assert np.array_equal(comp.cpu().numpy(), want)
            with pytest.raises(zc.ZcError):
                zc.compress_with_code(dev(b), b.numel(), p, code, dst=torch.zeros(len(want) - 16, dtype=torch.uint8, device=DEV))
    # Where the pages are small enough the kernel keeps every page's exponent stream in LDS until its place is known and
    # reads the source once.  Pages of 2 KiB (a stream may take 256 words there), coded with a dictionary that was
    # trained on other data, so that the streams of some pages (the whole tensor, every third page, one page) are
    # longer than the plain field and do not fit: their work items are coded a second time.  Pages of 4 and 8 KiB,
    # which the kernel sizes first and reads twice.
    rng = np.random.default_rng(91)
    for S in (8, 16, 32):
        cb = 2048
        p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=S, flags=R), o.params(o.FP8_E4M3, cb, streams=S, payload_order=1)
        a = wl.fp8_weight(300 * cb, seed=230)
        code = zc.train_code(dev(a), a.numel(), p)
        ln, md = o.train_code(a.numpy(), a.numel(), po)
        rare = torch.from_numpy((rng.integers(0, 3, 700 * cb).astype(np.uint8) << 3) | rng.integers(0, 8, 700 * cb).astype(np.uint8))   # exponents the dictionary gives its longest codes
        usual = wl.fp8_weight(700 * cb, seed=231)
        third = usual.clone().reshape(700, cb)
        third[::3] = rare.reshape(700, cb)[::3]
        one = usual.clone().reshape(700, cb)
        one[333] = rare.reshape(700, cb)[333]
        for name, b in (("rare", rare), ("every third page", third.reshape(-1)), ("one page", one.reshape(-1)), ("usual", usual)):
            print("one pass, streams kept in LDS, S", S, name, flush=True)
            want = o.compress_with_code(b.numpy(), b.numel(), po, ln, md)
            comp, info = zc.compress_with_code(dev(b), b.numel(), p, code)
            got = comp.cpu().numpy()
            assert got.shape == want.shape and np.array_equal(got, want), int(np.argmax(got[:len(want)] != want[:len(got)]))
            out, _ = zc.decompress(comp, zc.read_info(comp, check_index=True))
            torch.cuda.synchronize()
            assert torch.equal(out.cpu(), b)
        bt = zc.Batch([dev(x) for x in (usual, rare, third.reshape(-1))], [700 * cb] * 3, p)
        bt.compress_async(code)
        sizes = bt.refresh_info()
        for t, x in enumerate((usual, rare, third.reshape(-1))):
            want = o.compress_with_code(x.numpy(), x.numel(), po, ln, md)
            assert sizes[t] == len(want) and np.array_equal(bt.container(t).cpu().numpy(), want), t
        for cb in (4096, 8192):
            p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=S, flags=R), o.params(o.FP8_E4M3, cb, streams=S, payload_order=1)
            b = wl.fp8_weight(517 * cb, seed=232)
            print("one pass, pages sized first, S", S, "page", cb, flush=True)
            code = zc.train_code(dev(a), a.numel(), p)
            ln, md = o.train_code(a.numpy(), a.numel(), po)
            comp, info = zc.compress_with_code(dev(b), b.numel(), p, code)
            assert np.array_equal(comp.cpu().numpy(), o.compress_with_code(b.numpy(), b.numel(), po, ln, md))
    # codes of their own, built on the device: the same kernel takes the tensors whose code suits it (decided on the device),
    # the generic kernels the others of the same call: here a tensor with a constant exponent field and, with the
    # limit raised to 12 bits, one whose exponent code is longer than the page kernels take
    for S, L in ((8, (0, 0, 0)), (16, (12, 0, 0)), (4, (0, 0, 0))):
        cb = 16 * S * 8
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            p, po = zc.params(zc.FMT_FP8_E4M3, cb, L, S, policy, flags=R), o.params(o.FP8_E4M3, cb, L, S, policy, payload_order=1)
            steep = np.random.default_rng(5).choice(16, size=800 * cb, p=np.exp2(-np.arange(1, 17, dtype=float)) / np.exp2(-np.arange(1, 17, dtype=float)).sum())
            srcs = [wl.fp8_weight(2000 * cb, seed=210), torch.full((700 * cb,), 0x38, dtype=torch.uint8), wl.fp8_weight(3 * cb, seed=211),
                    torch.from_numpy((steep.astype(np.uint8) << 3) | np.random.default_rng(6).integers(0, 8, 800 * cb).astype(np.uint8)), wl.fp8_weight(1031 * cb, seed=212)]
            print("one pass, own codes S", S, "L", L, "policy", policy, flush=True)
            bt = zc.Batch([dev(x) for x in srcs], [x.numel() for x in srcs], p)
            sizes = bt.compress()
            for t, x in enumerate(srcs):
                want = o.compress(x.numpy(), x.numel(), po)
                got = bt.container(t).cpu().numpy()
                assert sizes[t] == len(want) and np.array_equal(got, want), (t, int(np.argmax(got[:len(want)] != want[:len(got)])))
            bt.decompress()
            torch.cuda.synchronize()
            for t, x in enumerate(srcs):
                assert torch.equal(bt.out[t].cpu()[:x.numel()], x), t
            bt.compress_async()
            assert bt.refresh_info() == sizes
            for t, x in enumerate(srcs):
                assert np.array_equal(bt.container(t).cpu().numpy(), o.compress(x.numpy(), x.numel(), po)), t
    rng = np.random.default_rng(78)

    def bf16_pages(n, n_exp, skew):
        sm = rng.integers(0, 256, n).astype(np.uint16)
        pick = rng.integers(0, n_exp, n) if skew == 0 else np.minimum(rng.geometric(skew, n) - 1, 199)
        ex = (pick.astype(np.uint16) * 3 + 60) & 0xFF
        return torch.from_numpy((((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)).astype(np.uint16).view(np.uint8).copy())

    for S in (4, 8, 16, 32):
        cb = 16 * S * 6
        for n_exp, skew in ((12, 0), (40, 0), (200, 0.08)):
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                p, po = zc.params(zc.FMT_BF16, cb, streams=S, policy=policy, flags=R), o.params(o.BF16, cb, streams=S, policy=policy, payload_order=1)
                a = bf16_pages(300 * cb // 2, n_exp, skew)
                code = zc.train_code(dev(a), a.numel() // 2, p)
                ln, md = o.train_code(a.numpy(), a.numel() // 2, po)
                for pages in (513, 1500):
                    b = bf16_pages(pages * cb // 2, n_exp, skew)
                    print("one pass bf16 S", S, "exponents", n_exp, "policy", policy, "pages", pages, flush=True)
                    want = o.compress_with_code(b.numpy(), b.numel() // 2, po, ln, md)
                    comp, info = zc.compress_with_code(dev(b), b.numel() // 2, p, code)
                    assert np.array_equal(comp.cpu().numpy(), want) and info.total_bytes == len(want)
                    out, _ = zc.decompress(comp, info)
                    torch.cuda.synchronize()
                    assert torch.equal(out.cpu(), b)
    # BF16 pages with codes of their own, built on the device: one call whose tensors have exponent codes of different
    # refill periods (8, 4 and 2 symbols), a constant exponent field and a table-coded sign+mantissa field (both left to
    # the generic kernels), pages of 4 KiB (streams kept in LDS) and of 16 KiB (sized first)
    def bf16_sm(n, n_exp, skew, sm_values):
        sm = rng.integers(0, sm_values, n).astype(np.uint16)
        pick = rng.integers(0, n_exp, n) if skew == 0 else np.minimum(rng.geometric(skew, n) - 1, 199)
        ex = (pick.astype(np.uint16) * 3 + 60) & 0xFF
        return torch.from_numpy((((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)).astype(np.uint16).view(np.uint8).copy())

    for S, cb in ((8, 4096), (16, 4096), (32, 16384), (4, 1024)):
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            p, po = zc.params(zc.FMT_BF16, cb, streams=S, policy=policy, flags=R), o.params(o.BF16, cb, streams=S, policy=policy, payload_order=1)
            srcs = [bf16_sm(700 * cb // 2, 12, 0, 256), bf16_sm(600 * cb // 2, 40, 0, 256), bf16_sm(1030 * cb // 2, 200, 0.08, 256),
                    bf16_sm(520 * cb // 2, 1, 0, 256), bf16_sm(640 * cb // 2, 30, 0, 5), bf16_sm(3 * cb // 2, 40, 0, 256)]
            print("one pass bf16, own codes S", S, "page", cb, "policy", policy, flush=True)
            bt = zc.Batch([dev(x) for x in srcs], [x.numel() // 2 for x in srcs], p)
            sizes = bt.compress()
            for t, x in enumerate(srcs):
                want = o.compress(x.numpy(), x.numel() // 2, po)
                got = bt.container(t).cpu().numpy()
                assert sizes[t] == len(want) and np.array_equal(got, want), (t, int(np.argmax(got[:len(want)] != want[:len(got)])))
            bt.decompress()
            torch.cuda.synchronize()
            for t, x in enumerate(srcs):
                assert torch.equal(bt.out[t].cpu()[:x.numel()], x), t
            bt.compress_async()
            assert bt.refresh_info() == sizes


def test_byte_grouped_symbols():
    # Sec. 3.2 (Fig. 7) / 3.4: field values coded in byte-sized groups; same bar as the plain formats
    F8, F4 = zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP4_E2M1_MX_BYTES
    for S in (64, 8, 1):
        cb = 4096
        for n in (1, 2, 16 * S - 1, 16 * S + 1, cb - 1, cb, cb + 1, 3 * cb + 17 * 16 + 5, 40 * cb + 3):
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                check_case(F8, n, cb, S, policy, tag="fp8-bytes")
    for S in (64, 16, 2):
        for n in (32, 32 * S * 3, 8192 - 32, 8192, 8192 + 32, 5 * 8192 + 96):
            check_case(F4, n, 4096, S, tag="fp4-bytes")
    # full chunks through the 64-lane kernel: both fields table decoded, long codes, raw, delta, limits
    check_case(F8, 6 * 65536 + 1234, 65536, 64, tag="fp8-bytes-full")
    check_case(F8, 6 * 65536 + 1234, 65536, 64, zc.POLICY_AUTO, tag="fp8-bytes-full-auto")
    check_case(F8, 6 * 65536, 65536, 64, L=(11, 9, 0), tag="fp8-bytes-limits")
    k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=2048, seed=9)
    check_case(F8, k.numel(), 2048, 8, data=(k.reshape(-1), None), tag="fp8-bytes-kv-pages")
    a, b = wl.fp8_weight(5 * 32768 + 77, seed=1), wl.fp8_weight(5 * 32768 + 77, seed=2)
    check_case(F8, a.numel(), 32768, 64, data=(a, None), base=b, tag="fp8-bytes-delta")
    m, sc = wl.mxfp4_weight(256, 3584, seed=3)
    check_case(F4, 256 * 3584, 262144, 64, data=(m.reshape(-1), sc.reshape(-1)), tag="fp4-bytes-full")
    check_case(F4, 256 * 3584, 16384, 64, zc.POLICY_AUTO, data=(m.reshape(-1), sc.reshape(-1)), tag="fp4-bytes-auto")
    # batch with chunk id lists and a static dictionary
    srcs = [wl.fp8_weight(n, seed=60 + i) for i, n in enumerate((4 * 16384, 7 * 16384 + 5, 16384))]
    p, po = zc.params(F8, 16384), o.params(F8, 16384)
    bt = zc.Batch([dev(s) for s in srcs], [s.numel() for s in srcs], p)
    sizes = bt.compress()
    for i, s in enumerate(srcs):
        assert np.array_equal(bt.container(i).cpu().numpy(), o.compress(s.numpy(), s.numel(), po))
    outs = bt.decompress()
    torch.cuda.synchronize()
    for out, s in zip(outs, srcs):
        assert torch.equal(out.cpu()[:s.numel()], s)
    code = zc.train_code(dev(srcs[1]), srcs[1].numel(), p)
    ln, md = o.train_code(srcs[1].numpy(), srcs[1].numel(), po)
    comp, info = zc.compress_with_code(dev(srcs[0]), srcs[0].numel(), p, code)
    assert np.array_equal(comp.cpu().numpy(), o.compress_with_code(srcs[0].numpy(), srcs[0].numel(), po, ln, md))
    # stats agree with the oracle's
    st, so = zc.stats(dev(srcs[1]), srcs[1].numel(), p), o.stats(srcs[1].numpy(), srcs[1].numel(), po)
    for f in range(2):
        assert list(st.field[f].hist) == list(so.field[f].hist) and st.field[f].payload_bits == so.field[f].payload_bits
        assert abs(st.field[f].entropy_bits - so.field[f].entropy_bits) < 1e-12
    assert st.container_bytes == so.container_bytes


def test_nvfp4():
    # Sec. 3.4: NVFP4 = E2M1 elements + one E4M3 scale byte per 16 elements
    F = zc.FMT_FP4_E2M1_NV
    for S in (64, 16, 2):
        for n in (16, 16 * S * 3, 8192 - 16, 8192, 8192 + 16, 5 * 8192 + 48):
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                check_case(F, n, 4096, S, policy, tag="nvfp4")
    m, sc = wl.nvfp4_weight(256, 3584, seed=3)
    check_case(F, 256 * 3584, 262144, 64, data=(m, sc), tag="nvfp4-full")          # 64-lane full-chunk kernel
    check_case(F, 256 * 3584, 16384, 64, zc.POLICY_AUTO, data=(m, sc), tag="nvfp4-auto")
    # random access: chunks by id with their scale bytes
    p, po = zc.params(F, 16384), o.params(F, 16384)
    comp, info = zc.compress(dev(m), 256 * 3584, p, scales=dev(sc))
    ids = torch.tensor([27, 0, 13], dtype=torch.int32, device=DEV)
    out, sco = zc.decompress_chunks(comp, info, ids)
    torch.cuda.synchronize()
    for k, c in enumerate(ids.tolist()):
        assert torch.equal(out.cpu()[k * 16384:(k + 1) * 16384], m[c * 16384:(c + 1) * 16384])
        assert torch.equal(sco.cpu()[k * 2048:(k + 1) * 2048], sc[c * 2048:(c + 1) * 2048])
    # batch + stats
    mats = [wl.nvfp4_weight(64, 1024 + 512 * i, seed=20 + i) for i in range(3)]
    bt = zc.Batch([dev(a) for a, _ in mats], [a.numel() * 2 for a, _ in mats], p, scales=[dev(b) for _, b in mats])
    bt.compress()
    for i, (a, b) in enumerate(mats):
        assert np.array_equal(bt.container(i).cpu().numpy(), o.compress(a.numpy(), a.numel() * 2, po, scales=b.numpy()))
    outs = bt.decompress()
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(mats):
        assert torch.equal(outs[i].cpu()[:a.numel()], a) and torch.equal(bt.scales_out[i].cpu()[:b.numel()], b)
    st, so = zc.stats(dev(m), 256 * 3584, p, scales=dev(sc)), o.stats(m.numpy(), 256 * 3584, po, scales=sc.numpy())
    assert st.raw_bytes == so.raw_bytes and st.container_bytes == so.container_bytes
    assert list(st.field[2].hist) == list(so.field[2].hist)


def test_fp8_page_encoder():
    # FP8 with 4..32 lanes per chunk: the sub-wavefront size/encode kernels, byte for byte against the oracle
    for S in (4, 8, 16, 32):
        for cb in (16 * S, 2048, 3 * 16 * S):
            n = 37 * cb + 5
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                check_case(zc.FMT_FP8_E4M3, n, cb, S, policy, tag="fp8-pages")
    a, b = wl.fp8_weight(50 * 2048 + 100, seed=71), wl.fp8_weight(50 * 2048 + 100, seed=72)
    check_case(zc.FMT_FP8_E4M3, a.numel(), 2048, 16, data=(a, None), base=b, tag="fp8-pages-delta")
    # enough chunks for several passes per workgroup (2 x 2048 x 4 x 64/S chunks)
    x = wl.fp8_weight(140000 * 128 + 77, seed=73)
    check_case(zc.FMT_FP8_E4M3, x.numel(), 128, 8, data=(x, None), tag="fp8-pages-passes")
    # a batch of K/V tensors with a dictionary: no histogram, the same kernels
    k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=2048, seed=74)
    p, po = zc.params(zc.FMT_FP8_E4M3, 2048, streams=8), o.params(o.FP8_E4M3, 2048, streams=8)
    code = zc.train_code(dev(k.reshape(-1)), k.numel(), p)
    ln, md = o.train_code(k.reshape(-1).numpy(), k.numel(), po)
    bt = zc.Batch([dev(k.reshape(-1)), dev(v.reshape(-1))], [k.numel(), v.numel()], p)
    bt.compress(code=code)
    for i, t in enumerate((k, v)):
        assert np.array_equal(bt.container(i).cpu().numpy(), o.compress_with_code(t.reshape(-1).numpy(), t.numel(), po, ln, md))


def _random_source(rng, fmt, n):
    """Element bytes (and scale bytes) with a randomly chosen amount of structure."""
    nbytes = (n * zc.elem_bits(fmt) + 7) // 8
    kind = int(rng.integers(0, 5))
    if kind == 0:      # uniform bytes: nothing compresses
        b = rng.integers(0, 256, nbytes, dtype=np.uint8)
    elif kind == 1:    # few distinct bytes with skewed frequencies: short and long codes
        vals = rng.integers(0, 256, int(rng.integers(2, 9)), dtype=np.uint8)
        pr = rng.dirichlet(np.full(len(vals), 0.3))
        b = rng.choice(vals, nbytes, p=pr).astype(np.uint8)
    elif kind == 2:    # one value: constant fields
        b = np.full(nbytes, int(rng.integers(0, 256)), np.uint8)
    elif kind == 3:    # geometric byte values: deep code trees (the length limit binds)
        b = np.minimum(rng.geometric(0.5, nbytes) - 1, 255).astype(np.uint8) * np.uint8(rng.integers(1, 9))
    else:              # the workload generators
        blk = zc.scale_block(fmt) or 1
        t, _ = make_input(fmt, (max(n, 1) + blk - 1) // blk * blk, int(rng.integers(0, 1000)))
        b = t.numpy().reshape(-1).view(np.uint8)[:nbytes].copy()
        assert b.size == nbytes
    sc = None
    if zc.scale_block(fmt):
        ns = n // zc.scale_block(fmt)
        sc = (rng.integers(0, 256, ns, dtype=np.uint8) if rng.integers(0, 2) else np.full(ns, 120, np.uint8) + rng.integers(0, 3, ns, dtype=np.uint8))
    return torch.from_numpy(b), None if sc is None else torch.from_numpy(sc)


def test_random_parameter_sweep():
    # seeded sweep over formats, lanes, chunk sizes, lengths, policies, length limits and data shapes
    rng = np.random.default_rng(20250827)
    fmts = (zc.FMT_BF16, zc.FMT_FP8_E4M3, zc.FMT_FP4_E2M1_MX, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP4_E2M1_MX_BYTES, zc.FMT_FP4_E2M1_NV,
            zc.FMT_FP8_E5M2)
    for case in range(2100):
        fmt = fmts[case % len(fmts)]
        S = int(2 ** rng.integers(0, 7))
        unit = 256 if zc.scale_block(fmt) else 16
        cb = unit * int(rng.integers(1, 40)) if rng.integers(0, 3) else int(2 ** rng.integers(10, 16))
        cb = max(cb // unit * unit, unit)
        E = cb * 8 // zc.elem_bits(fmt)
        n = int(rng.integers(0, 6 * E + 2)) if rng.integers(0, 4) else int(rng.integers(1, 4)) * E
        blk = zc.scale_block(fmt)
        if blk:
            n = n // blk * blk
        policy = int(rng.integers(0, 2))
        sb8 = fmt in (zc.FMT_BF16, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP4_E2M1_MX_BYTES, zc.FMT_FP8_E5M2)
        lo = 8 if sb8 else (4 if fmt == zc.FMT_FP8_E4M3 else 2)
        L = (int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0, int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0,
             int(rng.integers(8, 17)) if rng.integers(0, 2) else 0)
        src, sc = _random_source(rng, fmt, n)
        base = None
        if rng.integers(0, 4) == 0 and n:
            base = torch.from_numpy(rng.integers(0, 256, src.numel(), dtype=np.uint8) & np.uint8(rng.choice([0x01, 0x81, 0xFF])))
        if src.numel() == 0:
            src = torch.zeros(0, dtype=torch.uint8)
        check_case(fmt, n, cb, S, policy, L, data=(src, sc), base=base, tag="sweep-%d" % case, order=int(case % 4 == 1))


def test_random_sweep_whole_row_chunks_and_pages():
    # the same kind of sweep over the geometries the specialised kernels take: 64 lanes with chunks of whole 1 KiB
    # rows (1 to 32 of them), or 4 to 32 lanes with chunks of whole 16-byte runs per lane, for the formats that have
    # kernels of their own or go through the 64-lane kernel with 8-bit symbols
    rng = np.random.default_rng(20261128)
    fmts = (zc.FMT_BF16, zc.FMT_FP8_E5M2, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP8_E4M3, zc.FMT_BF16, zc.FMT_FP8_E5M2)
    for case in range(1800):
        fmt = fmts[case % len(fmts)]
        S = 64 if rng.integers(0, 4) else int(2 ** rng.integers(2, 6))
        cb = 1024 * int(rng.integers(1, 33)) if S == 64 else 16 * S * int(rng.integers(1, 17))
        E = cb * 8 // zc.elem_bits(fmt)
        n = int(rng.integers(1, 6)) * E if rng.integers(0, 3) else int(rng.integers(0, 5 * E + 2))
        policy = int(rng.integers(0, 2))
        lo = 4 if fmt == zc.FMT_FP8_E4M3 else 8
        L = (int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0, int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0, 0)
        src, sc = _random_source(rng, fmt, n)
        base = None
        if rng.integers(0, 3) == 0 and n:
            base = torch.from_numpy(rng.integers(0, 256, src.numel(), dtype=np.uint8) & np.uint8(rng.choice([0x01, 0x81, 0xFF, 0x03])))
        if src.numel() == 0:
            src = torch.zeros(0, dtype=torch.uint8)
        check_case(fmt, n, cb, S, policy, L, data=(src, sc), base=base, tag="rows-%d" % case, order=int(case % 3 == 0))


def test_random_sweep_chunks_of_256_kib():
    # the same kind of sweep over 64 lanes with chunks of 256 KiB, where the histogram pass also counts symbols per chunk lane
    # and the stream sizes come from those counts: FP8 (16 exponent counts per lane) and the formats of 8-bit symbols
    rng = np.random.default_rng(20261130)
    fmts = (zc.FMT_BF16, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP8_E5M2, zc.FMT_FP8_E4M3)
    cb = 262144
    for case in range(96):
        fmt = fmts[case % len(fmts)]
        E = cb * 8 // zc.elem_bits(fmt)
        n = int(rng.integers(1, 4)) * E if rng.integers(0, 2) else int(rng.integers(0, 3 * E + 2))
        policy = int(rng.integers(0, 2))
        lo = 4 if fmt == zc.FMT_FP8_E4M3 else 8
        L = (int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0, int(rng.integers(lo, 17)) if rng.integers(0, 2) else 0, 0)
        src, sc = _random_source(rng, fmt, n)
        base = None
        if rng.integers(0, 3) == 0 and n:
            base = torch.from_numpy(rng.integers(0, 256, src.numel(), dtype=np.uint8) & np.uint8(rng.choice([0x01, 0x81, 0xFF, 0x03])))
        if src.numel() == 0:
            src = torch.zeros(0, dtype=torch.uint8)
        check_case(fmt, n, cb, 64, policy, L, data=(src, sc), base=base, tag="256k-%d" % case, order=int(case % 3 == 0))


def test_random_sweep_of_batches():
    # random sets of tensors (1 to 8, whole and ragged lengths, empty ones) through zc_compress_batch and
    # zc_decompress_batch: every container against the oracle's, every round trip bit for bit.  What a set shares
    # (geometry, policy) and what it mixes (lengths, data) decide which kernels and work lists the plan uses.
    rng = np.random.default_rng(20261129)
    fmts = (zc.FMT_BF16, zc.FMT_FP8_E4M3, zc.FMT_FP4_E2M1_MX, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP8_E5M2, zc.FMT_FP4_E2M1_NV)
    for case in range(360):
        fmt = fmts[case % len(fmts)]
        blk = zc.scale_block(fmt)
        shape = int(rng.integers(0, 3))
        if shape == 0:
            S, cb = 64, 1024 * int(rng.integers(1, 17))
        elif shape == 1:
            S = int(2 ** rng.integers(2, 6))
            cb = 16 * S * int(rng.integers(1, 9))
        else:
            S, cb = int(2 ** rng.integers(0, 7)), 16 * int(rng.integers(1, 200))
        if blk:
            cb = 16384 if shape == 0 else max(cb // 256 * 256, 256)
        E = cb * 8 // zc.elem_bits(fmt)
        policy = int(rng.integers(0, 2))
        use_base = rng.integers(0, 4) == 0 and not blk
        ns, srcs, scs, bases = [], [], [], []
        for _ in range(int(rng.integers(1, 9))):
            n = int(rng.integers(1, 5)) * E if rng.integers(0, 2) else int(rng.integers(0, 4 * E + 2))
            if blk:
                n = n // blk * blk
            src, sc = _random_source(rng, fmt, n)
            if src.numel() == 0:
                src = torch.zeros(0, dtype=torch.uint8)
            ns.append(n)
            srcs.append(src)
            scs.append(sc)
            bases.append(torch.from_numpy(rng.integers(0, 256, src.numel(), dtype=np.uint8) & np.uint8(0x81)) if use_base else None)
        order = 1 if case % 3 == 1 else 0
        print("batch", case, "fmt", fmt, "S", S, "chunk", cb, "n", ns, "policy", policy, "base", bool(use_base), "order", order, flush=True)
        p, po = zc.params(fmt, cb, (0, 0, 0), S, policy, flags=zc.FLAG_REVERSE_FIELDS if order else 0), o.params(fmt, cb, (0, 0, 0), S, policy, payload_order=order)
        b = zc.Batch([dev(x) for x in srcs], ns, p, xor_bases=[dev(x) for x in bases] if use_base else None,
                     scales=[dev(x) for x in scs] if blk else None)
        sizes = b.compress()
        for t in range(len(ns)):
            # an empty tensor has no base as far as either side can tell (its device pointer is null)
            want = o.compress(srcs[t].numpy(), ns[t], po, xor_base=bases[t].numpy() if use_base and ns[t] else None,
                              scales=scs[t].numpy() if blk else None)
            got = b.container(t).cpu().numpy()
            assert sizes[t] == len(want), (t, sizes[t], len(want))
            assert np.array_equal(got, want), (t, int(np.argmax(got != want)))
        b.decompress()
        torch.cuda.synchronize()
        for t in range(len(ns)):
            nb = (ns[t] * zc.elem_bits(fmt) + 7) // 8
            assert torch.equal(b.out[t].cpu()[:nb], srcs[t].view(torch.uint8).reshape(-1)[:nb]), t
            if blk and ns[t]:
                assert torch.equal(b.scales_out[t].cpu()[:ns[t] // blk], scs[t]), t


def test_random_sweep_of_the_other_entry_points():
    # statistics, dictionary training and use, the call that allocates nothing and chunk lists (repeated and
    # out-of-range ids included) on random geometries and data, each against the oracle
    rng = np.random.default_rng(20261130)
    fmts = (zc.FMT_BF16, zc.FMT_FP8_E4M3, zc.FMT_FP4_E2M1_MX, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP8_E5M2, zc.FMT_FP4_E2M1_NV,
            zc.FMT_FP4_E2M1_MX_BYTES)
    host = lambda x: None if x is None else x.numpy()
    for case in range(280):
        fmt = fmts[case % len(fmts)]
        blk = zc.scale_block(fmt)
        shape = int(rng.integers(0, 3))
        if shape == 0:
            S, cb = 64, 1024 * int(rng.integers(1, 9))
        elif shape == 1:
            S = int(2 ** rng.integers(2, 6))
            cb = 16 * S * int(rng.integers(1, 9))
        else:
            S, cb = int(2 ** rng.integers(0, 7)), 16 * int(rng.integers(1, 120))
        if blk:
            cb = 16384 if shape == 0 else max(cb // 256 * 256, 256)
        E = cb * 8 // zc.elem_bits(fmt)
        policy = int(rng.integers(0, 2))

        def tensor():
            n = int(rng.integers(1, 6)) * E if rng.integers(0, 2) else int(rng.integers(1, 5 * E + 2))
            if blk:
                n = max(n // blk * blk, blk)
            return (n,) + _random_source(rng, fmt, n)

        (n_a, a, sa), (n_b, b, sb) = tensor(), tensor()
        order = 1 if case % 2 else 0
        print("entry points", case, "fmt", fmt, "S", S, "chunk", cb, "n", n_a, n_b, "policy", policy, "order", order, flush=True)
        p, po = zc.params(fmt, cb, (0, 0, 0), S, policy, flags=zc.FLAG_REVERSE_FIELDS if order else 0), o.params(fmt, cb, (0, 0, 0), S, policy, payload_order=order)
        compare_stats(zc.stats(dev(a), n_a, p, scales=dev(sa)), o.stats(a.numpy(), n_a, po, scales=host(sa)))
        # a dictionary trained on one tensor codes the other
        code = zc.train_code(dev(a), n_a, p, scales=dev(sa))
        ln, md = o.train_code(a.numpy(), n_a, po, scales=host(sa))
        for f in range(code.n_fields):
            assert list(code.code_len[f]) == ln[f].tolist() and code.mode[f] == md[f], f
        comp, info = zc.compress_with_code(dev(b), n_b, p, code, scales=dev(sb))
        assert np.array_equal(comp.cpu().numpy(), o.compress_with_code(b.numpy(), n_b, po, ln, md, scales=host(sb)))
        # the call that allocates nothing writes the container a plain compress writes
        want = o.compress(b.numpy(), n_b, po, scales=host(sb))
        dst = torch.empty(max(zc.compress_bound(n_b, p), 16), dtype=torch.uint8, device=DEV)
        zc.compress_noalloc(dev(b), n_b, p, dst, scales=dev(sb))
        torch.cuda.synchronize()
        assert zc.read_info(dst, check_index=True).total_bytes == len(want) and np.array_equal(dst[:len(want)].cpu().numpy(), want)
        # a chunk list over the dictionary's container
        nc = info.n_chunks
        k = int(rng.integers(1, 2 * nc + 2))
        ids = rng.integers(0, nc + (2 if rng.integers(0, 3) == 0 else 0), k).astype(np.int32)
        out = torch.full((k * cb,), 0xA5, dtype=torch.uint8, device=DEV)
        spc = E // blk if blk else 0                 # scale bytes of a whole chunk
        sc_out = torch.full((max(k * spc, 1),), 0xA5, dtype=torch.uint8, device=DEV) if blk else None
        zc.decompress_chunks(comp, info, torch.from_numpy(ids).to(DEV), out=out, scales_out=sc_out)
        torch.cuda.synchronize()
        rows, flat = out.cpu().numpy().reshape(k, cb), b.numpy().reshape(-1).view(np.uint8)
        for i, c in enumerate(ids):
            if c >= nc:
                assert (rows[i] == 0xA5).all(), ("a slot of an id out of range was written", i, c)
                continue
            lo, hi = int(c) * cb, min(int(c) * cb + cb, flat.size)
            assert np.array_equal(rows[i][:hi - lo], flat[lo:hi]), (i, c)
            if blk:
                s_lo, s_hi = int(c) * spc, min(int(c) * spc + spc, n_b // blk)
                assert np.array_equal(sc_out.cpu().numpy()[i * spc:i * spc + (s_hi - s_lo)], sb.numpy()[s_lo:s_hi]), ("scales", i, c)


def test_random_sweep_of_chunk_lists_over_batches():
    # sets of tensors decoded through lists of chunk ids (repeated ids, ids out of range, the short last chunk) in one
    # batch call: 64 lanes with whole rows (the specialised kernels' builds for lists), with odd chunk sizes, and pages
    rng = np.random.default_rng(20261201)
    fmts = (zc.FMT_FP8_E4M3, zc.FMT_BF16, zc.FMT_FP8_E4M3, zc.FMT_FP8_E4M3_BYTES, zc.FMT_FP8_E5M2, zc.FMT_FP8_E4M3)
    for case in range(240):
        fmt = fmts[case % len(fmts)]
        shape = int(rng.integers(0, 3))
        if shape == 0:
            S, cb = 64, 1024 * int(rng.integers(1, 9))
        elif shape == 1:
            S = int(2 ** rng.integers(2, 6))
            cb = 16 * S * int(rng.integers(1, 9))
        else:
            S, cb = 64, 16 * int(rng.integers(1, 200))
        E = cb * 8 // zc.elem_bits(fmt)
        policy = int(rng.integers(0, 2))
        whole_only = rng.integers(0, 2)
        ns, srcs, ids = [], [], []
        for _ in range(int(rng.integers(1, 7))):
            n = int(rng.integers(1, 6)) * E if (whole_only or rng.integers(0, 2)) else int(rng.integers(1, 5 * E + 2))
            ns.append(n)
            srcs.append(_random_source(rng, fmt, n)[0])
            nc = (n + E - 1) // E
            ids.append(rng.integers(0, nc + (2 if rng.integers(0, 4) == 0 else 0), int(rng.integers(1, 2 * nc + 2))).astype(np.int32))
        print("chunk lists", case, "fmt", fmt, "S", S, "chunk", cb, "n", ns, "policy", policy, flush=True)
        b = zc.Batch([dev(x) for x in srcs], ns, zc.params(fmt, cb, (0, 0, 0), S, policy))
        b.compress()
        b.set_chunk_ids([torch.from_numpy(i).to(DEV) for i in ids])
        for out in b.out:
            out.fill_(0xA5)
        b.decompress()
        torch.cuda.synchronize()
        for t in range(len(ns)):
            flat = srcs[t].numpy().reshape(-1).view(np.uint8)
            nc = (ns[t] + E - 1) // E
            rows = b.out[t].cpu().numpy()[:len(ids[t]) * cb].reshape(len(ids[t]), cb)
            for i, c in enumerate(ids[t]):
                if c >= nc:
                    assert (rows[i] == 0xA5).all(), ("a slot of an id out of range was written", t, i, c)
                    continue
                lo, hi = int(c) * cb, min(int(c) * cb + cb, flat.size)
                assert np.array_equal(rows[i][:hi - lo], flat[lo:hi]), (t, i, c)


def test_concurrent_callers_on_their_own_streams():
    # four host threads, each with a stream, a workspace and a set of tensors of its own, call the batch and the
    # single-tensor entry points at the same time: the library's page-locked staging is the only thing they share
    import threading
    errors = []

    def caller(k, rounds):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                fmt, cb, S = [(zc.FMT_FP8_E4M3, 65536, 64), (zc.FMT_BF16, 16384, 64), (zc.FMT_FP8_E4M3, 2048, 8), (zc.FMT_FP8_E4M3_BYTES, 32768, 64)][k]
                srcs = []
                for i in range(6):
                    n = (3 + i) * cb + (1000 + 38 * i if i % 2 else 0)
                    t = wl.bf16_weight(n // 2, seed=100 * k + i).view(torch.uint8) if fmt == zc.FMT_BF16 else wl.fp8_weight(n, seed=100 * k + i)
                    srcs.append(t.to(DEV))
                counts = [x.numel() // 2 if fmt == zc.FMT_BF16 else x.numel() for x in srcs]
                p = zc.params(fmt, cb, (0, 0, 0), S, zc.POLICY_HUFF_ALL)
                b = zc.Batch(srcs, counts, p)
                want = [len(o.compress(x.cpu().numpy(), n, o.params(fmt, cb, (0, 0, 0), S, zc.POLICY_HUFF_ALL))) for x, n in zip(srcs, counts)]
                for r in range(rounds):
                    assert b.compress() == want, (k, r)
                    b.decompress()
                    stream.synchronize()
                    for out, x in zip(b.out, srcs):
                        assert torch.equal(out[:x.numel()], x.reshape(-1)), (k, r)
                    if r % 8 == 0:
                        comp, info = zc.compress(srcs[1], counts[1], p)
                        out, _ = zc.decompress(comp, info)
                        stream.synchronize()
                        assert comp.numel() == want[1] and torch.equal(out[:srcs[1].numel()], srcs[1].reshape(-1)), (k, r)
        except Exception as e:                       # noqa: BLE001 - reported by the main thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=caller, args=(k, 40)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_random_sweep_fp8_chunks_of_one_histogram_block():
    # the same kind of sweep over the one shape whose size pass works from per-lane counts: FP8, 64 lanes, 256 KiB
    rng = np.random.default_rng(20251127)
    cb = 262144
    for case in range(24):
        n = int(rng.integers(0, 5 * cb + 2)) if rng.integers(0, 3) else int(rng.integers(1, 5)) * cb
        policy = int(rng.integers(0, 2))
        L = (int(rng.integers(4, 17)) if rng.integers(0, 2) else 0, int(rng.integers(4, 17)) if rng.integers(0, 2) else 0, 0)
        src, _ = _random_source(rng, zc.FMT_FP8_E4M3, n)
        base = None
        if rng.integers(0, 3) == 0 and n:
            base = torch.from_numpy(rng.integers(0, 256, src.numel(), dtype=np.uint8) & np.uint8(rng.choice([0x01, 0x81, 0xFF])))
        if src.numel() == 0:
            src = torch.zeros(0, dtype=torch.uint8)
        check_case(zc.FMT_FP8_E4M3, n, cb, 64, policy, L, data=(src, None), base=base, tag="sweep-one-block-%d" % case)


def test_bf16_two_coded_fields_whole_chunks():
    # BF16 with both fields table decoded on 64-lane whole chunks (the shape of a checkpoint delta), at every
    # refill period the two fields can share: limits 16 (period 2, codes beyond the lookup index), 11
    # (period 2), 8 (period 4), and unequal limits (different periods: the fields are decoded one by one)
    rng = np.random.default_rng(77)
    cb, S = 4096, 64
    E = cb // 2
    n = 5 * E + 1234
    # few distinct exponents and sign+mantissa bytes with a long tail of rare ones: deep trees in both fields
    ex = np.minimum(rng.geometric(0.45, n) - 1, 60).astype(np.uint16) + 100
    sm = (np.minimum(rng.geometric(0.3, n) - 1, 90).astype(np.uint16) * 37) & 0xFF
    bits = ((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)
    src = torch.from_numpy(bits.astype(np.uint16).view(np.uint8).copy())
    base = torch.from_numpy((rng.integers(0, 65536, n, dtype=np.uint16) & np.uint16(0x0181)).view(np.uint8).copy())
    for L in ((16, 16, 0), (11, 11, 0), (8, 8, 0), (8, 16, 0), (16, 9, 0)):
        for b in (None, base):
            check_case(zc.FMT_BF16, n, cb, S, zc.POLICY_HUFF_ALL, L, data=(src, None), base=b, tag="two-coded-L%d-%d" % L[:2])


def test_fp8_encoder_uneven_lanes():
    # 64-lane FP8 chunks whose lanes produce bits at very different rates: half of the lanes see one exponent
    # only (1-bit codes: a word stays owed for 8 to 16 steps) while the others use the long codes and ask for a
    # word almost every step, so the encoder's staging ring holds many complete words behind an owed one and
    # several segments leave it at once.  Also with lanes swapped every few rows.
    rng = np.random.default_rng(4242)
    cb, S = 65536, 64
    n = 3 * cb + 5000
    j = np.arange(n)
    lane = (j // 16) % 64
    row = (j % cb) // 1024
    for variant in range(3):
        if variant == 0:
            cheap = lane < 32
        elif variant == 1:
            cheap = ((lane + row // 5) % 64) < 32
        else:
            cheap = lane != 63                       # one busy lane among idle ones
        ex = np.where(cheap, 7, rng.integers(0, 16, n))
        sm = rng.integers(0, 16, n)
        b = ((sm & 8) << 4) | (ex << 3) | (sm & 7)
        src = torch.from_numpy(b.astype(np.uint8))
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E4M3, n, cb, S, policy, data=(src, None), tag="uneven-%d" % variant)


def test_dictionary_compress_without_sync():
    # the queue-only call leaves the same containers as the synchronising one; sizes come from the headers
    k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=4096, seed=81)
    srcs = [k.reshape(-1), v.reshape(-1), wl.fp8_weight(5 * 2048 + 77, seed=82)]
    p, po = zc.params(zc.FMT_FP8_E4M3, 2048, streams=8), o.params(o.FP8_E4M3, 2048, streams=8)
    code = zc.train_code(dev(srcs[0]), srcs[0].numel(), p)
    ln, md = o.train_code(srcs[0].numpy(), srcs[0].numel(), po)
    bt = zc.Batch([dev(s) for s in srcs], [s.numel() for s in srcs], p)
    for rep in range(2):                                  # twice: the workspace is reused
        bt.compress_async(code)
        sizes = bt.refresh_info()
        for i, s in enumerate(srcs):
            want = o.compress_with_code(s.numpy(), s.numel(), po, ln, md)
            assert sizes[i] == len(want) and np.array_equal(bt.container(i).cpu().numpy(), want)
    outs = bt.decompress()
    torch.cuda.synchronize()
    for out, s in zip(outs, srcs):
        assert torch.equal(out.cpu()[:s.numel()], s)
    # a destination below the worst-case bound is refused before anything is queued
    small = zc.Tensor()
    small.d_src, small.n_elems = dev(srcs[2]).data_ptr(), srcs[2].numel()
    buf = torch.empty(zc.compress_bound(srcs[2].numel(), p) - 16, dtype=torch.uint8, device=DEV)
    small.d_comp, small.comp_capacity = buf.data_ptr(), buf.numel()
    ws = torch.empty(zc.workspace_bytes([srcs[2].numel()], p), dtype=torch.uint8, device=DEV)
    arr = (zc.Tensor * 1)(small)
    st = zc.lib().zc_compress_batch_with_code_async(arr, 1, p, code, zc._ptr(ws), ws.numel(), zc._stream())
    assert st == zc.ERR_BUFFER_TOO_SMALL


def test_compress_without_sync_and_host_built_codes():
    # zc_compress_batch_async queues histogram, code construction (on the device), size pass, scan and encoder
    # and returns; the containers equal the oracle's, their sizes are in the headers.  Mixed shapes: a tensor the
    # specialised FP8 kernels take, one whose exponent code is too short for them, a constant one, a ragged one.
    rng = np.random.default_rng(99)
    cb = 4096
    srcs = [wl.fp8_weight(9 * cb + 77, seed=91),
            torch.from_numpy(((rng.integers(0, 2, 6 * cb) + 7) << 3).astype(np.uint8)),      # two exponents: 1-bit codes
            torch.full((3 * cb,), 0x38, dtype=torch.uint8),
            wl.fp8_weight(123, seed=92)]
    for S in (64, 8):
        p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=S), o.params(o.FP8_E4M3, cb, streams=S)
        bt = zc.Batch([dev(s) for s in srcs], [s.numel() for s in srcs], p)
        for rep in range(2):                                  # twice: the workspace is reused
            bt.compress_async()
            sizes = bt.refresh_info()
            for i, s in enumerate(srcs):
                want = o.compress(s.numpy(), s.numel(), po)
                assert sizes[i] == len(want) and np.array_equal(bt.container(i).cpu().numpy(), want), (S, rep, i)
        outs = bt.decompress()
        torch.cuda.synchronize()
        for out, s in zip(outs, srcs):
            assert torch.equal(out.cpu()[:s.numel()], s)
    # the same containers with the code built on the host (ZC_FLAG_HOST_CODES), also through the older, shorter
    # layout of zc_params (no flags field: device-built codes)
    for fmt, ofmt, n in ((zc.FMT_FP8_E4M3, o.FP8_E4M3, 70000), (zc.FMT_BF16, o.BF16, 35000)):
        s = wl.fp8_weight(n, seed=5) if fmt == zc.FMT_FP8_E4M3 else wl.bf16_weight(n, seed=5).view(torch.uint8).reshape(-1)
        want = o.compress(s.numpy(), n, o.params(ofmt, 4096))
        comp, info = zc.compress(dev(s), n, zc.params(fmt, 4096, flags=zc.FLAG_HOST_CODES))
        assert np.array_equal(comp.cpu().numpy(), want)
        short = zc.params(fmt, 4096)
        short.struct_size = 32
        comp, info = zc.compress(dev(s), n, short)
        assert np.array_equal(comp.cpu().numpy(), want)
    bad = zc.params(zc.FMT_FP8_E4M3, 4096, flags=4)               # an unknown flag bit
    with pytest.raises(zc.ZcError):
        zc.compress(dev(srcs[0]), srcs[0].numel(), bad)


def test_bf16_encoder_every_refill_period():
    # BF16, whole chunks, exponent field table coded next to a flat (HUFF_ALL) or raw (AUTO) sign+mantissa field: the
    # specialised encoders (64 lanes per chunk, and the page kernel's BF16 builds with 8), at longest exponent codes
    # of 1..4 bits (refill period 8), 5..8 (4) and beyond (2), with and without a base.  The last case has a 1-bit
    # code next to long ones, which the page kernel leaves to the generic encoder.
    rng = np.random.default_rng(31)
    for S, cb in ((64, 8192), (8, 1024)):
        n = 7 * (cb // 2) + 333                                 # seven whole chunks and a short one for the generic kernel
        sm = rng.integers(0, 256, n).astype(np.uint16)          # every sign+mantissa byte occurs: flat code / raw
        base = torch.from_numpy((rng.integers(0, 2, n, dtype=np.uint16) << 15).view(np.uint8).copy())     # flips signs only
        for n_exp, skew, lmax in ((2, 0, 1), (5, 0, 3), (12, 0, 4), (40, 0, 6), (200, 0.08, None), (201, 0.08, None)):
            # equally likely exponents (short codes) or a geometric tail (long ones), the last with one exponent that
            # takes 60 % of the values (a 1-bit code) in front of that tail
            pick = rng.integers(0, n_exp, n) if skew == 0 else np.minimum(rng.geometric(skew, n) - 1, 199)
            if n_exp == 201:
                pick = np.where(rng.random(n) < 0.6, 200, pick)
            ex = (pick.astype(np.uint16) * 3 + 60) & 0xFF
            bits = ((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)
            src = torch.from_numpy(bits.astype(np.uint16).view(np.uint8).copy())
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                for b in (None, base):
                    want, _, _ = check_case(zc.FMT_BF16, n, cb, S, policy, data=(src, None), base=b, tag="bf16-periods-%d" % n_exp)
            info = o_info(want)
            assert info["mode"][0] == 1 and (info["lmax"][0] == lmax if lmax else info["lmax"][0] >= 9), (n_exp, info)   # the case is what it is meant to be
            if S != 64:
                continue
            # the same exponents beside a table-coded sign+mantissa field: longest code 5..8 (refill period 4), then beyond (2)
            for tail in (40, 200):
                draw = rng.integers(0, tail, n) if tail == 40 else np.minimum(rng.geometric(0.12, n) - 1, tail - 1)
                sm2 = (draw.astype(np.uint16) * 7 + 1) & 0xFF
                bits2 = ((sm2 >> 7) << 15) | (ex << 7) | (sm2 & 0x7F)
                src2 = torch.from_numpy(bits2.astype(np.uint16).view(np.uint8).copy())
                want2, _, _ = check_case(zc.FMT_BF16, n, cb, S, zc.POLICY_HUFF_ALL, data=(src2, None), tag="bf16-periods-%d-sm%d" % (n_exp, tail))
                info2 = o_info(want2)
                assert info2["mode"][1] == 1 and (5 <= info2["lmax"][1] <= 8 if tail == 40 else info2["lmax"][1] >= 9), (n_exp, tail, info2)


def test_device_code_construction_hard_histograms():
    # exponent histograms that stress the package-merge on the device: Fibonacci counts (the deepest tree, the
    # limit binds hard), powers of two, all counts equal (every tie rule at once), a single heavy symbol among
    # many singletons, at limits from the alphabet size up.  The container's length table must be the oracle's
    # for that histogram, and the tensor must come back bit for bit.
    def fib(k):
        a, b, out = 1, 1, []
        for _ in range(k):
            out.append(a); a, b = b, a + b
        return out
    hists = {"fibonacci": fib(27), "powers": [1 << i for i in range(20)], "equal": [3] * 256, "equal-odd": [5] * 37,
             "heavy": [1] * 200 + [100000], "two": [7, 9], "ties": [1, 1, 2, 2, 4, 4, 8, 8, 16, 16, 32, 32] * 4}
    for name, counts in hists.items():
        counts = np.asarray(counts, dtype=np.int64)
        syms = (np.arange(len(counts)) * 5 + 3) % 256 if len(counts) < 256 else np.arange(256)      # not the first symbols of the alphabet
        h = np.zeros(256, np.uint64)
        h[syms] = counts.astype(np.uint64)
        ex = torch.repeat_interleave(torch.from_numpy(syms.astype(np.int32)).to(DEV), torch.from_numpy(counts).to(DEV))
        ex = ex[torch.randperm(ex.numel(), device=DEV, generator=torch.Generator(device=DEV).manual_seed(3))]
        n = ex.numel()
        bits = ((ex << 7) | 0x15).to(torch.int16)                    # one sign+mantissa value: a constant field
        src = bits.view(torch.uint8).reshape(-1)
        for limit in (8, 9, 11, 13, 16):
            comp, info = zc.compress(src, n, zc.params(zc.FMT_BF16, 4096, (limit, 0, 0), 64))
            want = np.asarray(o.code_lengths(h, limit), dtype=np.uint8)
            got = np.frombuffer(bytes(info.code_len[0]), dtype=np.uint8)
            assert info.mode[0] == zc.MODE_HUFF and info.mode[1] == zc.MODE_CONST, (name, limit)
            assert np.array_equal(got, want), (name, limit)
            assert info.max_len[0] == int(want.max())
            out, _ = zc.decompress(comp, info)
            torch.cuda.synchronize()
            assert torch.equal(out[:src.numel()], src), (name, limit)


def test_device_code_construction_wide_weights():
    # 2^28 + some BF16 values: 16 x the symbol count no longer fits 32 bits, so the device package-merge runs on
    # 64-bit weights.  The oracle's code lengths for the tensor's field histograms (counted here with torch) must
    # be the tables in the container, and the round trip must be exact.
    n = (1 << 28) + 4096 * 3 + 5
    g = torch.Generator(device=DEV).manual_seed(7)
    # exponents geometric around 120 (deep tree, many ties among the rare ones), sign+mantissa skewed
    ex = (120 + torch.clamp((torch.empty(n, device=DEV).exponential_(0.7, generator=g)).to(torch.int32), max=50)).to(torch.int32)
    sm = torch.clamp((torch.empty(n, device=DEV).exponential_(0.05, generator=g)).to(torch.int32), max=255)
    bits = (((sm >> 7) << 15) | (ex << 7) | (sm & 0x7F)).to(torch.int16)
    del ex, sm
    src = bits.view(torch.uint8).reshape(-1)
    p = zc.params(zc.FMT_BF16, 262144, (16, 12, 0), 64)
    comp, info = zc.compress(src, n, p)
    v = bits.to(torch.int32) & 0xFFFF
    h_e = torch.bincount((v >> 7) & 0xFF, minlength=256).cpu().numpy().astype(np.uint64)
    h_m = torch.bincount(((v >> 8) & 0x80) | (v & 0x7F), minlength=256).cpu().numpy().astype(np.uint64)
    del v
    assert int(h_e.sum()) == n and 16 * n >= 1 << 32
    for f, (h, limit) in enumerate(((h_e, 16), (h_m, 12))):
        want = np.asarray(o.code_lengths(h, limit), dtype=np.uint8)
        got = np.frombuffer(bytes(info.code_len[f]), dtype=np.uint8)
        assert info.mode[f] == zc.MODE_HUFF and np.array_equal(got, want), f
    out, _ = zc.decompress(comp, info)
    torch.cuda.synchronize()
    assert torch.equal(out[:src.numel()], src)


def test_tensor_beyond_4_gib():
    # One FP8 tensor of 4.5 GiB + a ragged tail: every byte offset past 2^32 must be computed in 64 bits.
    # The round trip is checked whole on the GPU; sampled chunks (first, the ones on both sides of the
    # 4 GiB line, the last whole one and the short tail) are encoded by the oracle from the tensor's own
    # code lengths and compared with the streams the library wrote.
    cb = 262144
    n = 18432 * cb + 1000
    parts = [wl.fp8_weight(2304 * cb, device=DEV, seed=3000 + i) for i in range(8)]
    src = torch.cat(parts + [wl.fp8_weight(1000, device=DEV, seed=3010)])
    del parts
    assert src.numel() == n and n > (1 << 32)
    p = zc.params(zc.FMT_FP8_E4M3, cb, streams=64)
    comp, info = zc.compress(src, n, p)
    print("beyond-4GiB compressed", info.total_bytes, flush=True)
    out, _ = zc.decompress(comp, info)
    torch.cuda.synchronize()
    assert torch.equal(out[:n], src)
    del out
    nc = info.n_chunks
    assert nc == 18433
    head = comp[:info.payload_offset].cpu().numpy()
    lens = [head[info.table_offset[f]:info.table_offset[f] + 16] for f in range(2)]
    index = [np.frombuffer(head[info.index_offset[f]:info.index_offset[f] + 4 * (nc + 1)].tobytes(), "<u4").astype(np.int64) for f in range(2)]
    assert info.mode[0] == zc.MODE_HUFF and info.mode[1] == zc.MODE_HUFF
    for c in (0, 16383, 16384, 18431, 18432):
        lo, hi = c * cb, min((c + 1) * cb, n)
        chunk = src[lo:hi].cpu().numpy()
        e, sm = o.split(o.FP8_E4M3, chunk, hi - lo)
        for f, syms in ((0, e), (1, sm)):
            a, b = int(info.payload_offset + 16 * index[f][c]), int(info.payload_offset + 16 * index[f][c + 1])
            got = comp[a:b].cpu().numpy()
            want = o.encode_stream(syms, lens[f], 16, 64)
            assert np.array_equal(got, want), (c, f)


def test_fp8_e5m2():
    # Sec. 3.2, the other FP8 variant: 5-bit exponent and 3-bit sign+mantissa values held in 8-bit symbols
    F = zc.FMT_FP8_E5M2
    for S in (64, 8, 1):
        cb = 4096
        for n in (1, 16 * S - 1, 16 * S + 1, cb - 1, cb, cb + 1, 3 * cb + 17 * 16 + 5, 40 * cb + 3):
            for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
                check_case(F, n, cb, S, policy, tag="e5m2")
    check_case(F, 6 * 65536 + 1234, 65536, 64, tag="e5m2-full")                       # 64-lane full-chunk kernel
    check_case(F, 6 * 65536, 65536, 64, L=(9, 8, 0), tag="e5m2-limits")
    a, b = wl.fp8_e5m2_weight(5 * 32768 + 77, seed=1), wl.fp8_e5m2_weight(5 * 32768 + 77, seed=2)
    check_case(F, a.numel(), 32768, 64, data=(a, None), base=b, tag="e5m2-delta")
    rng = np.random.default_rng(3)
    u = torch.from_numpy(rng.integers(0, 256, 3 * 16384 + 100, dtype=np.uint8))
    check_case(F, u.numel(), 16384, 64, zc.POLICY_AUTO, data=(u, None), tag="e5m2-uniform")
    c = torch.full((2 * 16384 + 5,), 0x3C, dtype=torch.uint8)
    check_case(F, c.numel(), 16384, 64, data=(c, None), tag="e5m2-constant")


def test_fp8_e5m2_weight_shape_kernel():
    # E5M2 weights: exponent field table decoded, sign+mantissa field with the flat 3-bit code over 0..7, which the E5M2
    # kernel decodes without a table.  Every refill period of the exponent field (2 with and without codes beyond the
    # lookup index, 4, 8), chunks of an odd and an even number of rows, a delta, a ragged tail, the batch route.
    F = zc.FMT_FP8_E5M2
    rng = np.random.default_rng(53)

    def e5m2_like(n, n_exp, geometric):
        sm = rng.integers(0, 8, n).astype(np.uint8)                       # uniform: the code comes out flat
        ex = (np.minimum(rng.geometric(geometric, n) - 1, n_exp - 1) if geometric else rng.integers(0, n_exp, n)).astype(np.uint8)
        return torch.from_numpy(((sm >> 2) << 7 | (ex << 2) | (sm & 3)).astype(np.uint8))

    for cb in (3072, 16384):
        n = 9 * cb + 777
        for tag, x, L, period, long_codes in (("p2-long", e5m2_like(n, 32, 0.45), (16, 0, 0), 2, True), ("p2", e5m2_like(n, 32, 0.45), (11, 0, 0), 2, False),
                                              ("p4", e5m2_like(n, 32, 0.45), (8, 8, 0), 4, False), ("p8", e5m2_like(n, 6, 0), (0, 0, 0), 8, False)):
            want, _, _ = check_case(F, n, cb, 64, L=L, data=(x, None), tag="e5m2-kernel-" + tag)
            info = zc.validate_container(want)
            assert info.mode[1] == zc.MODE_HUFF and list(info.code_len[1][:9]) == [3] * 8 + [0], tag
            lmax = info.max_len[0]
            assert (lmax > 11) == long_codes and {2: 9 <= lmax, 4: 5 <= lmax <= 8, 8: lmax <= 4}[period], (tag, lmax)
        base = e5m2_like(n, 32, 0.3)
        want, _, _ = check_case(F, n, cb, 64, data=(e5m2_like(n, 32, 0.45), None), base=base, tag="e5m2-kernel-delta")
        assert list(zc.validate_container(want).code_len[1][:9]) == [3] * 8 + [0]
    # a set of tensors in one launch
    srcs = [wl.fp8_e5m2_weight(5 * 65536 + 65536 * i, seed=60 + i) for i in range(3)]
    p, po = zc.params(F, 65536), o.params(F, 65536)
    bt = zc.Batch([dev(s_) for s_ in srcs], [s_.numel() for s_ in srcs], p)
    sizes = bt.compress()
    for i, s_ in enumerate(srcs):
        assert np.array_equal(bt.container(i).cpu().numpy(), o.compress(s_.numpy(), s_.numel(), po))
    plan = bt.plan_decompress()
    assert plan.fast_kernel == 7
    outs = bt.run_decompress()
    torch.cuda.synchronize()
    for out, s_ in zip(outs, srcs):
        assert torch.equal(out.cpu()[:s_.numel()], s_)
    # damaged streams stay inside the buffers
    comp, info = zc.compress(dev(srcs[0]), srcs[0].numel(), p)
    guard = 4096
    buf = torch.full((guard + comp.numel() + guard,), 0x5A, dtype=torch.uint8, device=DEV)
    body = buf[guard:guard + comp.numel()]
    body.copy_(comp)
    pay = int(info.payload_offset)
    body[pay:] = torch.from_numpy(rng.integers(0, 256, comp.numel() - pay).astype(np.uint8)).to(DEV)
    out = torch.full((guard + srcs[0].numel() + guard,), 0xC3, dtype=torch.uint8, device=DEV)
    zc.decompress(body, info, out=out[guard:guard + srcs[0].numel()])
    torch.cuda.synchronize()
    assert bool((out[:guard] == 0xC3).all()) and bool((out[guard + srcs[0].numel():] == 0xC3).all())
    assert bool((buf[:guard] == 0x5A).all()) and bool((buf[guard + comp.numel():] == 0x5A).all())


def test_planned_decode_replays_from_a_captured_graph():
    # A serving loop that decodes the same containers every step can record the planned decode once:
    # zc_decompress_batch_run only launches kernels.  Every replay is checked against the source, with the
    # outputs poisoned and eager work of this process in between (whole tensors, then a page list).
    for fmt, cb, S, n_tensors, n in ((zc.FMT_FP8_E4M3, 262144, 64, 3, 5 * 262144 + 4099), (zc.FMT_FP8_E4M3, 2048, 8, 4, 96 * 2048),
                                     (zc.FMT_BF16, 262144, 64, 2, 3 * 131072 + 77)):
        srcs = [make_input(fmt, n, 300 + i)[0] for i in range(n_tensors)]
        raws = [s.view(torch.uint8).reshape(-1) for s in srcs]
        b = zc.Batch([dev(s) for s in srcs], [n] * n_tensors, zc.params(fmt, cb, streams=S))
        b.compress()
        ids = None
        for use_ids in (False, True):
            if use_ids:
                if fmt != zc.FMT_FP8_E4M3 or cb != 2048:
                    continue
                ids = [wl.page_sample(n // cb, 0.5, seed=7 + i) for i in range(n_tensors)]
                b.set_chunk_ids([i.to(DEV) for i in ids])
            b.plan_decompress()
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                b.run_decompress()                      # warm-up on the capture stream
                side.synchronize()
                with torch.cuda.graph(g, stream=side):
                    b.run_decompress()
            torch.cuda.synchronize()
            for replay in range(4):
                for o in b.out:
                    o.fill_(0xA5)
                junk = torch.arange(1 << 16, device=DEV).float().cumsum(0)      # unrelated eager work
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                for i in range(n_tensors):
                    got = b.out[i].cpu()
                    if use_ids:
                        assert torch.equal(got.reshape(-1, cb), raws[i].reshape(-1, cb)[ids[i].long()]), (fmt, cb, replay, i)
                    else:
                        assert torch.equal(got[:raws[i].numel()], raws[i]), (fmt, cb, replay, i)
                assert torch.isfinite(junk[-1])
        b.set_chunk_ids(None)


def test_encoders_refill_periods_of_exactly_one_word():
    # A lane whose first refill periods each take exactly the 32 bits the decoder holds owes no word when it asks
    # for the next one: the state the specialised encoders' position queue must tell from "one word owed".
    # Built on purpose: symbols with the longest code (read from the oracle's table) fill the first periods of a
    # few lanes, for two rows on end, for one row, and for one period only.
    rng = np.random.default_rng(77)

    def pack(fmt, ex, sm):
        if fmt == zc.FMT_FP8_E4M3:
            return torch.from_numpy((((sm & 8) << 4) | (ex << 3) | (sm & 7)).astype(np.uint8))
        return torch.from_numpy((((sm >> 7) << 15) | (ex.astype(np.uint16) << 7) | (sm & 0x7F)).astype(np.uint16).view(np.uint8).copy())

    def patch(ex, rare, S, per_lane, target):
        per_row = per_lane * S
        for lane, rows in ((5 % S, 2), (S - 1, 1)):
            for r in range(rows):
                at = r * per_row + lane * per_lane
                ex[at:at + per_lane] = rare[rng.integers(0, len(rare), per_lane)]
        at = (S // 2) * per_lane
        ex[at:at + 32 // target] = rare[0]

    # the tensor's own code: a length limit of 8 that binds, so everything rare has an 8-bit code and stays there
    for fmt, S, cb, per_lane, limit, draw in ((zc.FMT_FP8_E4M3, 64, 8192, 16, (0, 0, 0), lambda n: np.minimum(rng.geometric(0.5, n) - 1, 14)),
                                              (zc.FMT_FP8_E4M3, 8, 1024, 16, (0, 0, 0), lambda n: np.minimum(rng.geometric(0.5, n) - 1, 14)),
                                              (zc.FMT_BF16, 64, 8192, 8, (8, 0, 0), lambda n: np.minimum(rng.geometric(0.5, n) - 1, 39) * 3 + 50),
                                              (zc.FMT_BF16, 8, 1024, 8, (8, 0, 0), lambda n: np.minimum(rng.geometric(0.5, n) - 1, 39) * 3 + 50)):
        n = 6 * (cb * 8 // zc.elem_bits(fmt)) + 37
        A = 16 if fmt == zc.FMT_FP8_E4M3 else 256
        ex, sm = draw(n), rng.integers(0, 256, n)
        po = o.params(fmt, cb, limit, S, zc.POLICY_HUFF_ALL)
        ln = np.asarray(o.compress(pack(fmt, ex, sm).numpy(), n, po)[64:64 + A])
        rare = np.flatnonzero(ln == 8)
        assert ln.max() == 8 and len(rare) >= 2, ln
        patch(ex, rare, S, per_lane, 8)
        src = pack(fmt, ex, sm)
        ln = np.asarray(o.compress(src.numpy(), n, po)[64:64 + A])
        assert (ln[rare] == 8).all(), ln                         # the case is what it is meant to be
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(fmt, n, cb, S, policy, L=limit, data=(src, None), tag="word-periods-own-code")

    # BF16 with 16-bit codes (two make a word): a dictionary trained on few exponents gives every other one the
    # longest code, whatever the tensor it is then used on holds
    n_train = 1 << 18
    train = pack(zc.FMT_BF16, np.minimum(rng.geometric(0.3, n_train) - 1, 20) + 100, rng.integers(0, 256, n_train))
    for S, cb in ((64, 8192), (8, 1024)):
        n = 6 * (cb // 2) + 37
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            p, po = zc.params(zc.FMT_BF16, cb, streams=S, policy=policy), o.params(zc.FMT_BF16, cb, streams=S, policy=policy)
            code = zc.train_code(dev(train), n_train, p)
            ln, md = o.train_code(train.numpy(), n_train, po)
            assert list(code.code_len[0]) == ln[0].tolist() and ln[0].max() == 16
            rare = np.flatnonzero(ln[0] == 16)
            ex = np.minimum(rng.geometric(0.3, n) - 1, 20) + 100
            patch(ex, rare, S, 8, 16)
            src = pack(zc.FMT_BF16, ex, rng.integers(0, 256, n))
            want = o.compress_with_code(src.numpy(), n, po, ln, md)
            comp, info = zc.compress_with_code(dev(src), n, p, code)
            assert np.array_equal(comp.cpu().numpy(), want), (S, policy)
            out, _ = zc.decompress(comp, info)
            torch.cuda.synchronize()
            assert torch.equal(out.cpu()[:src.numel()], src)


def test_fp8_chunks_of_one_histogram_block():
    # FP8, 64 lanes, 256 KiB chunks: the histogram pass counts exponents per chunk lane and the size pass works
    # from those counts.  Whole chunks next to a short last one, less than one chunk, a delta, a code the FP8
    # kernels do not take (longest exponent code below 5 bits: the generic size pass must do those chunks), the
    # longest code of 8 bits in whole-word groups, lanes of very different rates, and a batch that mixes them.
    rng = np.random.default_rng(123)
    cb = 262144
    cases = []
    n = 3 * cb + 70001
    cases.append(("weights", wl.fp8_weight(n, seed=5), None))
    cases.append(("delta", wl.fp8_weight(n, seed=6), wl.fp8_weight(n, seed=7)))
    cases.append(("short-tensor", wl.fp8_weight(cb - 16, seed=8), None))
    cases.append(("exactly-two", wl.fp8_weight(2 * cb, seed=9), None))
    e = rng.choice(4, size=n, p=[0.6, 0.25, 0.1, 0.05]).astype(np.uint8) + 5
    cases.append(("short-codes", torch.from_numpy(((e << 3) | rng.integers(0, 8, n).astype(np.uint8) | (rng.integers(0, 2, n).astype(np.uint8) << 7)).astype(np.uint8)), None))
    ex = np.minimum(rng.geometric(0.5, n) - 1, 14)
    j = np.arange(n)
    ex = np.where(((j // 16) % 64 == 5) & (j < 2 * cb), 14, ex)          # lane 5 of the first two chunks: 8-bit codes only
    ex = np.where(((j // 16) % 64 >= 32) & (j >= 2 * cb), 0, ex)          # half of the lanes of the third: 1-bit codes only
    sm = rng.integers(0, 16, n)
    cases.append(("long-codes", torch.from_numpy((((sm & 8) << 4) | (ex << 3) | (sm & 7)).astype(np.uint8)), None))
    for tag, src, base in cases:
        for policy in (zc.POLICY_HUFF_ALL, zc.POLICY_AUTO):
            check_case(zc.FMT_FP8_E4M3, src.numel(), cb, 64, policy, data=(src, None), base=base, tag="one-block-" + tag)
    # one batch of all tensors without a base
    plain = [c for c in cases if c[2] is None]
    p, po = zc.params(zc.FMT_FP8_E4M3, cb, streams=64), o.params(o.FP8_E4M3, cb, streams=64)
    b = zc.Batch([dev(c[1]) for c in plain], [c[1].numel() for c in plain], p)
    for rep in range(2):                                   # twice: the workspace is reused
        sizes = b.compress()
        for i, c in enumerate(plain):
            want = o.compress(c[1].numpy(), c[1].numel(), po)
            assert sizes[i] == len(want) and np.array_equal(b.container(i).cpu().numpy(), want), (c[0], rep)
    # and queued without a wait: the sizes are read from the headers afterwards
    b.arena.fill_(0x77)
    b.compress_async()
    sizes = b.refresh_info()
    for i, c in enumerate(plain):
        want = o.compress(c[1].numpy(), c[1].numel(), po)
        assert sizes[i] == len(want) and np.array_equal(b.container(i).cpu().numpy(), want), (c[0], "async")
    outs = b.decompress()
    torch.cuda.synchronize()
    for i, c in enumerate(plain):
        assert torch.equal(outs[i].cpu()[:c[1].numel()], c[1]), c[0]


def test_large_chunks():
    # chunks of several MiB: thousands of rows per wavefront through the staging and refill rings, chunk indices
    # with few entries, a short last chunk that is itself larger than most tensors of the other tests
    for fmt, cb, S, policy in ((zc.FMT_FP8_E4M3, 4 << 20, 64, zc.POLICY_HUFF_ALL), (zc.FMT_FP8_E4M3, 1 << 20, 64, zc.POLICY_AUTO),
                               (zc.FMT_BF16, 2 << 20, 64, zc.POLICY_HUFF_ALL), (zc.FMT_FP4_E2M1_MX, 1 << 20, 64, zc.POLICY_HUFF_ALL),
                               (zc.FMT_FP8_E4M3, 1 << 20, 16, zc.POLICY_HUFF_ALL), (zc.FMT_BF16, 1 << 20, 8, zc.POLICY_AUTO)):
        E = cb * 8 // zc.elem_bits(fmt)
        n = 2 * E + E // 3 // 32 * 32
        check_case(fmt, n, cb, S, policy, tag="large-chunks")
