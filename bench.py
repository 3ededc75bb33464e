#!/usr/bin/env python3
"""Benchmark of the field-split Huffman codec on one MI355X.

Workload (the configuration the headline metric is quoted on): the FP8 E4M3 weight set
shaped like 32 decoder layers of an 8B-class model (224 tensors, 6.98 GB), synthetic
N(0, 0.02) values with 0.1% outliers, per-tensor scaled to amax = 448, one Huffman code
per field per tensor, 256 KiB chunks, 64 lanes per chunk.

One step = one pass of the whole path over the set with inputs resident in HBM:
  compress   (field split + histogram, code construction, stream sizes, scan, encode)
  decompress (descriptor upload, then the chunked decode + re-interleave kernel)
`value` is the decompress throughput in GB/s of uncompressed bytes; the compress
throughput and the ratios ride along in the same JSON line, as do configurations 1, 3, 4
and 5 (`other_workloads`), the library's plain copy kernel timed in the same run
(`copy_kernel`: what a kernel that only moves bytes reaches here) and the CPU oracle timed
on the host (`cpu_baseline`).
"""
import argparse
import hashlib
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
# the headline kernel's source: the kernel's file and the device helpers it is built from
HEADLINE_KERNEL_SOURCES = [os.path.join(ROOT, "paper_2508_19263_amd", "csrc", f) for f in ("zc_decode_fast.hip", "zc_decode_device.h")]
HEADLINE_COUNTER_PROFILE = os.path.join(ROOT, "profiles", "k_decode_fp8__fp8_weight_set__counters.md")


def measured_traffic(workload):
    """HBM bytes per decode launch from the committed counter profile (FETCH_SIZE + WRITE_SIZE of a rocprofv3 --pmc
    run, each scaled by what the same counter reads for the plain copy kernel).  The profile carries the hash of the
    kernel's source files; when they have changed since, the figure is stale and None is reported."""
    try:
        text = open(HEADLINE_COUNTER_PROFILE).read()
        m = re.search(r"bench: workload=(\S+) kernel=(\S+) traffic_bytes=(\d+) source_sha256=([0-9a-f]+) commit=(\S+)", text)
        if not m or m.group(1) != workload:
            return None
        if hashlib.sha256(b"".join(open(f, "rb").read() for f in HEADLINE_KERNEL_SOURCES)).hexdigest()[:16] != m.group(4)[:16]:
            return None
        return int(m.group(3))
    except OSError:
        return None


def _times_ms(torch, fn, reps=5, warm=1):
    """Per-call durations (HIP events on the current stream, the one the library launches on), sorted."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in ev)


def _median(t):
    return t[len(t) // 2]


def _roofline(kernel, algo_bytes, ms, copy_gbps):
    gbps = algo_bytes / ms / 1e6
    return {"bound": "hbm", "kernel": kernel, "algorithmic_bytes_per_launch": int(algo_bytes), "achieved": gbps, "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "frac_of_copy_kernel": gbps / copy_gbps if copy_gbps else None}


def copy_kernel_gbps(torch, zc, dev):
    """The library's plain 16-bytes-per-lane copy over 4 GiB (read 4 GiB + write 4 GiB), median of 7: linear through
    memory, and one wavefront per 256 KiB chunk (the access pattern of the 64-lane decoders and encoders)."""
    n = 1 << 32
    src = torch.zeros(n, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    t = _times_ms(torch, lambda: zc.copy_reference(src, dst), reps=7, warm=3)
    tc = _times_ms(torch, lambda: zc.copy_reference(src, dst, 262144), reps=7, warm=3)
    del src, dst
    torch.cuda.empty_cache()
    return {"bytes_read": n, "bytes_written": n, "ms_median": _median(t), "ms_min": t[0], "GBps": 2 * n / _median(t) / 1e6,
            "frac_of_hbm_peak": 2 * n / _median(t) / 1e6 / HBM_PEAK_GBPS,
            "one_wavefront_per_256KiB_chunk": {"ms_median": _median(tc), "ms_min": tc[0], "GBps": 2 * n / _median(tc) / 1e6,
                                               "frac_of_hbm_peak": 2 * n / _median(tc) / 1e6 / HBM_PEAK_GBPS}}


def placement_spread(torch, batch, counts, dev, arenas=8):
    """The headline decode launch again, same containers, into output buffers at other places in HBM: `arenas` buffers
    allocated one after the other with 1, 4, 7, ... GiB of other allocations between them, all alive at once.  The
    kernel, its work list and the virtual layout inside a buffer are the same every time; what changes is which
    physical memory the 256 KiB output streams land in."""
    total = sum(counts)
    offs, at = [], 0
    for n in counts:
        offs.append(at)
        at += n
    keep, times, made, split = [], [], [], None
    first = batch.out
    try:
        for k in range(arenas):
            keep.append(torch.empty((1 + 3 * k) << 30, dtype=torch.uint8, device=dev))
            arena = torch.empty(total, dtype=torch.uint8, device=dev)
            made.append(arena)
            batch.set_outputs([arena[o:o + n] for o, n in zip(offs, counts)])
            batch.plan_decompress()
            times.append(_median(_times_ms(torch, batch.run_decompress)))
    except torch.OutOfMemoryError:
        pass
    if len(made) >= 2:
        # every other tensor into the first of these buffers, the rest into the last: the outputs of one launch then lie
        # in two distant parts of HBM (about 150 GiB apart in the allocation order)
        a, b = made[0], made[-1]
        batch.set_outputs([(a if i % 2 == 0 else b)[o:o + n] for i, (o, n) in enumerate(zip(offs, counts))])
        batch.plan_decompress()
        split = _median(_times_ms(torch, batch.run_decompress))
    batch.set_outputs(first)
    batch.plan_decompress()
    del keep, made
    torch.cuda.empty_cache()
    return {"decode_kernel_ms": times, "min": min(times) if times else None, "max": max(times) if times else None,
            "decode_kernel_ms_outputs_split_over_two_distant_buffers": split,
            "note": "same launch, same containers, output buffers elsewhere in HBM; the timed steps above use the first placement"}


def other_workloads(torch, wl, zc, dev, extras, copy_gbps):
    """Configs 1, 3, 4, 5 at full size: ratios, compress and decompress GB/s (median and min of 5), roofline blocks.
    extras: also the formats and variants beyond the five configurations."""
    out = {}

    def run(name, fmt, srcs, counts, chunk, streams, bases=None, scales=None, limit=(0, 0, 0), ids=None, dictionary=False,
            policy=zc.POLICY_HUFF_ALL, decode_kernel="", compress_kernels="", flags=0):
        p = zc.params(fmt, chunk, limit, streams, policy, flags=flags)
        b = zc.Batch(srcs, counts, p, xor_bases=bases, scales=scales)
        sizes = b.compress()
        b.plan_decompress()
        raw = sum(s.numel() * s.element_size() for s in srcs) + (sum(s.numel() for s in scales) if scales else 0)
        comp = sum(sizes)
        tc = _times_ms(torch, b.compress)
        b.plan_decompress()
        td = _times_ms(torch, b.run_decompress)
        ok = all(torch.equal(o.view(torch.uint8)[:s.numel() * s.element_size()], s.view(torch.uint8).reshape(-1)) for o, s in zip(b.out, srcs))
        st = zc.stats(srcs[0], counts[0], p, xor_base=bases[0] if bases else None, scales=scales[0] if scales else None)
        base_bytes = raw if bases else 0
        t_c, t_d = _median(tc), _median(td)
        r = {"uncompressed_bytes": raw, "compressed_bytes": comp, "ratio_total": comp / raw,
             "ratio_fields_payload": [st.field[f].ratio_payload for f in range(st.n_fields)],
             "compress_ms": t_c, "compress_ms_min": tc[0], "compress_GBps": raw / t_c / 1e6,
             "decompress_ms": t_d, "decompress_ms_min": td[0], "decompress_GBps": raw / t_d / 1e6,
             "compress_frac_of_hbm_peak_uncompressed": raw / t_c / 1e6 / HBM_PEAK_GBPS,
             "decompress_frac_of_hbm_peak_uncompressed": raw / t_d / 1e6 / HBM_PEAK_GBPS,
             # decode: containers (and the base of a delta) read, tensors written; compress: one code per tensor forces two
             # reads of the source (and base) plus the container written; what the passes read beyond that is overhead
             "roofline_decompress": _roofline(decode_kernel, raw + comp + base_bytes, t_d, copy_gbps),
             "roofline_compress": _roofline(compress_kernels, 2 * (raw + base_bytes) + comp, t_c, copy_gbps),
             "decompress_traffic_frac_of_hbm_peak": (raw + comp + base_bytes) / t_d / 1e6 / HBM_PEAK_GBPS,
             "round_trip_bit_exact": bool(ok)}
        if not ok:
            raise RuntimeError("round trip of %s is not bit exact" % name)
        if ids is not None:
            # random-access decode of a page sample of every tensor into dense buffers
            b.set_chunk_ids(ids)
            b.plan_decompress()
            outs = b.out
            tp = _times_ms(torch, b.run_decompress)
            nb = sum(o.numel() for o in outs)
            okp = all(torch.equal(outs[i].view(-1, chunk), srcs[i].view(torch.uint8).view(-1, chunk)[ids[i].long()]) for i in range(b.n))
            comp_read = comp * (nb / raw)
            # per page: its streams read, the page written, 4 bytes of id and 16 of index read
            page_algo = nb + comp_read + (nb // chunk) * 20
            r.update({"page_decode_ms": _median(tp), "page_decode_ms_min": tp[0], "page_decode_GBps": nb / _median(tp) / 1e6, "pages": nb // chunk,
                      "page_decode_bit_exact": bool(okp), "roofline_page_decode": _roofline(decode_kernel, page_algo, _median(tp), copy_gbps),
                      "page_decode_traffic_frac_of_hbm_peak": (nb + comp_read) / _median(tp) / 1e6 / HBM_PEAK_GBPS})
            if not okp:
                raise RuntimeError("page decode of %s is not bit exact" % name)
        if dictionary:
            # static dictionaries, one per tensor role (K, V: even and odd list positions), each trained on the
            # first tensor of its role and applied to all of that role: no histogram pass, no code construction
            del b
            torch.cuda.empty_cache()
            halves = []
            for role in (0, 1):
                sub = srcs[role::2]
                hb = zc.Batch(sub, counts[role::2], p)
                halves.append((hb, zc.train_code(sub[0], counts[role], p), sub))
            dsizes = sum(sum(hb.compress(code=code)) for hb, code, _ in halves)
            ts = _times_ms(torch, lambda: [hb.compress(code=code) for hb, code, _ in halves])
            oks = True
            for hb, code, sub in halves:
                hb.plan_decompress()
                hb.run_decompress()
                oks = oks and all(torch.equal(o.view(torch.uint8)[:s.numel() * s.element_size()], s.view(torch.uint8).reshape(-1)) for o, s in zip(hb.out, sub))
            r.update({"static_dictionary_compress_ms": _median(ts), "static_dictionary_compress_ms_min": ts[0],
                      "static_dictionary_compress_GBps": raw / _median(ts) / 1e6,
                      "static_dictionary_ratio_total": dsizes / raw, "static_dictionary_round_trip_bit_exact": bool(oks),
                      # a dictionary leaves one read of the source for the sizes and one for the encoder; with the fields in
                      # reverse order one kernel does both and the second read comes from the caches
                      "roofline_static_dictionary_compress": (_roofline("k_compress_pages_chained", raw + dsizes, _median(ts), copy_gbps) if flags & zc.FLAG_REVERSE_FIELDS
                                                              else _roofline("k_encode_fp8_sub (size pass) + k_scan + k_encode_fp8_sub", 2 * raw + dsizes, _median(ts), copy_gbps))})
            if not oks:
                raise RuntimeError("dictionary round trip of %s is not bit exact" % name)
            del halves
            b = None
        out[name] = r
        del b
        torch.cuda.empty_cache()

    S64 = "k_decode_s64"
    if extras:
        # config 2 again with byte-grouped symbols (two exponents per symbol; the flat sign+mantissa field raw)
        set2 = [t for _, t in wl.fp8_weight_set(32, device=dev)]
        n2 = [t.numel() for t in set2]
        run("c2_fp8_byte_symbols", zc.FMT_FP8_E4M3_BYTES, set2, n2, 262144, 64, policy=zc.POLICY_AUTO, decode_kernel=S64, compress_kernels="k_hist_rows8_lanes + k_codes + k_sizes_rows8_counts + k_scan + k_encode_bf16<BYTES>")
        run("c2_fp8_byte_symbols_limit_11", zc.FMT_FP8_E4M3_BYTES, set2, n2, 262144, 64, limit=(11, 11, 0), policy=zc.POLICY_AUTO, decode_kernel=S64, compress_kernels="k_hist_rows8_lanes + k_codes + k_sizes_rows8_counts + k_scan + k_encode_bf16<BYTES>")
        run("c2_fp8_plain_symbols_auto", zc.FMT_FP8_E4M3, set2, n2, 262144, 64, policy=zc.POLICY_AUTO, decode_kernel="k_decode_fp8", compress_kernels="k_hist_fp8_lanes + k_codes + k_sizes_fp8_counts + k_scan + k_encode_fp8")
        # the generic paths beside their specialised neighbours: a chunk size that is not whole rows of 1 KiB takes the
        # chunks that are not whole rows: the generic encoder, the 64-lane decoder's build for such chunks
        run("c2_fp8_chunks_of_48KiB_plus_16", zc.FMT_FP8_E4M3, set2, n2, 48 * 1024 + 16, 64, decode_kernel="k_decode_s64<TAIL>", compress_kernels="k_hist + k_codes + k_encode<false> + k_scan + k_encode<true>")
        run("c2_fp8_chunks_of_48KiB_specialised_kernels", zc.FMT_FP8_E4M3, set2, n2, 48 * 1024, 64, decode_kernel="k_decode_fp8", compress_kernels="k_hist + k_codes + k_sizes_fp8 + k_scan + k_encode_fp8")
        # random access to the chunks of weights (Sec. 3.1): a seeded quarter of every tensor's 256 KiB chunks, in random order
        chunk_ids = [wl.page_sample(t.numel() // 262144, 0.25, device=dev, seed=900 + i) for i, t in enumerate(set2)]
        run("c2_fp8_chunk_list", zc.FMT_FP8_E4M3, set2, n2, 262144, 64, ids=chunk_ids, decode_kernel="k_decode_fp8; the list: k_decode_s64<TAIL>",
            compress_kernels="k_hist_fp8_lanes + k_codes + k_sizes_fp8_counts + k_scan + k_encode_fp8")
        del chunk_ids
        ragged = [t[:t.numel() - 4096 - 7 * 16] for t in set2]
        run("c2_fp8_ragged_tails", zc.FMT_FP8_E4M3, ragged, [t.numel() for t in ragged], 262144, 64, decode_kernel="k_decode_fp8 + k_decode_s64<TAIL> (last chunks)", compress_kernels="k_hist_fp8_lanes + k_hist + k_codes + k_sizes_fp8_counts + k_sizes_tail (last chunks) + k_scan + k_encode_fp8 + k_encode (last chunks)")
        del set2, ragged
        set2 = [t for _, t in wl.fp8_weight_set(32, device=dev, e5m2=True)]
        run("c2_shapes_in_fp8_e5m2", zc.FMT_FP8_E5M2, set2, [t.numel() for t in set2], 262144, 64, decode_kernel=S64, compress_kernels="k_hist_fp8_lanes<E5M2> + k_codes + k_sizes_e5m2_counts + k_scan + k_encode_bf16<E5M2>")
        run("c2_shapes_in_fp8_e5m2_limit_8", zc.FMT_FP8_E5M2, set2, [t.numel() for t in set2], 262144, 64, limit=(8, 8, 0), decode_kernel=S64, compress_kernels="k_hist_fp8_lanes<E5M2> + k_codes + k_sizes_e5m2_counts + k_scan + k_encode_bf16<E5M2>")
        del set2
    x = wl.bf16_weight(1 << 20, device=dev, seed=0)
    run("c1_bf16_1M", zc.FMT_BF16, [x], [1 << 20], 65536, 64, limit=(16, 16, 0), decode_kernel="k_decode_bf16_s64", compress_kernels="k_hist + k_codes + k_encode (sizes) + k_scan + k_encode_bf16")
    mats = [wl.mxfp4_weight(8192, 28672, device=dev, seed=300 + i) for i in range(3)]
    run("c3_mxfp4_70b_mlp", zc.FMT_FP4_E2M1_MX, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64, scales=[m[1] for m in mats],
        decode_kernel="k_decode_s64 (chunk shared by four wavefronts)", compress_kernels="k_hist x2 + k_codes + k_encode (sizes) + k_scan + k_encode")
    if extras:
        # the same matrices 12 times over (36 matrices, 4.5 GB): enough chunks to fill the GPU, which 3 matrices do not
        big = [m for _ in range(12) for m in mats]
        run("c3_mxfp4_36_matrices", zc.FMT_FP4_E2M1_MX, [m[0] for m in big], [8192 * 28672] * 36, 262144, 64, scales=[m[1] for m in big], decode_kernel=S64, compress_kernels="k_hist x2 + k_codes + k_encode (sizes) + k_scan + k_encode")
        del big
        run("c3_mxfp4_70b_mlp_byte_symbols", zc.FMT_FP4_E2M1_MX_BYTES, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64,
            scales=[m[1] for m in mats], policy=zc.POLICY_AUTO, decode_kernel=S64, compress_kernels="k_hist x2 + k_codes + k_encode (sizes) + k_scan + k_encode")
        mats = [wl.nvfp4_weight(8192, 28672, device=dev, seed=310 + i) for i in range(3)]
        run("nvfp4_70b_mlp", zc.FMT_FP4_E2M1_NV, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64, scales=[m[1] for m in mats], decode_kernel=S64, compress_kernels="k_hist x2 + k_codes + k_encode (sizes) + k_scan + k_encode")
    del mats
    pairs = [wl.bf16_checkpoint_pair(4096 * 16384, device=dev, seed=400 + i) for i in range(16)]
    w0, w1 = [q[0] for q in pairs], [q[1] for q in pairs]
    bf16_c = "k_hist + k_codes + k_encode (sizes) + k_scan + k_encode_bf16"
    bf16_lanes_c = "k_hist_rows8_lanes + k_codes + k_sizes_rows8_counts + k_scan + k_encode_bf16"       # 256 KiB chunks: sizes from counts per lane
    run("c4_bf16_checkpoint_w1", zc.FMT_BF16, w1, [4096 * 16384] * 16, 262144, 64, limit=(16, 16, 0), decode_kernel="k_decode_bf16_s64", compress_kernels=bf16_lanes_c)
    run("c4_bf16_checkpoint_xor_delta", zc.FMT_BF16, w1, [4096 * 16384] * 16, 262144, 64, bases=w0, limit=(16, 16, 0), decode_kernel="k_decode_bf16_s64", compress_kernels=bf16_lanes_c)
    if extras:
        run("c4_bf16_checkpoint_xor_delta_limit_11", zc.FMT_BF16, w1, [4096 * 16384] * 16, 262144, 64, bases=w0, limit=(11, 11, 0), decode_kernel="k_decode_bf16_s64", compress_kernels=bf16_lanes_c)
        run("c4_bf16_checkpoint_xor_delta_64KiB_chunks", zc.FMT_BF16, w1, [4096 * 16384] * 16, 65536, 64, bases=w0, limit=(16, 16, 0), decode_kernel="k_decode_bf16_s64", compress_kernels=bf16_c)
    del pairs, w0, w1
    kv = []
    for layer in range(32):
        k, v = wl.fp8_kv_pair(device=dev, seed=500 + layer)
        kv += [k.reshape(-1), v.reshape(-1)]
    n_pages = kv[0].numel() // 2048
    ids = [wl.page_sample(n_pages, 0.25, device=dev, seed=600 + i) for i in range(len(kv))]
    page_c = "k_hist + k_codes + k_encode_fp8_sub (sizes) + k_scan + k_encode_fp8_sub"
    run("c5_fp8_kv_pages", zc.FMT_FP8_E4M3, kv, [t.numel() for t in kv], 2048, 8, ids=ids, dictionary=True, decode_kernel="k_decode_fp8_sub<8>", compress_kernels=page_c)
    # the same with the fields in reverse order in the payload (ZC_FLAG_REVERSE_FIELDS): the dictionary call is one pass
    run("c5_fp8_kv_pages_reverse_fields", zc.FMT_FP8_E4M3, kv, [t.numel() for t in kv], 2048, 8, ids=ids, dictionary=True, decode_kernel="k_decode_fp8_sub<8>",
        compress_kernels="k_hist + k_codes + k_compress_pages_chained (sizes, scan and encoder in one pass over the source)", flags=zc.FLAG_REVERSE_FIELDS)
    if extras:
        # lanes per page: the tuning of configuration 5 (S = 8 is what the other rows use), and 64 lanes per page, which
        # takes the generic kernels
        for S in (4, 16, 32, 64):
            run("c5_fp8_kv_pages_S%d" % S, zc.FMT_FP8_E4M3, kv, [t.numel() for t in kv], 2048, S, ids=ids,
                decode_kernel="k_decode_fp8_sub<%d>" % S if S < 64 else "k_decode (generic)", compress_kernels=page_c if S < 64 else "k_hist + k_codes + k_encode<false> + k_scan + k_encode<true>")
    # one decoding step's worth of new pages: 64 tensors x 32 pages of 2 KiB, dictionary known: latency, not throughput
    step_pages = [t[:32 * 2048].contiguous() for t in kv]
    p5 = zc.params(zc.FMT_FP8_E4M3, 2048, (0, 0, 0), 8)
    code_k = zc.train_code(kv[0], kv[0].numel(), p5)
    sb = zc.Batch(step_pages, [32 * 2048] * len(step_pages), p5)
    sb.compress(code=code_k)
    t_sync = _median(_times_ms(torch, lambda: sb.compress(code=code_k)))
    t_async = _median(_times_ms(torch, lambda: sb.compress_async(code_k)))
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    for _ in range(20):
        sb.compress_async(code_k)
    host_us = (time.perf_counter() - h0) / 20 * 1e6
    torch.cuda.synchronize()
    sb.refresh_info()
    sb.decompress()
    torch.cuda.synchronize()
    ok_step = all(torch.equal(o[:s.numel()], s) for o, s in zip(sb.out, step_pages))
    # the same pages with codes of their own, built on the device: histogram, codes, sizes, scan, encoder queued
    t_own_sync = _median(_times_ms(torch, lambda: sb.compress()))
    t_own_async = _median(_times_ms(torch, lambda: sb.compress_async()))
    torch.cuda.synchronize()
    sb.refresh_info()
    sb.decompress()
    torch.cuda.synchronize()
    ok_step = ok_step and all(torch.equal(o[:s.numel()], s) for o, s in zip(sb.out, step_pages))
    out["c5_one_step_of_new_pages"] = {"tensors": len(step_pages), "pages": 32 * len(step_pages), "bytes": 32 * 2048 * len(step_pages),
                                       "compress_with_dictionary_ms": t_sync, "queued_without_wait_gpu_ms": t_async,
                                       "queued_without_wait_host_us_per_call": host_us,
                                       "own_codes_compress_ms": t_own_sync, "own_codes_queued_without_wait_gpu_ms": t_own_async,
                                       "round_trip_bit_exact": bool(ok_step)}
    if not ok_step:
        raise RuntimeError("round trip of one step of new pages is not bit exact")
    del sb, step_pages
    del kv
    if extras:
        # the same cache shape in BF16: 16-token pages of 4 KiB, 16 layers
        kv = []
        for layer in range(16):
            k, v = wl.bf16_kv_pair(device=dev, seed=700 + layer)
            kv += [k.reshape(-1), v.reshape(-1)]
        n_pages = kv[0].numel() * 2 // 4096
        ids = [wl.page_sample(n_pages, 0.25, device=dev, seed=800 + i) for i in range(len(kv))]
        # AUTO: the sign+mantissa bytes do not compress and are stored as they are (Sec. 3.1)
        run("bf16_kv_pages", zc.FMT_BF16, kv, [t.numel() for t in kv], 4096, 8, ids=ids, policy=zc.POLICY_AUTO, decode_kernel="k_decode_bf16_sub<8>", compress_kernels="k_hist + k_codes + k_encode_fp8_sub<BF16> (sizes) + k_scan + k_encode_fp8_sub<BF16>")
        # with the fields in reverse order a dictionary call codes, places and writes these pages in one read of them
        run("bf16_kv_pages_reverse_fields", zc.FMT_BF16, kv, [t.numel() for t in kv], 4096, 8, ids=ids, policy=zc.POLICY_AUTO, dictionary=True, flags=zc.FLAG_REVERSE_FIELDS,
            decode_kernel="k_decode_bf16_sub<8>", compress_kernels="k_hist + k_codes + k_compress_pages_chained<BF16> (sizes, scan and encoder in one pass over the source)")
    return out


# ---- the CPU oracle beside it --------------------------------------------------------------------------------
# Samples of every configuration, generated on the host with the workload module's own generators (same recipes,
# reduced sizes), through the single-threaded oracle: decode best of `reps`, compress once.

def _oracle_samples(wl, sample_bytes):
    """name -> (format, element bytes as numpy, n_elems, chunk, lanes, limit, base or None, scales or None)."""
    import torch
    s = {}
    n = sample_bytes
    s["c2_fp8_weights"] = (2, wl.fp8_weight(n, seed=901).numpy(), n, 262144, 64, (0, 0, 0), None, None)
    x = wl.bf16_weight(1 << 20, seed=0).view(torch.uint8).numpy()
    s["c1_bf16_1M"] = (1, x, 1 << 20, 65536, 64, (16, 16, 0), None, None)
    rows = max(1, n * 2 // 28672)
    p, sc = wl.mxfp4_weight(rows, 28672, seed=902)
    s["c3_mxfp4"] = (3, p.numpy(), rows * 28672, 262144, 64, (0, 0, 0), None, sc.numpy())
    w0, w1 = wl.bf16_checkpoint_pair(n // 2, seed=903)
    s["c4_bf16_w1"] = (1, w1.view(torch.uint8).numpy(), n // 2, 262144, 64, (16, 16, 0), None, None)
    s["c4_bf16_delta"] = (1, w1.view(torch.uint8).numpy(), n // 2, 262144, 64, (16, 16, 0), w0.view(torch.uint8).numpy(), None)
    tokens = max(16, n // (4 * 8 * 128) // 16 * 16)
    k, _v = wl.fp8_kv_pair(batch=4, heads=8, tokens=tokens, seed=904)
    s["c5_fp8_kv_pages"] = (2, k.numpy().reshape(-1), k.numel(), 2048, 8, (0, 0, 0), None, None)
    return s


def _oracle_time(o, np, sample, reps, repeat_to_bytes=0):
    fmt, x, n, chunk, lanes, limit, base, scales = sample
    po = o.params(fmt, chunk, limit, lanes, 0)
    raw = x.nbytes + (scales.nbytes if scales is not None else 0)
    passes = max(1, -(-repeat_to_bytes // raw)) if repeat_to_bytes else 1          # a small tensor is gone through several times
    t = time.perf_counter()
    for _ in range(passes):
        c = o.compress(x, n, po, xor_base=base, scales=scales)
    t_c = (time.perf_counter() - t) / passes
    best = None
    for _ in range(reps):
        t = time.perf_counter()
        for _ in range(passes):
            rc, out, _sc = o.decompress(c, x.nbytes, xor_base=base, n_scales=0 if scales is None else len(scales))
        d = (time.perf_counter() - t) / passes
        best = d if best is None else min(best, d)
        assert rc == 0 and np.array_equal(out, x)
    return {"sample_bytes": raw, "passes": passes, "decompress_GBps": raw / best / 1e9, "compress_GBps": raw / t_c / 1e9,
            "decompress_s_best_of_%d" % reps: best, "compress_s": t_c}


def oracle_worker(index, nbytes):
    """One of the processes of the all-cores leg: its own FP8 tensor (seeded by its index) through the oracle's decoder.
    Never touches the GPU.  Prints the seconds its decode took."""
    import numpy as np
    from oracle import zc_oracle as o
    from paper_2508_19263_amd import workloads as wl
    x = wl.fp8_weight(nbytes, seed=950 + index).numpy()
    po = o.params(o.FP8_E4M3, 262144, (0, 0, 0), 64, 0)
    c = o.compress(x, nbytes, po)
    t = time.perf_counter()
    rc, out, _ = o.decompress(c, nbytes)
    d = time.perf_counter() - t
    assert rc == 0 and np.array_equal(out, x)
    print("%.6f" % d)


def cpu_baseline(args):
    import numpy as np
    from oracle import zc_oracle as o
    from paper_2508_19263_amd import workloads as wl
    full = args.cpu_baseline_full
    head_bytes = 64 << 20
    other_bytes = (256 << 20) if full else (16 << 20)
    reps = 3
    t0 = time.perf_counter()
    samples = _oracle_samples(wl, other_bytes)
    per = {}
    head = dict(samples)["c2_fp8_weights"] if full else (2, wl.fp8_weight(head_bytes, seed=901).numpy(), head_bytes, 262144, 64, (0, 0, 0), None, None)
    per["c2_fp8_weights"] = _oracle_time(o, np, head, reps)
    for name, smp in samples.items():
        if name == "c2_fp8_weights":
            continue
        per[name] = _oracle_time(o, np, smp, reps, repeat_to_bytes=(256 << 20) if (full and name == "c1_bf16_1M") else (8 << 20) if name == "c1_bf16_1M" else 0)
    # all host cores: as many independent single-threaded oracle processes as the box gives this job, each over a tensor
    # of its own; the slowest decides
    cores = min(os.cpu_count() or 1, 16)
    each = (64 << 20) if full else (16 << 20)
    env = dict(os.environ, OMP_NUM_THREADS="1", MKL_NUM_THREADS="1")      # the workers only generate their input with torch
    procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--oracle-worker", str(i), str(each)], stdout=subprocess.PIPE, text=True, env=env)
             for i in range(cores)]
    secs = []
    for pr in procs:
        outp, _ = pr.communicate(timeout=600)
        if pr.returncode != 0:
            raise RuntimeError("oracle worker failed")
        secs.append(float(outp.strip().splitlines()[-1]))
    head_r = per["c2_fp8_weights"]
    return {"value": head_r["decompress_GBps"], "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "oracle decompress of a %d MiB tensor of the headline workload's recipe (FP8 E4M3, 256 KiB chunks), best of %d; "
                      "its compress ran at %.4f GB/s" % (head_r["sample_bytes"] >> 20, reps, head_r["compress_GBps"]),
            "per_workload_1_core": per,
            "all_host_cores": {"processes": cores, "bytes_each": each, "decompress_GBps": cores * each / max(secs) / 1e9,
                               "slowest_process_s": max(secs), "fastest_process_s": min(secs)},
            "host_cores_visible": os.cpu_count(), "wall_s": time.perf_counter() - t0,
            "note": "samples: %d MiB of the headline workload, %d MiB of each other one%s; --cpu-baseline-full times 256 MiB of every workload"
                    % (per["c2_fp8_weights"]["sample_bytes"] >> 20, other_bytes >> 20, "" if full else " (bounded so that the default run stays short)")}


def main():
    if len(sys.argv) >= 4 and sys.argv[1] == "--oracle-worker":
        oracle_worker(int(sys.argv[2]), int(sys.argv[3]))
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers in the weight set (32 = the full configuration)")
    ap.add_argument("--chunk-kib", type=int, default=256)
    ap.add_argument("--max-len", type=int, default=0, help="code length limit of the exponent field (0 = library default)")
    ap.add_argument("--policy", choices=["huff_all", "auto"], default="huff_all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-full", action="store_true", help="time the oracle on 256 MiB of every workload (minutes of CPU time)")
    ap.add_argument("--decode-only", action="store_true", help="timed steps run only the decode kernel (for profiling)")
    ap.add_argument("--no-verify", action="store_true", help="skip the round-trip check (kernel experiments only)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the FP8 weight set (the metric); by default configurations 1, 3, 4 and 5 are timed too "
                         "and reported under 'other_workloads' in the same JSON line")
    ap.add_argument("--other-workloads", action="store_true",
                    help="also the formats and variants beyond the five configurations (byte-grouped symbols, E5M2, NVFP4, "
                         "BF16 K/V pages, MXFP4 at a size that fills the GPU, lane and limit sweeps, the generic kernels)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (every chunk and tensor is "
              "independent, so N GPUs would each take whole tensors); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_19263_amd import workloads as wl
    from paper_2508_19263_amd import zc

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    policy = zc.POLICY_AUTO if args.policy == "auto" else zc.POLICY_HUFF_ALL
    p = zc.params(zc.FMT_FP8_E4M3, args.chunk_kib * 1024, (args.max_len, 0, 0), 64, policy)

    copy = copy_kernel_gbps(torch, zc, dev)

    names, srcs = [], []
    for name, t in wl.fp8_weight_set(args.layers, device=dev):
        names.append(name)
        srcs.append(t)
    counts = [t.numel() for t in srcs]
    raw_bytes = sum(counts)
    batch = zc.Batch(srcs, counts, p)
    batch.prepare_outputs()

    def step(ev):
        if ev:
            ev[0].record()
        if not args.decode_only:
            batch.compress()
            torch.cuda.synchronize()      # decompress is timed from an idle stream: upload of its plan, then the kernel
        if ev:
            ev[1].record()
        if not args.decode_only:
            batch.plan_decompress()
        if ev:
            ev[2].record()
        batch.run_decompress()
        if ev:
            ev[3].record()

    sizes = batch.compress()
    batch.plan_decompress()
    comp_bytes = sum(sizes)
    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_comp = sorted(e[0].elapsed_time(e[1]) for e in events)
    ms_plan = [e[1].elapsed_time(e[2]) for e in events]
    ms_kern = sorted(e[2].elapsed_time(e[3]) for e in events)
    mean = lambda v: sum(v) / len(v)
    ms_decomp = mean(ms_plan) + mean(ms_kern)
    ms_step = wall * 1000.0 / args.steps

    # bit-exact round trip of the whole set
    ok = args.no_verify or all(torch.equal(o[:n], s) for o, s, n in zip(batch.out, srcs, counts))
    if not ok:
        print("ROUND TRIP MISMATCH", file=sys.stderr)
        sys.exit(1)

    # per-field ratios on layer 0 (payload bits / raw bits), container ratio on the whole set
    f0_bits = f1_bits = f_syms = 0
    for i in range(min(7, len(srcs))):
        st = zc.stats(srcs[i], counts[i], p)
        f0_bits += st.field[0].payload_bits
        f1_bits += st.field[1].payload_bits
        f_syms += st.field[0].n_symbols
    ratio_exp = f0_bits / (4.0 * f_syms)
    ratio_sm = f1_bits / (4.0 * f_syms)

    workload = "fp8_e4m3_weight_set_8b_x%d" % args.layers
    algo_bytes = comp_bytes + raw_bytes               # decode reads the containers, writes the tensors
    kern_s = mean(ms_kern) / 1000.0
    roof = _roofline("k_decode_fp8", algo_bytes, mean(ms_kern), copy["GBps"])
    roof["frac_of_chunked_copy_kernel"] = roof["achieved"] / copy["one_wavefront_per_256KiB_chunk"]["GBps"]
    roof["traffic"] = measured_traffic(workload)
    result = {
        "metric": "decompress GB/s (uncompressed bytes) + compression ratio, FP8 E4M3 weights",
        "value": raw_bytes / (ms_decomp / 1000.0) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": workload, "tensors": len(srcs), "uncompressed_bytes": raw_bytes,
                   "chunk_bytes": args.chunk_kib * 1024, "streams_per_chunk": 64, "policy": args.policy,
                   "max_code_len_exponent": args.max_len or 8, "decode_only": args.decode_only},
        "compression_ratio": {"total_container": comp_bytes / raw_bytes, "exponent_payload": ratio_exp,
                              "sign_mantissa_payload": ratio_sm, "compressed_bytes": comp_bytes},
        "decompress_ms": ms_decomp, "decode_kernel_ms": mean(ms_kern), "decode_kernel_ms_median": _median(ms_kern), "decode_kernel_ms_min": ms_kern[0],
        "compress_ms": mean(ms_comp), "compress_ms_median": _median(ms_comp), "compress_ms_min": ms_comp[0],
        "compress_GBps": (raw_bytes / (mean(ms_comp) / 1000.0) / 1e9) if mean(ms_comp) > 0 else None,
        "decompress_frac_of_hbm_peak_uncompressed": raw_bytes / (ms_decomp / 1000.0) / 1e9 / HBM_PEAK_GBPS,
        "target_40_percent_of_hbm_peak": {"in_algorithmic_traffic": roof["frac"] >= 0.40,
                                          "in_uncompressed_bytes": raw_bytes / (ms_decomp / 1000.0) / 1e9 / HBM_PEAK_GBPS >= 0.40,
                                          "note": "decoding moves 1 + ratio bytes per uncompressed byte, so 0.40 of the peak in uncompressed bytes "
                                                  "would take more traffic than the plain copy kernel reaches here"},
        "round_trip_bit_exact": bool(ok) and not args.no_verify,
        "roofline": roof,
        "roofline_compress": None if args.decode_only else _roofline("k_hist_fp8_lanes + k_codes + k_sizes_fp8_counts + k_scan + k_encode_fp8",
                                                                     2 * raw_bytes + comp_bytes, mean(ms_comp), copy["GBps"]),
        "copy_kernel": copy,
    }

    if not args.decode_only:
        result["output_placement"] = placement_spread(torch, batch, counts, dev)
        algo = comp_bytes + raw_bytes
        result["output_placement"]["best_frac_of_hbm_peak"] = algo / result["output_placement"]["min"] / 1e6 / HBM_PEAK_GBPS if result["output_placement"]["min"] else None
        sp = result["output_placement"]["decode_kernel_ms_outputs_split_over_two_distant_buffers"]
        result["output_placement"]["split_frac_of_hbm_peak"] = algo / sp / 1e6 / HBM_PEAK_GBPS if sp else None

    failed = None
    if not args.headline_only:
        # the other four configurations (and, on request, the extra formats)
        del batch, srcs
        torch.cuda.empty_cache()
        try:
            result["other_workloads"] = other_workloads(torch, wl, zc, dev, args.other_workloads, copy["GBps"])
        except Exception as e:                                  # noqa: BLE001 - reported in the line AND in the exit status
            failed = "%s: %s" % (type(e).__name__, e)
            result["other_workloads"] = {"error": failed}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args)
    print(json.dumps(result))
    if failed:
        print("other workloads failed: " + failed, file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
