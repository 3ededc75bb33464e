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
throughput and the ratios ride along in the same JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
# HBM bytes per decode launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each
# scaled by what the same counter reads for a plain copy of known size); None = not measured
MEASURED_TRAFFIC_BYTES = {"fp8_e4m3_weight_set_8b_x32": 12965000000}


def _time_ms(torch, fn, reps=5):
    fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in ev)
    return t[len(t) // 2]


def other_workloads(torch, wl, zc, dev, extras):
    """Configs 1, 3, 4, 5 at full size: ratios, compress and decompress GB/s (median of 5).
    extras: also the formats and variants beyond the five configurations."""
    out = {}

    def run(name, fmt, srcs, counts, chunk, streams, bases=None, scales=None, limit=(0, 0, 0), ids=None, dictionary=False,
            policy=zc.POLICY_HUFF_ALL):
        p = zc.params(fmt, chunk, limit, streams, policy)
        b = zc.Batch(srcs, counts, p, xor_bases=bases, scales=scales)
        sizes = b.compress()
        b.plan_decompress()
        raw = sum(s.numel() * s.element_size() for s in srcs) + (sum(s.numel() for s in scales) if scales else 0)
        t_c = _time_ms(torch, b.compress)
        b.plan_decompress()
        t_d = _time_ms(torch, b.run_decompress)
        ok = all(torch.equal(o.view(torch.uint8)[:s.numel() * s.element_size()], s.view(torch.uint8).reshape(-1)) for o, s in zip(b.out, srcs))
        st = zc.stats(srcs[0], counts[0], p, xor_base=bases[0] if bases else None, scales=scales[0] if scales else None)
        r = {"uncompressed_bytes": raw, "compressed_bytes": sum(sizes), "ratio_total": sum(sizes) / raw,
             "ratio_fields_payload": [st.field[f].ratio_payload for f in range(st.n_fields)],
             "compress_ms": t_c, "compress_GBps": raw / t_c / 1e6, "decompress_ms": t_d, "decompress_GBps": raw / t_d / 1e6,
             "compress_frac_of_hbm_peak_uncompressed": raw / t_c / 1e6 / HBM_PEAK_GBPS,
             "decompress_frac_of_hbm_peak_uncompressed": raw / t_d / 1e6 / HBM_PEAK_GBPS,
             "decompress_traffic_frac_of_hbm_peak": (raw + sum(sizes) + (raw if bases else 0)) / t_d / 1e6 / HBM_PEAK_GBPS,
             "round_trip_bit_exact": bool(ok)}
        if ids is not None:
            # random-access decode of a page sample of every tensor into dense buffers
            b.set_chunk_ids(ids)
            b.plan_decompress()
            outs = b.out
            t_p = _time_ms(torch, b.run_decompress)
            nb = sum(o.numel() for o in outs)
            okp = all(torch.equal(outs[i].view(-1, chunk), srcs[i].view(torch.uint8).view(-1, chunk)[ids[i].long()]) for i in range(b.n))
            comp_read = sum(sizes) * (nb / raw)
            r.update({"page_decode_ms": t_p, "page_decode_GBps": nb / t_p / 1e6, "pages": nb // chunk, "page_decode_bit_exact": bool(okp),
                      "page_decode_traffic_frac_of_hbm_peak": (nb + comp_read) / t_p / 1e6 / HBM_PEAK_GBPS})
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
            t_s = _time_ms(torch, lambda: [hb.compress(code=code) for hb, code, _ in halves])
            oks = True
            for hb, code, sub in halves:
                hb.plan_decompress()
                hb.run_decompress()
                oks = oks and all(torch.equal(o.view(torch.uint8)[:s.numel()], s.view(torch.uint8).reshape(-1)) for o, s in zip(hb.out, sub))
            r.update({"static_dictionary_compress_ms": t_s, "static_dictionary_compress_GBps": raw / t_s / 1e6,
                      "static_dictionary_ratio_total": dsizes / raw, "static_dictionary_round_trip_bit_exact": bool(oks)})
            del halves
            b = None
        out[name] = r
        del b
        torch.cuda.empty_cache()

    if extras:
        # config 2 again with byte-grouped symbols (two exponents per symbol; the flat sign+mantissa field raw)
        set2 = [t for _, t in wl.fp8_weight_set(32, device=dev)]
        run("c2_fp8_byte_symbols", zc.FMT_FP8_E4M3_BYTES, set2, [t.numel() for t in set2], 262144, 64, policy=zc.POLICY_AUTO)
        run("c2_fp8_byte_symbols_limit_11", zc.FMT_FP8_E4M3_BYTES, set2, [t.numel() for t in set2], 262144, 64, limit=(11, 11, 0), policy=zc.POLICY_AUTO)
        run("c2_fp8_plain_symbols_auto", zc.FMT_FP8_E4M3, set2, [t.numel() for t in set2], 262144, 64, policy=zc.POLICY_AUTO)
        del set2
        set2 = [t for _, t in wl.fp8_weight_set(32, device=dev, e5m2=True)]
        run("c2_shapes_in_fp8_e5m2", zc.FMT_FP8_E5M2, set2, [t.numel() for t in set2], 262144, 64)
        del set2
    x = wl.bf16_weight(1 << 20, device=dev, seed=0)
    run("c1_bf16_1M", zc.FMT_BF16, [x], [1 << 20], 65536, 64, limit=(16, 16, 0))
    mats = [wl.mxfp4_weight(8192, 28672, device=dev, seed=300 + i) for i in range(3)]
    run("c3_mxfp4_70b_mlp", zc.FMT_FP4_E2M1_MX, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64, scales=[m[1] for m in mats])
    if extras:
        # the same matrices 12 times over (36 matrices, 4.5 GB): enough chunks to fill the GPU, which 3 matrices do not
        big = [m for _ in range(12) for m in mats]
        run("c3_mxfp4_36_matrices", zc.FMT_FP4_E2M1_MX, [m[0] for m in big], [8192 * 28672] * 36, 262144, 64, scales=[m[1] for m in big])
        del big
        run("c3_mxfp4_70b_mlp_byte_symbols", zc.FMT_FP4_E2M1_MX_BYTES, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64,
            scales=[m[1] for m in mats], policy=zc.POLICY_AUTO)
        mats = [wl.nvfp4_weight(8192, 28672, device=dev, seed=310 + i) for i in range(3)]
        run("nvfp4_70b_mlp", zc.FMT_FP4_E2M1_NV, [m[0] for m in mats], [8192 * 28672] * 3, 262144, 64, scales=[m[1] for m in mats])
    del mats
    pairs = [wl.bf16_checkpoint_pair(4096 * 16384, device=dev, seed=400 + i) for i in range(16)]
    w0, w1 = [q[0] for q in pairs], [q[1] for q in pairs]
    run("c4_bf16_checkpoint_w1", zc.FMT_BF16, w1, [4096 * 16384] * 16, 262144, 64, limit=(16, 16, 0))
    run("c4_bf16_checkpoint_xor_delta", zc.FMT_BF16, w1, [4096 * 16384] * 16, 262144, 64, bases=w0, limit=(16, 16, 0))
    del pairs, w0, w1
    kv = []
    for layer in range(32):
        k, v = wl.fp8_kv_pair(device=dev, seed=500 + layer)
        kv += [k.reshape(-1), v.reshape(-1)]
    n_pages = kv[0].numel() // 2048
    ids = [wl.page_sample(n_pages, 0.25, device=dev, seed=600 + i) for i in range(len(kv))]
    run("c5_fp8_kv_pages", zc.FMT_FP8_E4M3, kv, [t.numel() for t in kv], 2048, 8, ids=ids, dictionary=True)
    # one decoding step's worth of new pages: 64 tensors x 32 pages of 2 KiB, dictionary known: latency, not throughput
    step_pages = [t[:32 * 2048].contiguous() for t in kv]
    p5 = zc.params(zc.FMT_FP8_E4M3, 2048, (0, 0, 0), 8)
    code_k = zc.train_code(kv[0], kv[0].numel(), p5)
    sb = zc.Batch(step_pages, [32 * 2048] * len(step_pages), p5)
    sb.compress(code=code_k)
    t_sync = _time_ms(torch, lambda: sb.compress(code=code_k))
    t_async = _time_ms(torch, lambda: sb.compress_async(code_k))
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
    t_own_sync = _time_ms(torch, lambda: sb.compress())
    t_own_async = _time_ms(torch, lambda: sb.compress_async())
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
        run("bf16_kv_pages", zc.FMT_BF16, kv, [t.numel() for t in kv], 4096, 8, ids=ids, policy=zc.POLICY_AUTO)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers in the weight set (32 = the full configuration)")
    ap.add_argument("--chunk-kib", type=int, default=256)
    ap.add_argument("--max-len", type=int, default=0, help="code length limit of the exponent field (0 = library default)")
    ap.add_argument("--policy", choices=["huff_all", "auto"], default="huff_all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-only", action="store_true", help="timed steps run only the decode kernel (for profiling)")
    ap.add_argument("--no-verify", action="store_true", help="skip the round-trip check (kernel experiments only)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the FP8 weight set (the metric); by default configurations 1, 3, 4 and 5 are timed too "
                         "and reported under 'other_workloads' in the same JSON line")
    ap.add_argument("--other-workloads", action="store_true",
                    help="also the formats and variants beyond the five configurations (byte-grouped symbols, E5M2, NVFP4, "
                         "BF16 K/V pages, MXFP4 at a size that fills the GPU)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed steps run one plain elementwise kernel that reads 1 GiB and writes 1 GiB "
                         "(scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
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
    ms_comp = [e[0].elapsed_time(e[1]) for e in events]
    ms_plan = [e[1].elapsed_time(e[2]) for e in events]
    ms_kern = [e[2].elapsed_time(e[3]) for e in events]
    mean = lambda v: sum(v) / len(v)
    ms_decomp = mean(ms_plan) + mean(ms_kern)
    ms_step = wall * 1000.0 / args.steps

    if args.copy_calibration:
        cal = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        cal_out = torch.empty_like(cal)
        torch.add(cal, 1, out=cal_out)
        torch.cuda.synchronize()
        del cal, cal_out

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
        "decompress_ms": ms_decomp, "decode_kernel_ms": mean(ms_kern), "decode_kernel_ms_min": min(ms_kern),
        "compress_ms": mean(ms_comp), "compress_GBps": (raw_bytes / (mean(ms_comp) / 1000.0) / 1e9) if mean(ms_comp) > 0 else None,
        "decompress_frac_of_hbm_peak_uncompressed": raw_bytes / (ms_decomp / 1000.0) / 1e9 / HBM_PEAK_GBPS,
        "round_trip_bit_exact": bool(ok) and not args.no_verify,
        "roofline": {"bound": "hbm", "kernel": "k_decode_fp8", "achieved": algo_bytes / kern_s / 1e9, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": algo_bytes / kern_s / 1e9 / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_launch": algo_bytes, "traffic": MEASURED_TRAFFIC_BYTES.get(workload)},
    }

    host = None
    if not args.no_cpu_baseline:
        host = [srcs[i].cpu().numpy() for i in range(min(7, len(srcs)))]      # layer 0: q, k, v, o, gate, up, down
    if not args.headline_only:
        # the other four configurations (and, on request, the extra formats); a failure here must not cost the line above
        del batch, srcs
        torch.cuda.empty_cache()
        try:
            result["other_workloads"] = other_workloads(torch, wl, zc, dev, args.other_workloads)
        except Exception as e:                                  # noqa: BLE001 - reported, not raised
            result["other_workloads"] = {"error": "%s: %s" % (type(e).__name__, e)}

    if not args.no_cpu_baseline:
        # the oracle as it stands, single thread, on a bounded sample of the same workload
        import numpy as np
        from oracle import zc_oracle as o
        po = o.params(o.FP8_E4M3, args.chunk_kib * 1024, (args.max_len, 0, 0), 64, 1 if args.policy == "auto" else 0)
        t_c = t_d = 0.0
        nbytes = 0
        for x in host:
            t = time.perf_counter(); c = o.compress(x, len(x), po); t_c += time.perf_counter() - t
            t = time.perf_counter(); rc, out, _ = o.decompress(c, len(x)); t_d += time.perf_counter() - t
            assert rc == 0 and np.array_equal(out, x)
            nbytes += len(x)
        result["cpu_baseline"] = {"value": nbytes / t_d / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": "oracle decompress of layer 0's seven tensors (%d bytes, %.1f s); "
                                            "its compress ran at %.4f GB/s" % (nbytes, t_d, nbytes / t_c / 1e9),
                                  "host_cores_visible": os.cpu_count()}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
