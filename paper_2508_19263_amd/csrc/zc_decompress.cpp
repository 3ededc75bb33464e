// The decompress side of the C ABI (zc_read_info, zc_decompress, zc_decompress_chunks, zc_decompress_batch and its
// plan / run halves): which kernel takes which container, descriptors, work lists, launches.  See include/zc.h.
#include <hip/hip_runtime.h>

#include <cstring>
#include <vector>

#include "zc_host.h"

using namespace zc;

namespace {

// Can the specialised FP8 kernel decode this container's full chunks?
struct FastKind { bool ok; int exp_kind, sm_kind; };

FastKind fast_kind(const zc_info &info)
{
    FastKind k = {false, 0, 0};
    if (info.format != ZC_FMT_FP8_E4M3 || info.streams != 64 || info.chunk_bytes % 1024) return k;
    // the kernel is written for a refill period of 4 symbols, i.e. a longest code of 5..8 bits
    if (info.mode[0] != ZC_MODE_HUFF || refill_period(16, info.max_len[0]) != 4) return k;
    if (info.mode[1] == ZC_MODE_RAW) k.sm_kind = 1;
    else if (info.mode[1] == ZC_MODE_HUFF) {
        for (int v = 0; v < 16; v++) if (info.code_len[1][v] != 4) return k;   // flat: canonical code == symbol
        k.sm_kind = 0;
    } else return k;
    k.exp_kind = info.max_len[0] <= 6 ? 1 : 0;
    k.ok = true;
    return k;
}

// Can the 64-lane full-chunk kernel decode this container?  Returns the number of LDS rings
// it needs per wavefront (1 or 2), or 0 if the container has to go through the generic kernel.
uint32_t s64_rings(const zc_info &info)
{
    if (info.streams != 64 || info.chunk_bytes % (is_fp4(info.format) ? 16384u : 1024u)) return 0;
    uint32_t huff = 0;
    const TensorDev d = make_desc(info);
    for (uint32_t f = 0; f < info.n_fields; f++) {
        if (info.mode[f] == ZC_MODE_EMPTY) return 0;
        if (f < 2 && d.kind[f] == 0) huff++;
    }
    return huff < 1 ? 1 : huff;
}

// Can the BF16 kernel written for weights, checkpoints and their deltas decode this container's full chunks?  64 lanes,
// chunks of whole rows, exponent field table decoded, sign+mantissa field table decoded on the same refill period or
// stored plainly.  Returns the rings it needs per wavefront (1 or 2), 0 if not.
uint32_t bf16_s64_rings(const zc_info &info)
{
    if (info.format != ZC_FMT_BF16 || !s64_rings(info)) return 0;
    const TensorDev d = make_desc(info);
    if (d.kind[0] != 0 || (d.period[0] != 2 && d.period[0] != 4 && d.period[0] != 8)) return 0;
    if (d.kind[1] == 0) return d.period[1] == d.period[0] ? 2 : 0;
    return 1;
}

// Can the E5M2 kernel decode this container's full chunks?  64 lanes, chunks of whole rows, exponent field table
// decoded on a refill period of 2, 4 or 8, sign+mantissa field coded with the flat 3-bit code over the values 0..7.
bool e5m2_s64_ok(const zc_info &info)
{
    if (info.format != ZC_FMT_FP8_E5M2 || !s64_rings(info)) return false;
    const TensorDev d = make_desc(info);
    if (d.kind[0] != 0 || (d.period[0] != 2 && d.period[0] != 4 && d.period[0] != 8)) return false;
    if (info.mode[1] != ZC_MODE_HUFF) return false;
    for (int v = 0; v < 256; v++) if (info.code_len[1][v] != (v < 8 ? 3 : 0)) return false;
    return true;
}

// Can the 64-lane kernel's build for chunks that are not whole rows decode this container's chunks (a short last chunk,
// or every chunk when the chunk size is not a multiple of 1 KiB)?  64 lanes, a format of two fields, no empty field.
bool s64_tail_ok(const zc_info &info)
{
    if (info.streams != 64 || info.n_fields != 2 || is_fp4(info.format)) return false;
    return info.mode[0] != ZC_MODE_EMPTY && info.mode[1] != ZC_MODE_EMPTY;
}

// Are both element fields stored plainly (flat code, raw, constant)?  Then the rows of a chunk do not depend on
// each other and the 64-lane kernel may share a chunk among the four wavefronts of a workgroup.
bool s64_split_ok(const zc_info &info)
{
    if (!s64_rings(info)) return false;
    const TensorDev d = make_desc(info);
    return d.kind[0] != 0 && d.kind[1] != 0;
}

// Can the sub-wavefront FP8 kernel (S < 64, e.g. K/V pages) decode this container's full chunks
// into a destination of dst_bytes?
bool fp8_sub_ok(const zc_info &info, uint64_t dst_bytes)
{
    if (info.format != ZC_FMT_FP8_E4M3 || info.streams < 4 || info.streams > 32) return false;
    if (info.chunk_bytes % (16 * info.streams) || info.chunk_bytes > (1u << 24)) return false;
    if (info.mode[0] != ZC_MODE_HUFF || refill_period(16, info.max_len[0]) != 4) return false;
    const TensorDev d = make_desc(info);
    if (d.kind[1] != 1 && d.kind[1] != 2) return false;
    // one 32-bit offset space per buffer: payload, destination and (for a delta) the base tensor
    if (info.total_bytes - info.payload_offset > 0xF0000000ull || dst_bytes > 0xF0000000ull) return false;
    if (info.xor_delta && info.n_elems > 0xF0000000ull) return false;
    return true;
}

// The same question for the sub-wavefront BF16 kernel: exponent field table decoded, sign+mantissa flat or raw.
bool bf16_sub_ok(const zc_info &info, uint64_t dst_bytes)
{
    if (info.format != ZC_FMT_BF16 || info.streams < 4 || info.streams > 32) return false;
    if (info.chunk_bytes % (16 * info.streams) || info.chunk_bytes > (1u << 24)) return false;
    const TensorDev d = make_desc(info);
    if (info.mode[0] != ZC_MODE_HUFF || d.kind[0] != 0 || (d.kind[1] != 1 && d.kind[1] != 2)) return false;
    if (info.total_bytes - info.payload_offset > 0xF0000000ull || dst_bytes > 0xF0000000ull) return false;
    if (info.xor_delta && info.n_elems * 2 > 0xF0000000ull) return false;
    return true;
}

// either of the two
bool sub_ok(const zc_info &info, uint64_t dst_bytes) { return fp8_sub_ok(info, dst_bytes) || bf16_sub_ok(info, dst_bytes); }


// the chunk index of every field, read back field by field and checked on the host
zc_status check_index(const zc_info &info, const uint8_t *d_comp, hipStream_t hs)
{
    uint32_t prev = 0;
    std::vector<uint32_t> idx((size_t)info.n_chunks + 1);
    for (uint32_t k = 0; k < info.n_fields; k++) {
        const uint32_t f = field_at(k, info.n_fields, info.payload_order != 0);
        HIP_TRY(hipMemcpyAsync(idx.data(), d_comp + info.index_offset[f], idx.size() * 4, hipMemcpyDeviceToHost, hs));
        HIP_TRY(hipStreamSynchronize(hs));
        const zc_status st = check_index_field(idx.data(), info.n_chunks, &prev);
        if (st) return st;
    }
    if (info.payload_offset + 16ull * prev != info.total_bytes) return ZC_ERR_CORRUPT;
    return ZC_OK;
}

// What every decode entry point requires of the container description it is handed: a caller may pass a zc_info
// it filled or cached itself (zc_compress_batch*_async leave total_bytes at 0 on purpose), so nothing here is
// taken on trust.  A description whose size fields cannot belong to a container is refused: the kernels would
// otherwise return early, or decode empty streams, and the call would report success with nothing decoded.
zc_status check_decode_info(const zc_info &info, uint64_t comp_bytes)
{
    if (!elem_bits(info.format) || info.streams == 0 || info.streams > 64 || (info.streams & (info.streams - 1))) return ZC_ERR_INVALID_ARG;
    if (info.chunk_bytes == 0 || info.chunk_bytes % 16) return ZC_ERR_INVALID_ARG;
    if (info.n_fields != (uint32_t)num_fields(info.format)) return ZC_ERR_INVALID_ARG;
    if (info.payload_offset < kHeaderBytes || info.total_bytes < info.payload_offset || info.total_bytes > comp_bytes) return ZC_ERR_INVALID_ARG;
    const uint64_t per_chunk = (uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(info.format);
    if ((info.n_elems + per_chunk - 1) / per_chunk != info.n_chunks) return ZC_ERR_INVALID_ARG;
    return ZC_OK;
}

zc_status decode_common(const void *d_comp, uint64_t comp_bytes, const zc_info *info_in, const uint32_t *d_ids, uint32_t n_ids, bool by_ids,
                        void *d_dst, uint64_t dst_capacity, void *d_scales_out, const void *d_xor_base, void *stream)
{
    if (!d_comp || !aligned16(d_comp)) return ZC_ERR_INVALID_ARG;
    zc_info local;
    if (!info_in) {
        zc_status st = zc_read_info(d_comp, comp_bytes, 0, &local, stream);
        if (st) return st;
        info_in = &local;
    }
    const zc_info &info = *info_in;
    const zc_status known = check_decode_info(info, comp_bytes);
    if (known) return known;
    const uint64_t raw = (info.n_elems * (uint64_t)elem_bits(info.format) + 7) / 8;
    const uint64_t need = by_ids ? (uint64_t)n_ids * info.chunk_bytes : raw;
    const uint32_t slots = by_ids ? n_ids : info.n_chunks;
    if (slots == 0) return ZC_OK;
    if (by_ids && !d_ids) return ZC_ERR_INVALID_ARG;
    if (!d_dst || !aligned16(d_dst)) return ZC_ERR_INVALID_ARG;
    if (dst_capacity < need) return ZC_ERR_BUFFER_TOO_SMALL;
    if (info.n_fields == 3 && (!d_scales_out || !aligned16(d_scales_out))) return ZC_ERR_INVALID_ARG;
    if (info.xor_delta && (!d_xor_base || !aligned16(d_xor_base))) return ZC_ERR_INVALID_ARG;
    TensorDev d = make_desc(info);
    d.comp = (uint8_t *)d_comp; d.dst = (uint8_t *)d_dst; d.scales_out = (uint8_t *)d_scales_out;
    d.base = info.xor_delta ? (const uint8_t *)d_xor_base : nullptr;
    d.ids = by_ids ? d_ids : nullptr; d.n_ids = by_ids ? n_ids : 0; d.dst_bytes = need;
    const uint32_t cpi = chunks_per_work_item(info.streams);
    const FastKind fk = fast_kind(info);
    uint32_t first_slot = 0;
    const uint32_t rings = s64_rings(info);
    const uint64_t elems_per_chunk = (uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(info.format);
    if (sub_ok(info, need) && (!by_ids || info.n_elems % elems_per_chunk == 0)) {
        // small chunks (pages): several per wavefront.  An id list may name a short last chunk, which
        // this kernel does not take, so lists go here only when every chunk is whole.
        const uint32_t n_fast = by_ids ? n_ids : (uint32_t)(info.n_elems / elems_per_chunk);
        const uint32_t spg = sub_slots_per_group(info.streams, n_fast);
        if (info.format == ZC_FMT_BF16) LAUNCH_TRY(launch_decode_bf16_sub(info.streams, info.xor_delta != 0, nullptr, nullptr, (n_fast + spg - 1) / spg, &d, spg, stream));
        else LAUNCH_TRY(launch_decode_fp8_sub(info.streams, info.xor_delta != 0, by_ids, nullptr, nullptr, (n_fast + spg - 1) / spg, &d, spg, stream));
        first_slot = n_fast;
    } else if ((fk.ok || rings) && !by_ids) {
        // full chunks through a specialised kernel, a short last chunk through the generic one
        const uint32_t n_full = (uint32_t)(info.n_elems / ((uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(info.format)));
        const uint32_t n_fast = (n_full + kWavesPerGroup - 1) / kWavesPerGroup;
        if (fk.ok) LAUNCH_TRY(launch_decode_fp8_fast(fk.exp_kind, fk.sm_kind, info.xor_delta != 0, false, nullptr, nullptr, n_fast, &d, stream));
        else if (e5m2_s64_ok(info)) LAUNCH_TRY(launch_decode_e5m2(info.xor_delta != 0, nullptr, nullptr, n_fast, &d, stream));
        else if (bf16_s64_rings(info)) LAUNCH_TRY(launch_decode_bf16_s64(bf16_s64_rings(info), info.xor_delta != 0, nullptr, nullptr, n_fast, &d, stream));
        else {
            const bool split = s64_split_ok(info);
            LAUNCH_TRY(launch_decode_s64(info.format, rings, info.xor_delta != 0, split, nullptr, nullptr, split ? n_full : n_fast, &d, stream));
        }
        first_slot = n_full;
    } else if (fk.ok && by_ids) {
        // a list over a container the FP8 kernel takes: the whole chunks it names through that kernel's build for lists;
        // the short last chunk, if there is one (the list may name it), through the 64-lane kernel's build for such chunks
        LAUNCH_TRY(launch_decode_fp8_fast(fk.exp_kind, fk.sm_kind, info.xor_delta != 0, true, nullptr, nullptr, (n_ids + kWavesPerGroup - 1) / kWavesPerGroup, &d, stream));
        if (info.n_elems % elems_per_chunk)
            LAUNCH_TRY(launch_decode_s64_tail(info.format, info.xor_delta != 0, nullptr, nullptr, (n_ids + cpi - 1) / cpi, &d, 0, true, stream));
        first_slot = slots;
    }
    if (first_slot < slots) {
        // what is left: chunks that are not whole rows and id lists with 64 lanes (the 64-lane kernel's build for those, for
        // the formats of two fields), geometries no specialised kernel takes
        const uint32_t n_work = (slots - first_slot + cpi - 1) / cpi;
        if (s64_tail_ok(info)) LAUNCH_TRY(launch_decode_s64_tail(info.format, info.xor_delta != 0, nullptr, nullptr, n_work, &d, first_slot, false, stream));
        else LAUNCH_TRY(launch_decode(info.format, nullptr, nullptr, n_work, cpi, &d, first_slot, stream));
    }
    return ZC_OK;
}

}  // namespace

// ----------------------------------------------------------------------- C ABI

extern "C" {

zc_status zc_copy_reference(const void *d_src, void *d_dst, uint64_t bytes, uint32_t chunk_bytes, void *stream)
{
    if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || bytes % 16) return ZC_ERR_INVALID_ARG;
    if (chunk_bytes && (chunk_bytes % 1024 || bytes % chunk_bytes || bytes / chunk_bytes > 0x7FFFFFFFull)) return ZC_ERR_INVALID_ARG;
    if (chunk_bytes) LAUNCH_TRY(launch_copy_chunked(d_src, d_dst, bytes, chunk_bytes, stream));
    else LAUNCH_TRY(launch_copy(d_src, d_dst, bytes, stream));
    return ZC_OK;
}

zc_status zc_read_info(const void *d_comp, uint64_t comp_bytes, int check_index_too, zc_info *out, void *stream)
{
    if (!d_comp || !out) return ZC_ERR_INVALID_ARG;
    if (comp_bytes < kHeaderBytes) return ZC_ERR_CORRUPT;
    uint8_t head[kBlobBytes];
    const uint64_t have = comp_bytes < kBlobBytes ? comp_bytes : kBlobBytes;
    hipStream_t hs = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(head, d_comp, have, hipMemcpyDeviceToHost, hs));
    HIP_TRY(hipStreamSynchronize(hs));
    zc_status st = parse_info(head, have, comp_bytes, out);
    if (st) return st;
    if (check_index_too) return check_index(*out, (const uint8_t *)d_comp, hs);
    return ZC_OK;
}

zc_status zc_decompress(const void *d_comp, uint64_t comp_bytes, const zc_info *info, void *d_dst, uint64_t dst_capacity,
                        void *d_scales_out, const void *d_xor_base, void *stream)
{
    return decode_common(d_comp, comp_bytes, info, nullptr, 0, false, d_dst, dst_capacity, d_scales_out, d_xor_base, stream);
}

zc_status zc_decompress_chunks(const void *d_comp, uint64_t comp_bytes, const zc_info *info, const uint32_t *d_chunk_ids, uint32_t n_ids,
                               void *d_dst, uint64_t dst_capacity, void *d_scales_out, const void *d_xor_base, void *stream)
{
    return decode_common(d_comp, comp_bytes, info, d_chunk_ids, n_ids, true, d_dst, dst_capacity, d_scales_out, d_xor_base, stream);
}

zc_status zc_decompress_batch_plan(const zc_tensor *tensors, uint32_t n_tensors, void *d_ws, uint64_t ws_bytes,
                                   zc_batch_plan *plan, void *stream)
{
    if (!plan) return ZC_ERR_INVALID_ARG;
    std::memset(plan, 0, sizeof(*plan));
    if (n_tensors == 0) return ZC_OK;
    if (!tensors || !d_ws || !aligned16(d_ws)) return ZC_ERR_INVALID_ARG;
    const uint32_t fmt = tensors[0].info.format, S = tensors[0].info.streams;
    if (!elem_bits(fmt) || S == 0 || S > 64 || (S & (S - 1))) return ZC_ERR_INVALID_ARG;
    for (uint32_t t = 0; t < n_tensors; t++) {
        const zc_tensor &x = tensors[t];
        if (x.info.format != fmt || x.info.streams != S) return ZC_ERR_INVALID_ARG;
        const zc_status known = check_decode_info(x.info, x.out_bytes > x.comp_capacity ? x.out_bytes : x.comp_capacity);
        if (known) return known;
    }
    const uint32_t cpi = chunks_per_work_item(S);
    // the specialised kernel is used when every tensor of the set qualifies in the same way
    FastKind fk = fast_kind(tensors[0].info);
    for (uint32_t t = 1; t < n_tensors && fk.ok; t++) {
        const FastKind k = fast_kind(tensors[t].info);
        if (!k.ok || k.exp_kind != fk.exp_kind || k.sm_kind != fk.sm_kind || tensors[t].info.xor_delta != tensors[0].info.xor_delta) fk.ok = false;
    }
    // small chunks (S < 64): the sub-wavefront FP8 kernel when every tensor qualifies
    bool sub = S < 64;
    for (uint32_t t = 0; t < n_tensors && sub; t++) {
        const zc_info &info = tensors[t].info;
        const uint64_t raw_bytes = info.n_elems * (uint64_t)elem_bits(fmt) / 8, per_chunk = (uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(fmt);
        const uint64_t need = tensors[t].d_chunk_ids ? (uint64_t)tensors[t].n_chunk_ids * info.chunk_bytes : raw_bytes;
        if (!sub_ok(info, need) || info.xor_delta != tensors[0].info.xor_delta) sub = false;
        if (tensors[t].d_chunk_ids && info.n_elems % per_chunk) sub = false;
    }
    // otherwise the 64-lane full-chunk kernel, when every tensor qualifies
    uint32_t rings = 0;
    if (!fk.ok && !sub) {
        rings = 2;
        uint32_t most = 1;
        for (uint32_t t = 0; t < n_tensors && rings; t++) {
            const uint32_t r = s64_rings(tensors[t].info);
            if (r == 0 || tensors[t].info.xor_delta != tensors[0].info.xor_delta) rings = 0;
            else if (r > most) most = r;
        }
        if (rings) rings = most;
    }
    bool split = rings != 0;
    for (uint32_t t = 0; t < n_tensors && split; t++) split = s64_split_ok(tensors[t].info);
    bool e5m2 = rings != 0;
    for (uint32_t t = 0; t < n_tensors && e5m2; t++) e5m2 = e5m2_s64_ok(tensors[t].info);
    // BF16 sets whose every tensor has the shape of the BF16 kernel go there instead
    uint32_t bf16_rings = rings ? 1 : 0;
    for (uint32_t t = 0; t < n_tensors && bf16_rings; t++) {
        const uint32_t r = bf16_s64_rings(tensors[t].info);
        bf16_rings = r == 0 ? 0 : (r > bf16_rings ? r : bf16_rings);
    }
    const bool fast = fk.ok || rings != 0 || sub;
    uint64_t all_slots = 0;
    for (uint32_t t = 0; t < n_tensors; t++) all_slots += tensors[t].d_chunk_ids ? tensors[t].n_chunk_ids : tensors[t].info.n_chunks;
    const uint32_t spg = sub ? sub_slots_per_group(S, all_slots) : split ? 1u : kWavesPerGroup;
    std::vector<TensorDev> descs(n_tensors);
    std::vector<WorkItem> fast_work, work;
    for (uint32_t t = 0; t < n_tensors; t++) {
        const zc_tensor &x = tensors[t];
        const zc_info &info = x.info;
        if (!x.d_comp || !aligned16(x.d_comp) || (info.n_elems && (!x.d_dst || !aligned16(x.d_dst)))) return ZC_ERR_INVALID_ARG;
        if (info.n_fields == 3 && info.n_elems && (!x.d_scales_out || !aligned16(x.d_scales_out))) return ZC_ERR_INVALID_ARG;
        if (info.xor_delta && (!x.d_xor_base || !aligned16(x.d_xor_base))) return ZC_ERR_INVALID_ARG;
        descs[t] = make_desc(info);
        descs[t].comp = (uint8_t *)x.d_comp; descs[t].dst = (uint8_t *)x.d_dst; descs[t].scales_out = (uint8_t *)x.d_scales_out;
        descs[t].base = info.xor_delta ? (const uint8_t *)x.d_xor_base : nullptr;
        const uint64_t raw = (info.n_elems * (uint64_t)elem_bits(fmt) + 7) / 8;
        descs[t].ids = x.d_chunk_ids; descs[t].n_ids = x.d_chunk_ids ? x.n_chunk_ids : 0;
        descs[t].dst_bytes = x.d_chunk_ids ? (uint64_t)x.n_chunk_ids * info.chunk_bytes : raw;
        const uint32_t slots = x.d_chunk_ids ? x.n_chunk_ids : info.n_chunks;
        uint32_t first_generic = 0;
        const uint64_t per_chunk = (uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(fmt);
        if (fast && (sub || !x.d_chunk_ids)) {
            const uint32_t n_full = (uint32_t)(info.n_elems / per_chunk);
            const uint32_t n_fast = x.d_chunk_ids ? slots : n_full;        // lists reach here only when every chunk is whole
            for (uint32_t c = 0; c < n_fast; c += spg) fast_work.push_back({t, c});
            first_generic = n_fast;
        } else if (fk.ok && x.d_chunk_ids) {
            // a list over a container the FP8 kernel takes: every slot to that kernel's build for lists, which takes the
            // whole chunks; every slot to the second list too when the tensor has a short last chunk the list may name
            // (the build for such chunks then skips the whole ones)
            for (uint32_t c = 0; c < slots; c += spg) fast_work.push_back({t, c});
            if (info.n_elems % per_chunk == 0) first_generic = slots;
        }                                                                   // any other id list with 64-lane chunks goes to the second list
        for (uint32_t c = first_generic; c < slots; c += cpi) work.push_back({t, c});
    }
    order_for_xcds(fast_work);
    const uint64_t descs_bytes = align256((uint64_t)n_tensors * sizeof(TensorDev));
    const uint64_t fast_bytes = align256(fast_work.size() * sizeof(WorkItem));
    if (ws_bytes < descs_bytes + fast_bytes + work.size() * sizeof(WorkItem)) return ZC_ERR_BUFFER_TOO_SMALL;
    uint8_t *ws = (uint8_t *)d_ws;
    // one copy from the page-locked staging buffer: no wait, the host arrays above may go away at once
    const Piece all[3] = {{0, descs.data(), descs.size() * sizeof(TensorDev)},
                          {descs_bytes, fast_work.data(), fast_work.size() * sizeof(WorkItem)},
                          {descs_bytes + fast_bytes, work.data(), work.size() * sizeof(WorkItem)}};
    const zc_status up = stage_upload(ws, 0, descs_bytes + fast_bytes + work.size() * sizeof(WorkItem), all, 3, stream);
    if (up) return up;
    plan->format = fmt; plan->streams = S; plan->n_tensors = n_tensors;
    plan->n_fast_work = (uint32_t)fast_work.size(); plan->n_work = (uint32_t)work.size();
    plan->fast_exp_kind = (uint32_t)fk.exp_kind; plan->fast_sm_kind = (uint32_t)fk.sm_kind; plan->xor_delta = tensors[0].info.xor_delta;
    plan->fast_kernel = fk.ok ? 1u : (rings ? (e5m2 ? 7u : bf16_rings ? 6u : split ? 4u : 2u) : (sub ? (fmt == ZC_FMT_BF16 ? 5u : 3u) : 0u));
    plan->n_rings = sub ? spg : (bf16_rings ? bf16_rings : rings);
    plan->scattered = 0;
    for (uint32_t t = 0; t < n_tensors; t++) if (tensors[t].d_chunk_ids) plan->scattered = 1;
    // the second list (chunks that are not whole rows, id lists with 64 lanes) goes through the 64-lane kernel's build for
    // such chunks when every tensor allows it
    plan->tail_kernel = 1;
    for (uint32_t t = 0; t < n_tensors && plan->tail_kernel; t++)
        if (tensors[t].info.n_elems && (!s64_tail_ok(tensors[t].info) || tensors[t].info.xor_delta != tensors[0].info.xor_delta)) plan->tail_kernel = 0;
    // lists over containers the FP8 kernel takes: that kernel has the whole chunks of the second list
    if (plan->tail_kernel && fk.ok && plan->scattered) plan->tail_kernel = 2;
    plan->fast_work_offset = descs_bytes; plan->work_offset = descs_bytes + fast_bytes;
    return ZC_OK;
}

zc_status zc_decompress_batch_run(const zc_batch_plan *plan, const void *d_ws, void *stream)
{
    if (!plan) return ZC_ERR_INVALID_ARG;
    if (plan->n_tensors == 0 || (plan->n_work == 0 && plan->n_fast_work == 0)) return ZC_OK;
    if (!d_ws || !elem_bits(plan->format) || plan->streams == 0 || plan->streams > 64 || (plan->streams & (plan->streams - 1))) return ZC_ERR_INVALID_ARG;
    const uint8_t *ws = (const uint8_t *)d_ws;
    if (plan->n_fast_work && plan->fast_kernel == 1)
        LAUNCH_TRY(launch_decode_fp8_fast((int)plan->fast_exp_kind, (int)plan->fast_sm_kind, plan->xor_delta != 0, plan->scattered != 0, (const TensorDev *)ws,
                                          (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && (plan->fast_kernel == 2 || plan->fast_kernel == 4))
        LAUNCH_TRY(launch_decode_s64(plan->format, plan->n_rings, plan->xor_delta != 0, plan->fast_kernel == 4, (const TensorDev *)ws,
                                     (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 6)
        LAUNCH_TRY(launch_decode_bf16_s64(plan->n_rings, plan->xor_delta != 0, (const TensorDev *)ws,
                                          (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 7)
        LAUNCH_TRY(launch_decode_e5m2(plan->xor_delta != 0, (const TensorDev *)ws, (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 3)
        LAUNCH_TRY(launch_decode_fp8_sub(plan->streams, plan->xor_delta != 0, plan->scattered != 0, (const TensorDev *)ws,
                                         (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, plan->n_rings, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 5)
        LAUNCH_TRY(launch_decode_bf16_sub(plan->streams, plan->xor_delta != 0, (const TensorDev *)ws,
                                          (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, plan->n_rings, stream));
    else if (plan->n_fast_work) return ZC_ERR_INVALID_ARG;
    if (plan->n_work && (plan->tail_kernel == 1 || plan->tail_kernel == 2) && plan->streams == 64)
        LAUNCH_TRY(launch_decode_s64_tail(plan->format, plan->xor_delta != 0, (const TensorDev *)ws, (const WorkItem *)(ws + plan->work_offset), plan->n_work,
                                          nullptr, 0, plan->tail_kernel == 2, stream));
    else if (plan->n_work)
        LAUNCH_TRY(launch_decode(plan->format, (const TensorDev *)ws, (const WorkItem *)(ws + plan->work_offset), plan->n_work,
                                 chunks_per_work_item(plan->streams), nullptr, 0, stream));
    return ZC_OK;
}

zc_status zc_decompress_batch(const zc_tensor *tensors, uint32_t n_tensors, void *d_ws, uint64_t ws_bytes, void *stream)
{
    zc_batch_plan plan;
    zc_status st = zc_decompress_batch_plan(tensors, n_tensors, d_ws, ws_bytes, &plan, stream);
    if (st) return st;
    return zc_decompress_batch_run(&plan, d_ws, stream);
}

}  // extern "C"
