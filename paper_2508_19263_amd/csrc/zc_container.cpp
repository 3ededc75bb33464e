// Container layout, parameter checks and container validation: host arithmetic only (no HIP call), so that
// this file also builds with a plain C++ compiler for the CPU tests and the sanitizer builds.
// See include/zc.h for the container's description.
#include <algorithm>
#include <cstring>
#include <vector>

#include "zc_host.h"

namespace zc {

// zc_params is size-versioned: the first layout ended with `policy` (32 bytes), the current one adds `flags`.
// A caller built against either is served; fields it does not have read as zero.
constexpr uint32_t kParamsBytesV1 = 32;

zc_status check_params(const zc_params *given, Geometry *g)
{
    if (!given) return ZC_ERR_INVALID_ARG;
    if (given->struct_size != sizeof(zc_params) && given->struct_size != kParamsBytesV1) return ZC_ERR_UNSUPPORTED;
    zc_params local;
    std::memset(&local, 0, sizeof(local));
    std::memcpy(&local, given, given->struct_size);
    const zc_params *p = &local;
    if (!elem_bits(p->format)) return ZC_ERR_UNSUPPORTED;
    if (p->flags & ~(uint32_t)(ZC_FLAG_HOST_CODES | ZC_FLAG_REVERSE_FIELDS)) return ZC_ERR_INVALID_ARG;
    g->host_codes = (p->flags & ZC_FLAG_HOST_CODES) != 0;
    g->reversed = (p->flags & ZC_FLAG_REVERSE_FIELDS) != 0;
    g->fmt = p->format;
    g->S = p->streams_per_chunk ? p->streams_per_chunk : 64;
    if (g->S > 64 || (g->S & (g->S - 1))) return ZC_ERR_INVALID_ARG;
    if (p->chunk_bytes == 0 || p->chunk_bytes % 16) return ZC_ERR_INVALID_ARG;
    if (is_fp4(p->format) && p->chunk_bytes % 256) return ZC_ERR_INVALID_ARG;
    if (p->policy > ZC_POLICY_AUTO) return ZC_ERR_INVALID_ARG;
    g->nf = (uint32_t)num_fields(p->format);
    g->chunk_bytes = p->chunk_bytes;
    g->elems_per_chunk = (uint64_t)p->chunk_bytes * 8 / (uint64_t)elem_bits(p->format);
    for (uint32_t f = 0; f < g->nf; f++) {
        const int sb = sym_bits(p->format, (int)f);
        int L = (int)p->max_code_len[f];
        if (L == 0) L = sb == 8 ? 16 : 8;
        if (L < sb || L > 16) return ZC_ERR_INVALID_ARG;      // 2^L must cover the alphabet
        g->limit[f] = L;
    }
    return ZC_OK;
}

zc_status check_count(const Geometry &g, uint64_t n_elems, uint64_t *n_chunks)
{
    if (is_fp4(g.fmt) && n_elems % scale_block(g.fmt)) return ZC_ERR_INVALID_ARG;
    const uint64_t nc = (n_elems + g.elems_per_chunk - 1) / g.elems_per_chunk;
    if (nc >= 0xFFFFFFFFull) return ZC_ERR_INVALID_ARG;
    *n_chunks = nc;
    return ZC_OK;
}

uint64_t field_symbols(uint32_t fmt, int f, uint64_t n_elems)
{
    if (f == 2) return n_elems / scale_block(fmt);
    const uint64_t grp = (uint64_t)group_of(fmt);
    return (n_elems + grp - 1) / grp;                       // a last partial group counts as one symbol
}

// offsets of tables / indices / payload for a tensor of nc chunks
void layout(uint32_t fmt, uint64_t nc, uint64_t table_off[3], uint64_t index_off[3], uint64_t *payload_off)
{
    uint64_t off = kHeaderBytes;
    const int nf = num_fields(fmt);
    for (int f = 0; f < nf; f++) { table_off[f] = off; off += pad16(1ull << sym_bits(fmt, f)); }
    for (int f = 0; f < nf; f++) { index_off[f] = off; off += pad16(4 * (nc + 1)); }
    *payload_off = off;
}

void fill_info(const Geometry &g, uint32_t policy, bool xor_delta, uint64_t n_elems, uint64_t nc, const FieldCode fc[3], uint64_t total, zc_info *info)
{
    std::memset(info, 0, sizeof(*info));
    info->format = g.fmt; info->policy = policy; info->streams = g.S; info->n_fields = g.nf;
    info->xor_delta = xor_delta; info->chunk_bytes = g.chunk_bytes; info->n_chunks = (uint32_t)nc;
    info->payload_order = g.reversed ? 1 : 0;
    info->n_elems = n_elems; info->total_bytes = total;
    layout(g.fmt, nc, info->table_offset, info->index_offset, &info->payload_offset);
    for (uint32_t f = 0; f < g.nf; f++) {
        info->mode[f] = (uint8_t)fc[f].mode; info->sym_bits[f] = (uint8_t)sym_bits(g.fmt, (int)f);
        info->max_len[f] = (uint8_t)fc[f].lmax; info->const_symbol[f] = (uint8_t)fc[f].konst;
        std::memcpy(info->code_len[f], fc[f].len, 256);
    }
}

// header + tables exactly as they sit at the start of the container (total_bytes is
// patched in by the scan kernel)
void serialize_blob(const zc_info &info, uint8_t *blob)
{
    std::memset(blob, 0, kBlobBytes);
    put32(blob, kMagic);
    blob[4] = 1; blob[6] = (uint8_t)info.format; blob[7] = (uint8_t)info.policy;
    blob[8] = (uint8_t)info.streams; blob[9] = (uint8_t)info.n_fields; blob[10] = (uint8_t)((info.xor_delta ? 1 : 0) | (info.payload_order ? 2 : 0));
    put32(blob + 12, info.chunk_bytes);
    put64(blob + 16, info.n_elems);
    put32(blob + 24, info.n_chunks);
    for (uint32_t f = 0; f < info.n_fields; f++) {
        blob[32 + 4 * f] = info.mode[f]; blob[33 + 4 * f] = info.sym_bits[f];
        blob[34 + 4 * f] = info.max_len[f]; blob[35 + 4 * f] = info.const_symbol[f];
        std::memcpy(blob + info.table_offset[f], info.code_len[f], (size_t)1 << info.sym_bits[f]);
    }
    put64(blob + 48, info.total_bytes);
    put64(blob + 56, info.payload_offset);
}

// how the specialised kernels treat a field: 0 table, 1 flat code, 2 raw, 3 constant
uint8_t field_kind(uint32_t mode, uint32_t sym_bits_, const uint8_t *code_len)
{
    if (mode == ZC_MODE_RAW) return 2;
    if (mode != ZC_MODE_HUFF) return 3;
    // flat: every symbol present with length sym_bits, so the canonical code is the symbol itself
    for (uint32_t v = 0; v < (1u << sym_bits_); v++) if (code_len[v] != sym_bits_) return 0;
    return 1;
}

TensorDev make_desc(const zc_info &info)
{
    TensorDev d;
    std::memset(&d, 0, sizeof(d));
    d.n_elems = info.n_elems; d.total_bytes = info.total_bytes; d.payload_off = info.payload_offset;
    d.n_chunks = info.n_chunks; d.chunk_bytes = info.chunk_bytes; d.streams = info.streams;
    for (uint32_t f = 0; f < info.n_fields; f++) {
        d.table_off[f] = (uint32_t)info.table_offset[f]; d.index_off[f] = (uint32_t)info.index_offset[f];
        d.mode[f] = info.mode[f]; d.lmax[f] = info.max_len[f]; d.konst[f] = info.const_symbol[f];
        d.period[f] = (uint8_t)refill_period(run_len(info.format, (int)f), info.max_len[f]);
        d.kind[f] = field_kind(info.mode[f], info.sym_bits[f], info.code_len[f]);
    }
    return d;
}

// slots one workgroup of the sub-wavefront kernel takes: enough passes to amortise its table
// build, few enough to leave >= ~2048 workgroups
uint32_t sub_slots_per_group(uint32_t streams, uint64_t slots)
{
    const uint32_t per_pass = kWavesPerGroup * (64 / streams);
    uint64_t passes = slots / (2048ull * per_pass);
    if (passes < 1) passes = 1;
    if (passes > 8) passes = 8;
    return (uint32_t)passes * per_pass;
}

// Workgroups are handed to the 8 XCDs (each with an L2 of its own) in turn, so workgroup p runs on XCD
// p % 8.  Reordering the list so that every XCD walks through one contiguous eighth of it keeps an XCD's
// wavefronts in neighbouring chunks (measured on the FP8 weight set: 2.60 instead of 2.63 ms).
void order_for_xcds(std::vector<WorkItem> &items)
{
    const size_t n = items.size();
    if (n < 16) return;
    std::vector<WorkItem> out(n);
    for (size_t p = 0; p < n; p++) out[p] = items[xcd_order_source(p, n)];
    items.swap(out);
}

zc_status parse_info(const uint8_t *c, uint64_t have, uint64_t comp_bytes, zc_info *out)
{
    if (have < kHeaderBytes || comp_bytes < kHeaderBytes) return ZC_ERR_CORRUPT;
    if (get32(c) != kMagic || c[4] != 1 || c[5] != 0) return ZC_ERR_CORRUPT;
    std::memset(out, 0, sizeof(*out));
    out->format = c[6]; out->policy = c[7]; out->streams = c[8]; out->n_fields = c[9]; out->xor_delta = c[10] & 1; out->payload_order = (c[10] >> 1) & 1;
    out->chunk_bytes = get32(c + 12); out->n_elems = get64(c + 16); out->n_chunks = get32(c + 24);
    out->total_bytes = get64(c + 48); out->payload_offset = get64(c + 56);
    zc_params p;
    std::memset(&p, 0, sizeof(p));
    p.struct_size = sizeof(p); p.format = out->format; p.chunk_bytes = out->chunk_bytes; p.streams_per_chunk = out->streams; p.policy = out->policy;
    Geometry g;
    if (out->streams == 0 || check_params(&p, &g) != ZC_OK || out->n_fields != g.nf) return ZC_ERR_CORRUPT;
    uint64_t nc;
    if (check_count(g, out->n_elems, &nc) != ZC_OK || nc != out->n_chunks) return ZC_ERR_CORRUPT;
    uint64_t payload;
    layout(out->format, nc, out->table_offset, out->index_offset, &payload);
    if (payload != out->payload_offset || out->total_bytes < payload || out->total_bytes > comp_bytes || (out->total_bytes - payload) % 16) return ZC_ERR_CORRUPT;
    for (uint32_t f = 0; f < g.nf; f++) {
        out->mode[f] = c[32 + 4 * f]; out->sym_bits[f] = c[33 + 4 * f]; out->max_len[f] = c[34 + 4 * f]; out->const_symbol[f] = c[35 + 4 * f];
        if (out->mode[f] > ZC_MODE_CONST || out->sym_bits[f] != sym_bits(out->format, (int)f)) return ZC_ERR_CORRUPT;
        const uint32_t A = 1u << out->sym_bits[f];
        if (out->table_offset[f] + A > have) return ZC_ERR_CORRUPT;
        std::memcpy(out->code_len[f], c + out->table_offset[f], A);
        if (out->mode[f] == ZC_MODE_HUFF) {
            uint64_t kraft = 0;
            uint32_t lmax = 0;
            for (uint32_t v = 0; v < A; v++) {
                const uint32_t l = out->code_len[f][v];
                if (l > 16) return ZC_ERR_CORRUPT;
                if (l) { kraft += 1ull << (16 - l); if (l > lmax) lmax = l; }
            }
            if (kraft != 65536 || lmax != out->max_len[f]) return ZC_ERR_CORRUPT;   // complete prefix code
        } else if (out->const_symbol[f] >= A) return ZC_ERR_CORRUPT;
        if (out->mode[f] == ZC_MODE_EMPTY && out->n_elems) return ZC_ERR_CORRUPT;
    }
    return ZC_OK;
}

zc_status check_index_field(const uint32_t *idx, uint32_t n_chunks, uint32_t *prev)
{
    if (idx[0] != *prev) return ZC_ERR_CORRUPT;             // a field's streams start where the field before ended
    uint32_t last = *prev;
    for (uint64_t i = 0; i <= n_chunks; i++) {
        if (idx[i] < last) return ZC_ERR_CORRUPT;
        last = idx[i];
    }
    *prev = last;
    return ZC_OK;
}

}  // namespace zc

using namespace zc;

// ----------------------------------------------------------------------- C ABI (host-only entry points)

extern "C" {

const char *zc_status_string(zc_status s)
{
    switch (s) {
    case ZC_OK: return "ok";
    case ZC_ERR_INVALID_ARG: return "invalid argument";
    case ZC_ERR_UNSUPPORTED: return "unsupported format or struct size";
    case ZC_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case ZC_ERR_CORRUPT: return "corrupt container";
    case ZC_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

uint64_t zc_compress_bound(uint64_t n_elems, const zc_params *params)
{
    Geometry g;
    uint64_t nc;
    if (check_params(params, &g) || check_count(g, n_elems, &nc)) return 0;
    uint64_t table_off[3], index_off[3], total;
    layout(g.fmt, nc, table_off, index_off, &total);
    for (uint32_t f = 0; f < g.nf; f++) {
        // per lane: its bits rounded up to a word plus two look-ahead words; per stream: padding
        const uint64_t ns = field_symbols(g.fmt, (int)f, n_elems);
        total += nc * ((uint64_t)g.S * 12 + 32) + pad16((ns * (uint64_t)g.limit[f] + 7) / 8);
    }
    return total;
}

zc_status zc_build_code(const uint64_t *hist, uint32_t alphabet, uint32_t limit, uint8_t *len_out, uint16_t *code_out)
{
    if (!hist || !len_out || !code_out || alphabet == 0 || alphabet > 256) return ZC_ERR_INVALID_ARG;
    if (!build_code_lengths(hist, (int)alphabet, (int)limit, len_out)) return ZC_ERR_INVALID_ARG;
    assign_canonical(len_out, (int)alphabet, code_out);
    return ZC_OK;
}

int zc_code_stale(const zc_info *code, const zc_info *written, double slack)
{
    if (!code || !written || code->format != written->format || code->n_elems == 0 || written->n_elems == 0) return -1;
    if (!elem_bits(code->format) || !(slack >= 0.0)) return -1;
    auto raw = [](const zc_info *i) {
        return (double)((i->n_elems * (uint64_t)elem_bits(i->format) + 7) / 8 + (is_fp4(i->format) ? i->n_elems / scale_block(i->format) : 0));
    };
    return (double)written->total_bytes / raw(written) > (double)code->total_bytes / raw(code) + slack ? 1 : 0;
}

zc_status zc_validate_container(const void *host_bytes, uint64_t have_bytes, uint64_t container_bytes, int check_index, zc_info *out)
{
    if (!host_bytes || !out || have_bytes > container_bytes) return ZC_ERR_INVALID_ARG;
    const uint8_t *c = (const uint8_t *)host_bytes;
    zc_status st = parse_info(c, have_bytes, container_bytes, out);
    if (st || !check_index) return st;
    if (out->payload_offset > have_bytes) return ZC_ERR_INVALID_ARG;   // the whole index must be there to be checked
    uint32_t prev = 0;
    std::vector<uint32_t> idx((size_t)out->n_chunks + 1);
    for (uint32_t k = 0; k < out->n_fields; k++) {
        const uint32_t f = field_at(k, out->n_fields, out->payload_order != 0);
        std::memcpy(idx.data(), c + out->index_offset[f], idx.size() * 4);
        st = check_index_field(idx.data(), out->n_chunks, &prev);
        if (st) return st;
    }
    return out->payload_offset + 16ull * prev == out->total_bytes ? ZC_OK : ZC_ERR_CORRUPT;
}

}  // extern "C"
