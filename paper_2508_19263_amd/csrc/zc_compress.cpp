// The compress side of the C ABI (zc_compress*, zc_stats, zc_train_code, zc_workspace_bytes): argument checks,
// workspace layout, work lists, and the kernel sequence histogram -> code construction -> stream sizes -> scan ->
// encode.  A plain compress call builds its codes on the device; statistics, dictionary training and
// ZC_FLAG_HOST_CODES build them on the host.  See include/zc.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <optional>
#include <thread>
#include <vector>

#include "zc_host.h"

namespace zc {

// ---- workspace carving ------------------------------------------------------


// The geometry for which the histogram pass also counts exponents per chunk lane, so that the size pass need
// not read the source again (k_hist_fp8_lanes, k_sizes_fp8_counts)
bool lane_counts_shape(const Geometry &g) { return g.fmt == ZC_FMT_FP8_E4M3 && g.S == 64 && g.chunk_bytes == kHistBlockBytes; }
// The same for BF16 and FP8 in byte symbols (k_hist_rows8_lanes, k_sizes_rows8_counts): 64 KiB of counts per chunk
bool lane_counts8_shape(const Geometry &g) { return (g.fmt == ZC_FMT_BF16 || g.fmt == ZC_FMT_FP8_E4M3_BYTES) && g.S == 64 && g.chunk_bytes == kHistBlockBytes; }
// and for FP8 E5M2 (k_hist_fp8_lanes<true>, k_sizes_e5m2_counts): 40 counts per chunk lane
bool lane_counts_e5m2_shape(const Geometry &g) { return g.fmt == ZC_FMT_FP8_E5M2 && g.S == 64 && g.chunk_bytes == kHistBlockBytes; }

zc_status plan_workspace(const Geometry &g, const uint64_t *n_elems, uint32_t T, Workspace *w)
{
    uint64_t hw = 0, sw = 0, cw = 0, ww = 0, units = 0;
    const uint32_t cpi = chunks_per_work_item(g.S);
    for (uint32_t t = 0; t < T; t++) {
        uint64_t nc;
        zc_status st = check_count(g, n_elems[t], &nc);
        if (st) return st;
        const uint64_t bytes = (n_elems[t] * (uint64_t)elem_bits(g.fmt) + 7) / 8;
        hw += (bytes + kHistBlockBytes - 1) / kHistBlockBytes;
        if (g.nf == 3) sw += (n_elems[t] / scale_block(g.fmt) + kHistBlockBytes - 1) / kHistBlockBytes;
        cw += (nc + cpi - 1) / cpi;
        ww += is_fp4(g.fmt) ? nc : (nc + cpi - 1) / cpi;          // FP4: one whole chunk per work item
        units += nc * g.nf;
    }
    if (hw > 0x7FFFFFFFull || cw > 0x7FFFFFFFull || ww > 0x7FFFFFFFull || units > 0xFFFFFFFFull) return ZC_ERR_INVALID_ARG;
    uint64_t off = 0;
    // what the host writes comes first and is contiguous, so that it goes up in one copy
    w->descs = off; off = align256(off + (uint64_t)T * sizeof(TensorDev));
    w->hist_work = off; off = align256(off + hw * sizeof(WorkItem));
    w->scale_work = off; off = align256(off + sw * sizeof(WorkItem));
    w->chunk_work = off; off = align256(off + cw * sizeof(WorkItem));
    w->fast_work = off; off = align256(off + cw * sizeof(WorkItem));
    w->whole_work = off; off = align256(off + ww * sizeof(WorkItem));
    w->other_work = off; off = align256(off + cw * sizeof(WorkItem));
    w->blobs = off; off = align256(off + (uint64_t)T * kBlobBytes);
    w->enc = off; off = align256(off + (uint64_t)T * 768 * 4);      // last: written on the device when the code is built there
    w->host_end = off;
    w->hist = off; off = align256(off + (uint64_t)T * 3 * 256 * 8);
    w->units = off; off = align256(off + units * 4);
    w->scan = off; off = align256(off + (uint64_t)T * sizeof(ScanOut));
    // FP8 with 64 lanes and chunks of one histogram block: 16 exponent counts of 16 bits per chunk lane
    w->lane_counts = off;
    if (lane_counts_shape(g)) off = align256(off + units / 2 * (64 * 16 * 2));
    // BF16 / FP8 in byte symbols, same geometry: 256 counts of 16 bits per chunk lane and field
    if (lane_counts8_shape(g)) off = align256(off + units / 2 * (2 * 64 * 256 * 2));
    // FP8 E5M2, same geometry: 32 exponent and 8 sign+mantissa counts of 16 bits per chunk lane
    if (lane_counts_e5m2_shape(g)) off = align256(off + units / 2 * (64 * 40 * 2));
    w->total = off;
    w->n_hist_work = (uint32_t)hw; w->n_scale_work = (uint32_t)sw; w->n_chunk_work = (uint32_t)cw; w->n_units = units;
    return ZC_OK;
}

// ---- a few threads for the per-tensor code construction ------------------------
// Tensors are independent, so a large set is split into contiguous ranges, one per thread; the calling
// thread takes the first range.  The destructor joins whatever was started, so an early return between
// construction and run() is safe (the workers then leave without doing anything).

// The lists of one tensor when the code is built on the device: the route (which kernel suits the code) is not
// known yet, so whole chunks are listed for every kernel that may take them, and the kernel that is not meant
// returns at once.
TensorLists device_code_lists(const Geometry &g, const CompressShape &sh, uint64_t n_elems, uint64_t nc, bool fast_shape)
{
    TensorLists L = {};
    const uint64_t bytes = (n_elems * (uint64_t)elem_bits(g.fmt) + 7) / 8;
    const uint32_t whole_chunks = (uint32_t)(n_elems / g.elems_per_chunk);
    // a histogram block is a chunk when sh.lanes is set: whole chunks go to the kernel that counts per lane too
    const uint32_t lane_blocks = (sh.lanes || sh.lanes8 || sh.lanes_e5m2) ? whole_chunks : 0;
    L.lane_hist = {0, lane_blocks, 1};
    L.hist = {lane_blocks, (uint32_t)((bytes + kHistBlockBytes - 1) / kHistBlockBytes), 1};
    if (L.hist.end < L.hist.first) L.hist.end = L.hist.first;
    if (g.nf == 3) L.scale = {0, (uint32_t)((n_elems / scale_block(g.fmt) + kHistBlockBytes - 1) / kHistBlockBytes), 1};
    if (fast_shape) L.fast = {0, whole_chunks, sh.fast_step};
    if (sh.whole_shape) L.whole = {0, whole_chunks, sh.whole_step};
    else if (fast_shape) L.other = {0, whole_chunks, sh.cpi};
    L.slow = {(fast_shape || sh.whole_shape) ? whole_chunks : 0u, (uint32_t)nc, sh.cpi};
    return L;
}

CompressShape compress_shape(const Geometry &g, bool device_codes, uint64_t all_chunks)
{
    CompressShape sh;
    sh.cpi = chunks_per_work_item(g.S);
    sh.lanes = device_codes && lane_counts_shape(g);
    sh.lanes8 = device_codes && lane_counts8_shape(g);
    sh.lanes_e5m2 = device_codes && lane_counts_e5m2_shape(g);
    sh.bf16 = g.fmt == ZC_FMT_BF16;
    sh.whole_shape = g.S == 64 && g.chunk_bytes % 1024 == 0;
    sh.rows8 = sh.whole_shape && (g.fmt == ZC_FMT_BF16 || g.fmt == ZC_FMT_FP8_E4M3_BYTES || g.fmt == ZC_FMT_FP8_E5M2);
    // FP4 elements rarely compress, so their fields are stored plainly and a chunk's rows can be shared by the four
    // wavefronts of a workgroup: one chunk per work item there
    sh.whole_mode = is_fp4(g.fmt) ? 2 : 1;
    sh.whole_step = sh.whole_mode == 2 ? 1u : kWavesPerGroup;
    sh.fast_step = g.S == 64 ? kWavesPerGroup : sub_slots_per_group(g.S, all_chunks);
    return sh;
}

// Geometry the specialised size/encode kernels take: FP8 with 64 lanes and chunks of whole 1 KiB rows, or FP8 /
// BF16 with 4..32 lanes per chunk (pages) for the sub-wavefront kernels as long as the tensor AND the payload of
// its container fit their 32-bit offsets (with tiny pages the look-ahead words make the worst-case container
// larger than the tensor).  Whether the code suits them too is known once the code is: TensorDev::route.
bool compress_fast_shape(const Geometry &g, uint64_t n_elems, uint64_t bound_bytes)
{
    const bool page_ok = g.S >= 4 && g.S < 64 && g.chunk_bytes % (16 * g.S) == 0 && bound_bytes <= 0xF0000000ull;
    if (g.fmt == ZC_FMT_BF16) return page_ok && n_elems * 2 <= 0xF0000000ull;
    if (g.fmt != ZC_FMT_FP8_E4M3) return false;
    return g.S == 64 ? g.chunk_bytes % 1024 == 0 : (page_ok && n_elems <= 0xF0000000ull);
}

// field split + histogram (a1-a3)
zc_status CompressQueue::queue_histogram() const
{
    LAUNCH_TRY(launch_zero(d_hist(), (uint64_t)T * 3 * 256, stream));
    LAUNCH_TRY(launch_hist(g.fmt, d_descs(), d_list(w.hist_work), n_hist, 0, d_hist(), stream));
    if (sh.lanes8) LAUNCH_TRY(launch_hist_rows8_lanes(g.fmt, d_descs(), d_list(w.hist_work) + n_hist, n_lane_hist, d_hist(), (uint32_t *)d_lane_counts(), stream));
    else LAUNCH_TRY(launch_hist_fp8_lanes(sh.lanes_e5m2, d_descs(), d_list(w.hist_work) + n_hist, n_lane_hist, d_hist(), d_lane_counts(), stream));
    if (g.nf == 3) LAUNCH_TRY(launch_hist(g.fmt, d_descs(), d_list(w.scale_work), n_scale, (int)scale_block(g.fmt), d_hist(), stream));
    return ZC_OK;
}

// code construction on the device (a4)
zc_status CompressQueue::queue_codes(uint32_t policy) const
{
    CodeParams cp;
    cp.fmt = g.fmt; cp.policy = policy; cp.nf = g.nf; cp.blob_bytes = (uint32_t)kBlobBytes; cp.run_len = (uint32_t)run_len(g.fmt, 0);
    for (int f = 0; f < kMaxFields; f++) cp.limit[f] = f < (int)g.nf ? g.limit[f] : 0;
    LAUNCH_TRY(launch_codes(d_descs(), T, d_hist(), cp, ws + w.blobs, d_enc(), stream));
    return ZC_OK;
}

// stream sizes (a5) and their exclusive scan into the chunk index (a6)
zc_status CompressQueue::queue_sizes_and_scan() const
{
    if (chained)
        LAUNCH_TRY(launch_compress_pages_chained(g.S, sh.bf16 ? 16u : 0u, chain_hold, d_descs(), d_list(w.fast_work), n_fast, chain_step, d_enc(), ws + w.blobs, (uint32_t)kBlobBytes,
                                                 (uint64_t *)(ws + chain_status), (uint64_t *)(ws + chain_counter), (ScanOut *)(ws + w.scan), stream));
    else if (g.S == 64 && sh.lanes) LAUNCH_TRY(launch_sizes_fp8_counts(d_descs(), d_list(w.fast_work), n_fast, d_enc(), d_lane_counts(), d_units(), stream));
    else if (g.S == 64) LAUNCH_TRY(launch_sizes_fp8(d_descs(), d_list(w.fast_work), n_fast, d_enc(), d_units(), stream));
    else LAUNCH_TRY(launch_encode_fp8_sub(g.S, 0, sh.bf16, d_descs(), d_list(w.fast_work), n_fast, d_enc(), d_units(), sh.fast_step, stream));
    // generic kernels: the whole-chunk list leaves route 1 to the FP8 kernels (route 2 there is the BF16 encoder,
    // whose sizes come from this pass); the list of page-shaped tensors leaves both routes to the page kernels
    // (with the symbols counted per lane, route 2 has its sizes from the counts)
    if (sh.lanes8) LAUNCH_TRY(launch_sizes_rows8_counts(g.fmt, d_descs(), d_list(w.whole_work), n_whole, d_enc(), (const uint32_t *)d_lane_counts(), d_units(), stream));
    // (E5M2 has no encoder of its own, route 0, and all its whole chunks are sized from the counts)
    if (sh.lanes_e5m2) LAUNCH_TRY(launch_sizes_e5m2_counts(d_descs(), d_list(w.whole_work), n_whole, d_enc(), d_lane_counts(), d_units(), stream));
    else
        LAUNCH_TRY(launch_sizes(g.fmt, sh.whole_mode, sh.lanes8 ? 0x6 : 0x2, d_descs(), d_list(w.whole_work), n_whole, d_enc(), d_units(), stream));
    LAUNCH_TRY(launch_sizes(g.fmt, 0, 0x6, d_descs(), d_list(w.other_work), n_other, d_enc(), d_units(), stream));
    // what the whole-chunk kernels leave over: with 64 lanes and chunks of whole rows only a tensor's short last chunk,
    // sized from its lanes' bit totals; otherwise every chunk, walked by the generic size pass
    if (sh.whole_shape && g.nf == 2) LAUNCH_TRY(launch_sizes_tail(g.fmt, d_descs(), d_list(w.chunk_work), n_slow, d_enc(), d_units(), stream));
    else LAUNCH_TRY(launch_sizes(g.fmt, 0, 0, d_descs(), d_list(w.chunk_work), n_slow, d_enc(), d_units(), stream));
    // the chained kernel has placed and written the tensors of its route (FP8: 1, BF16: 2) itself
    LAUNCH_TRY(launch_scan(d_descs(), T, (int)g.nf, g.reversed, chained ? (sh.bf16 ? 0x4 : 0x2) : 0, d_units(), (ScanOut *)(ws + w.scan), stats_only ? nullptr : ws + w.blobs,
                           (uint32_t)kBlobBytes, stream));
    return ZC_OK;
}

// chunked encode (a7)
zc_status CompressQueue::queue_encoders() const
{
    if (chained) {}                                             // encoded where they were sized
    else if (g.S == 64) LAUNCH_TRY(launch_encode_fp8(d_descs(), d_list(w.fast_work), n_fast, d_enc(), stream));
    else LAUNCH_TRY(launch_encode_fp8_sub(g.S, 1, sh.bf16, d_descs(), d_list(w.fast_work), n_fast, d_enc(), d_units(), sh.fast_step, stream));
    LAUNCH_TRY(launch_encode(g.fmt, sh.whole_mode, 0x6, d_descs(), d_list(w.whole_work), n_whole, d_enc(), stream));
    if (sh.rows8) LAUNCH_TRY(launch_encode_bf16(g.fmt, d_descs(), d_list(w.whole_work), n_whole, d_enc(), stream));
    LAUNCH_TRY(launch_encode(g.fmt, 0, 0x6, d_descs(), d_list(w.other_work), n_other, d_enc(), stream));
    LAUNCH_TRY(launch_encode(g.fmt, 0, 0, d_descs(), d_list(w.chunk_work), n_slow, d_enc(), stream));
    return ZC_OK;
}

// argument checks of one tensor of a compress-side call
zc_status check_compress_tensor(const Geometry &g, const zc_tensor &x, bool stats_only)
{
    if (x.n_elems && (!x.d_src || !aligned16(x.d_src))) return ZC_ERR_INVALID_ARG;
    if (x.d_xor_base && !aligned16(x.d_xor_base)) return ZC_ERR_INVALID_ARG;
    if (g.nf == 3 && x.n_elems && (!x.d_scales || !aligned16(x.d_scales))) return ZC_ERR_INVALID_ARG;
    if (!stats_only && (!x.d_comp || !aligned16(x.d_comp))) return ZC_ERR_INVALID_ARG;
    return ZC_OK;
}

// the compress-side descriptor of one tensor without what depends on its code; false: the destination cannot even
// hold the container's prologue
bool compress_desc(const Geometry &g, const zc_tensor &x, uint64_t nc, uint64_t units_off, bool stats_only, TensorDev *out)
{
    uint64_t table_off[3] = {0, 0, 0}, index_off[3] = {0, 0, 0}, payload_off;
    layout(g.fmt, nc, table_off, index_off, &payload_off);
    if (!stats_only && x.comp_capacity < payload_off) return false;
    TensorDev &d = *out;
    std::memset(&d, 0, sizeof(d));
    d.src = (const uint8_t *)x.d_src; d.base = (const uint8_t *)x.d_xor_base; d.scales = (const uint8_t *)x.d_scales;
    d.comp = stats_only ? nullptr : (uint8_t *)x.d_comp;
    d.n_elems = x.n_elems; d.n_chunks = (uint32_t)nc; d.chunk_bytes = g.chunk_bytes; d.streams = g.S;
    d.payload_off = payload_off;
    for (uint32_t f = 0; f < g.nf; f++) { d.table_off[f] = (uint32_t)table_off[f]; d.index_off[f] = (uint32_t)index_off[f]; }
    d.dst_bytes = stats_only ? 0 : x.comp_capacity;         // compress: bytes that may be written at comp
    d.units_off = (uint32_t)units_off;
    return true;
}

}  // namespace zc

using namespace zc;

namespace {

class CodeCrew {
public:
    CodeCrew(uint32_t n_items, uint32_t n_threads, const std::function<zc_status(uint32_t)> &fn)
        : n_(n_items), k_(n_threads < 1 ? 1 : n_threads), fn_(fn), status_(k_, ZC_OK)
    {
        for (uint32_t k = 1; k < k_; k++)
            pool_.emplace_back([this, k] {
                {
                    std::unique_lock<std::mutex> lock(m_);
                    cv_.wait(lock, [this] { return state_ != 0; });
                    if (state_ == 2) return;
                }
                range(k);
            });
    }
    ~CodeCrew() { open(2); for (auto &t : pool_) t.join(); }
    CodeCrew(const CodeCrew &) = delete;
    CodeCrew &operator=(const CodeCrew &) = delete;
    zc_status run()
    {
        open(1);
        range(0);
        for (auto &t : pool_) t.join();
        pool_.clear();
        for (uint32_t k = 0; k < k_; k++) if (status_[k]) return status_[k];
        return ZC_OK;
    }
private:
    void open(int state)
    {
        { std::lock_guard<std::mutex> lock(m_); if (state_ == 0) state_ = state; }
        cv_.notify_all();
    }
    void range(uint32_t k)
    {
        for (uint32_t t = (uint32_t)((uint64_t)n_ * k / k_); t < (uint32_t)((uint64_t)n_ * (k + 1) / k_); t++) {
            const zc_status s1 = fn_(t);
            if (s1) { status_[k] = s1; return; }
        }
    }
    uint32_t n_, k_;
    std::function<zc_status(uint32_t)> fn_;
    std::vector<zc_status> status_;
    std::vector<std::thread> pool_;
    std::mutex m_;
    std::condition_variable cv_;
    int state_ = 0;          // 0 = wait, 1 = go, 2 = leave
};

// ---- code construction from the device histograms ---------------------------
// hist3: the three 256-bin device histograms of one tensor (meaning depends on the format)
zc_status build_codes(const Geometry &g, uint32_t policy, uint64_t n_elems, const uint64_t *hist3, FieldCode fc[3], bool train = false)
{
    for (uint32_t f = 0; f < g.nf; f++) {
        FieldCode &c = fc[f];
        std::memset(&c, 0, sizeof(c));
        const int sb = sym_bits(g.fmt, (int)f), A = 1 << sb;
        // marginals of the joint byte histogram (FP8: one element per byte, FP4: two)
        // formats with 8-bit symbols in both fields are counted per field by the kernel
        if (g.fmt == ZC_FMT_BF16 || (group_of(g.fmt) > 1 && f < 2)) std::memcpy(c.hist, hist3 + 256 * f, 256 * 8);
        else if (g.fmt == ZC_FMT_FP8_E4M3) {
            for (int b = 0; b < 256; b++) {
                const int sym = f == 0 ? (b >> 3) & 0xF : ((b >> 4) & 8) | (b & 7);
                c.hist[sym] += hist3[b];
            }
        } else if (g.fmt == ZC_FMT_FP8_E5M2) {
            for (int b = 0; b < 256; b++) {
                const int sym = f == 0 ? (b >> 2) & 0x1F : ((b >> 5) & 4) | (b & 3);
                c.hist[sym] += hist3[b];
            }
        } else if (f == 2) std::memcpy(c.hist, hist3 + 512, 256 * 8);
        else {
            for (int b = 0; b < 256; b++)
                for (int h = 0; h < 2; h++) {
                    const int nib = (b >> (4 * h)) & 0xF;
                    const int sym = f == 0 ? (nib >> 1) & 3 : ((nib >> 2) & 2) | (nib & 1);
                    c.hist[sym] += hist3[b];
                }
        }
        c.n_symbols = field_symbols(g.fmt, (int)f, n_elems);
        uint64_t sum = 0;
        for (int v = 0; v < A; v++) { sum += c.hist[v]; if (c.hist[v]) { c.distinct++; c.konst = (uint32_t)v; } }
        if (sum != c.n_symbols) return ZC_ERR_DEVICE;          // the histogram kernel must count every symbol once
        if (train) {
            // static dictionary (Sec. 3.3, 5.2): every count raised by one, so that every symbol of the
            // alphabet can be coded when the dictionary is applied to other tensors
            uint64_t total = 0;
            for (int v = 0; v < A; v++) { c.hist[v] += 1; total += c.hist[v]; }
            if (!build_code_lengths(c.hist, A, g.limit[f], c.len)) return ZC_ERR_INVALID_ARG;
            for (int v = 0; v < A; v++) { c.payload_bits += c.hist[v] * c.len[v]; if (c.len[v] > c.lmax) c.lmax = c.len[v]; }
            c.mode = ZC_MODE_HUFF; c.konst = 0;
            if (policy == ZC_POLICY_AUTO && 16 * c.payload_bits > 15 * total * (uint64_t)sb) { c.mode = ZC_MODE_RAW; c.lmax = 0; std::memset(c.len, 0, sizeof(c.len)); }
            continue;
        }
        c.mode = ZC_MODE_EMPTY;
        if (c.distinct == 1) c.mode = ZC_MODE_CONST;
        else if (c.distinct > 1) {
            c.konst = 0;
            if (!build_code_lengths(c.hist, A, g.limit[f], c.len)) return ZC_ERR_INVALID_ARG;
            for (int v = 0; v < A; v++) { c.payload_bits += c.hist[v] * c.len[v]; if (c.len[v] > c.lmax) c.lmax = c.len[v]; }
            c.mode = ZC_MODE_HUFF;
            // Sec. 3.1: a field that does not compress is stored as is
            if (policy == ZC_POLICY_AUTO && 16 * c.payload_bits > 15 * c.n_symbols * (uint64_t)sb) {
                c.mode = ZC_MODE_RAW; c.lmax = 0; std::memset(c.len, 0, sizeof(c.len));
                c.payload_bits = c.n_symbols * (uint64_t)sb;
            } else assign_canonical(c.len, A, c.code);
        }
    }
    return ZC_OK;
}

// field codes taken from a precomputed dictionary instead of this tensor's histogram
zc_status codes_from_dictionary(const Geometry &g, uint64_t n_elems, const zc_info &dict, FieldCode fc[3])
{
    if (dict.format != g.fmt) return ZC_ERR_INVALID_ARG;
    for (uint32_t f = 0; f < g.nf; f++) {
        FieldCode &c = fc[f];
        std::memset(&c, 0, sizeof(c));
        const int sb = sym_bits(g.fmt, (int)f), A = 1 << sb;
        c.n_symbols = field_symbols(g.fmt, (int)f, n_elems);
        c.mode = ZC_MODE_EMPTY;
        if (c.n_symbols == 0) continue;
        if (dict.mode[f] == ZC_MODE_RAW) { c.mode = ZC_MODE_RAW; c.payload_bits = c.n_symbols * (uint64_t)sb; continue; }
        if (dict.mode[f] != ZC_MODE_HUFF) return ZC_ERR_INVALID_ARG;
        uint64_t kraft = 0;
        for (int v = 0; v < A; v++) {
            const uint32_t l = dict.code_len[f][v];
            if (l == 0 || l > 16) return ZC_ERR_INVALID_ARG;      // it must be able to code every symbol
            c.len[v] = (uint8_t)l;
            kraft += 1ull << (16 - l);
            if (l > c.lmax) c.lmax = l;
        }
        if (kraft != 65536) return ZC_ERR_INVALID_ARG;
        c.mode = ZC_MODE_HUFF;
        assign_canonical(c.len, A, c.code);
    }
    return ZC_OK;
}

uint32_t reverse_bits(uint32_t v, int n)
{
    uint32_t r = 0;
    for (int i = 0; i < n; i++) r |= ((v >> i) & 1u) << (n - 1 - i);
    return r;
}

// One compress-side call (compress, statistics, dictionary training), from the argument checks to the last
// kernel queued.  The members are what its steps share; run() is the sequence.
class CompressCall {
public:
    // dict: precomputed dictionary to code with (no histogram pass), or null.  train: stop after the code
    // construction with smoothed counts (codes_out receives the dictionary).  no_sync: queue everything, wait for
    // nothing, read nothing back.
    CompressCall(zc_tensor *tensors, uint32_t T, const zc_params *params, void *d_ws, uint64_t ws_bytes, void *stream,
                 bool stats_only, std::vector<FieldCode> *codes_out, std::vector<ScanOut> *scan_out,
                 const zc_info *dict, bool train, bool no_sync)
        : tensors(tensors), T(T), params(params), ws((uint8_t *)d_ws), ws_bytes(ws_bytes), stream(stream), hs((hipStream_t)stream),
          stats_only(stats_only), codes_out(codes_out), scan_out(scan_out), dict(dict), train(train), no_sync(no_sync) {}

    zc_status run()
    {
        zc_status st = check_params(params, &g);
        if (st) return st;
        if (T == 0) return ZC_OK;
        st = prepare();
        if (st) return st;
        if (uses_device_codes()) return run_with_device_codes();
        return run_with_host_codes();
    }

private:
    // ---- arguments
    zc_tensor *const tensors;
    const uint32_t T;
    const zc_params *const params;
    uint8_t *const ws;
    const uint64_t ws_bytes;
    void *const stream;
    const hipStream_t hs;
    const bool stats_only;
    std::vector<FieldCode> *const codes_out;
    std::vector<ScanOut> *const scan_out;
    const zc_info *const dict;
    const bool train, no_sync;
    // ---- what prepare() derives from them
    CompressQueue q;                        // geometry, workspace layout, list sizes, launches
    Geometry &g = q.g;
    Workspace &w = q.w;
    CompressShape &sh = q.sh;
    std::vector<TensorDev> descs;
    std::vector<uint64_t> ncs;              // chunks per tensor
    std::vector<uint8_t> fast_shapes;       // compress_fast_shape() per tensor
    bool roomy = false;                     // every destination can hold the worst case
    // the work lists as the host writes them (see TensorLists)
    std::vector<WorkItem> hist_work, scale_work, lane_hist_work, fast_work, whole_work, other_work, slow_work;

    bool uses_device_codes() const { return !dict && !stats_only && !train && !g.host_codes; }
    bool fast_shape(uint32_t t) const { return fast_shapes[t] != 0; }
    void set_list_sizes()
    {
        q.n_hist = (uint32_t)hist_work.size(); q.n_lane_hist = (uint32_t)lane_hist_work.size(); q.n_scale = (uint32_t)scale_work.size();
        q.n_fast = (uint32_t)fast_work.size(); q.n_whole = (uint32_t)whole_work.size(); q.n_other = (uint32_t)other_work.size();
        q.n_slow = (uint32_t)slow_work.size();
    }
    static void append(std::vector<WorkItem> &list, uint32_t t, const ListRange &r)
    {
        if (r.step) for (uint64_t c = r.first; c < r.end; c += r.step) list.push_back({t, (uint32_t)c});
    }

    // argument checks, workspace layout, descriptors, histogram work lists
    zc_status prepare()
    {
        if (!tensors || !ws || !aligned16(ws)) return ZC_ERR_INVALID_ARG;
        std::vector<uint64_t> counts(T);
        for (uint32_t t = 0; t < T; t++) {
            zc_tensor &x = tensors[t];
            counts[t] = x.n_elems;
            const zc_status bad = check_compress_tensor(g, x, stats_only);
            if (bad) return bad;
        }
        zc_status st = plan_workspace(g, counts.data(), T, &w);
        if (st) return st;
        if (ws_bytes < w.total) return ZC_ERR_BUFFER_TOO_SMALL;
        q.ws = ws; q.stream = stream; q.T = T; q.stats_only = stats_only;
        descs.resize(T);
        ncs.resize(T);
        fast_shapes.resize(T);
        uint64_t units_off = 0, all_chunks = 0;
        for (uint32_t t = 0; t < T; t++) { check_count(g, tensors[t].n_elems, &ncs[t]); all_chunks += ncs[t]; }
        sh = compress_shape(g, uses_device_codes(), all_chunks);
        for (uint32_t t = 0; t < T; t++) {
            zc_tensor &x = tensors[t];
            const uint64_t nc = ncs[t];
            fast_shapes[t] = compress_fast_shape(g, x.n_elems, zc_compress_bound(x.n_elems, params)) ? 1 : 0;
            if (!compress_desc(g, x, nc, units_off, stats_only, &descs[t])) return ZC_ERR_BUFFER_TOO_SMALL;
            units_off += nc * g.nf;
            const TensorLists L = device_code_lists(g, sh, x.n_elems, nc, fast_shape(t));
            append(lane_hist_work, t, L.lane_hist);
            append(hist_work, t, L.hist);
            append(scale_work, t, L.scale);
        }
        roomy = !stats_only;
        for (uint32_t t = 0; t < T && roomy; t++) roomy = tensors[t].comp_capacity >= zc_compress_bound(tensors[t].n_elems, params);
        if (no_sync && !roomy) return ZC_ERR_BUFFER_TOO_SMALL;
        return ZC_OK;
    }

    // The tail of every call that reads sizes back.  When every destination can hold the worst case, the sizes
    // need not be known on the host first: the encoder is queued right behind the scan and the sizes are read back
    // meanwhile.  Otherwise the host waits for the sizes and checks them before anything is written.  `landing`:
    // page-locked, first the ScanOut of every tensor, then extra_bytes copied from d_extra.
    zc_status encode_and_read_sizes(LandingLease &landing, const void *d_extra, uint64_t extra_bytes)
    {
        const uint64_t scan_bytes = (uint64_t)T * sizeof(ScanOut);
        HIP_TRY(hipMemcpyAsync(landing.ptr, ws + w.scan, scan_bytes, hipMemcpyDeviceToHost, hs));
        if (extra_bytes) HIP_TRY(hipMemcpyAsync(landing.ptr + scan_bytes, d_extra, extra_bytes, hipMemcpyDeviceToHost, hs));
        if (roomy) {
            // wait for the copies only, not for the encoder queued behind them
            hipEvent_t copied;
            HIP_TRY(hipEventCreateWithFlags(&copied, hipEventDisableTiming));
            const hipError_t e1 = hipEventRecord(copied, hs);
            const zc_status s1 = e1 == hipSuccess ? q.queue_encoders() : ZC_ERR_DEVICE;
            const hipError_t e2 = e1 == hipSuccess ? hipEventSynchronize(copied) : e1;
            (void)hipEventDestroy(copied);
            if (s1) return s1;
            if (e2 != hipSuccess) return ZC_ERR_DEVICE;
        } else HIP_TRY(hipStreamSynchronize(hs));
        const ScanOut *scan = reinterpret_cast<const ScanOut *>(landing.ptr);
        for (uint32_t t = 0; t < T; t++) {
            if (scan[t].total_units == 0xFFFFFFFFu) return ZC_ERR_DEVICE;      // a workgroup of the one-pass kernel gave up waiting in its chain
            const uint64_t total = descs[t].payload_off + 16ull * scan[t].total_units;
            tensors[t].out_bytes = total;
            if (!stats_only && total > tensors[t].comp_capacity) return ZC_ERR_BUFFER_TOO_SMALL;
        }
        if (scan_out) scan_out->assign(scan, scan + T);
        if (stats_only || roomy) return ZC_OK;
        return q.queue_encoders();
    }

    // A dictionary call over FP8 or BF16 pages, every tensor of so few whole pages that one workgroup sizes, places and encodes
    // them (the pages a decoding step appends to a K/V cache, Sec. 5.2): one kernel instead of size pass, scan and encoder.
    bool pages_fit_one_workgroup() const
    {
        if (!dict || stats_only || (g.fmt != ZC_FMT_FP8_E4M3 && g.fmt != ZC_FMT_BF16) || g.S < 4 || g.S > 32) return false;
        if (g.fmt == ZC_FMT_BF16 && sh.whole_shape) return false;       // route 2 then means the 64-lane encoder
        const uint32_t route = g.fmt == ZC_FMT_BF16 ? 2u : 1u;          // the page kernels' route of the format
        for (uint32_t t = 0; t < T; t++)
            if (descs[t].route != route || ncs[t] == 0 || ncs[t] > compress_pages_fused_limit() || tensors[t].n_elems % g.elems_per_chunk) return false;
        return true;
    }
    zc_status run_fused_pages()
    {
        uint32_t periods = 0;                                           // BF16: one build per refill period of the exponent field
        if (sh.bf16)
            for (uint32_t t = 0; t < T; t++) periods |= descs[t].period[0];
        LAUNCH_TRY(launch_compress_pages_fused(g.S, periods, g.reversed, q.d_descs(), T, q.d_enc(), ws + w.blobs, (uint32_t)kBlobBytes, (ScanOut *)(ws + w.scan), stream));
        if (no_sync) {
            for (uint32_t t = 0; t < T; t++) tensors[t].out_bytes = 0;
            return ZC_OK;
        }
        // the sizes are known when the kernel, encoder included, is through; a destination below the worst case only
        // loses what lies beyond it (the encoder's stores are range checked) and the call reports that it was too small
        LandingLease landing((uint64_t)T * sizeof(ScanOut));
        if (!landing.ptr) return ZC_ERR_DEVICE;
        HIP_TRY(hipMemcpyAsync(landing.ptr, ws + w.scan, (uint64_t)T * sizeof(ScanOut), hipMemcpyDeviceToHost, hs));
        HIP_TRY(hipStreamSynchronize(hs));
        const ScanOut *scan = reinterpret_cast<const ScanOut *>(landing.ptr);
        zc_status st = ZC_OK;
        for (uint32_t t = 0; t < T; t++) {
            tensors[t].out_bytes = descs[t].payload_off + 16ull * scan[t].total_units;
            tensors[t].info.total_bytes = tensors[t].out_bytes;
            if (tensors[t].out_bytes > tensors[t].comp_capacity) st = ZC_ERR_BUFFER_TOO_SMALL;
        }
        if (scan_out) scan_out->assign(scan, scan + T);
        return st;
    }

    // A dictionary call over FP8 or BF16 tensors of whole pages whose containers keep their fields in reverse order: the
    // sign+mantissa streams have their places by count alone and the exponent streams theirs from a running sum that the
    // workgroups hand on while they run, so one kernel reads the pages once (Sec. 5.2).  BF16: one refill period for all.
    bool pages_in_one_pass() const
    {
        if (!dict || stats_only || !g.reversed || (g.fmt != ZC_FMT_FP8_E4M3 && g.fmt != ZC_FMT_BF16) || g.S < 4 || g.S > 32) return false;
        const uint32_t route = g.fmt == ZC_FMT_BF16 ? 2u : 1u;
        for (uint32_t t = 0; t < T; t++) {
            if (descs[t].route != route || ncs[t] == 0 || tensors[t].n_elems % g.elems_per_chunk) return false;
            if (descs[t].period[0] != descs[0].period[0] || ncs[t] * (g.chunk_bytes / 32) >= 0x80000000ull) return false;
        }
        return true;
    }
    // Words of LDS per page if that kernel is to keep the exponent streams there until their places are known (the
    // source is then read once), or 0: the plain size of a page's exponent field (BF16, whose exponents usually code to
    // a third: half of that), when a workgroup has room for a pass of such pages.  A page whose stream does not fit after
    // all is coded a second time, so this is a matter of speed only.
    uint32_t chained_hold() const
    {
        const uint32_t words = g.chunk_bytes / (g.fmt == ZC_FMT_BF16 ? 16 : 8), per_pass = kWavesPerGroup * (64 / g.S);
        return (words % 4 == 0 && words >= 16 && words * per_pass <= compress_pages_held_words()) ? words : 0u;
    }
    // pages per work item of that kernel: whole passes of a workgroup.  As many as the LDS holds where the streams are
    // kept there; else few enough that the second read of them comes from the caches, enough to spread what an item
    // costs besides (C5 on MI355X, 8 lanes: 1.74 / 1.52 / 1.56 / 1.75 ms with 64 / 128 / 256 / 512 KiB per item; 16 lanes:
    // 2.33 / 1.76 / 1.56 / 1.58 ms with 32 / 64 / 128 / 256 KiB)
    uint32_t chained_step() const
    {
        const uint32_t per_pass = kWavesPerGroup * (64 / g.S);
        uint32_t passes = 131072 / (per_pass * g.chunk_bytes);     // about 128 KiB per item
        if (chained_hold()) passes = compress_pages_held_words() / (chained_hold() * per_pass);
        if (passes < 1) passes = 1;
        while (passes * per_pass > compress_pages_chained_limit()) passes--;
        return passes * per_pass;
    }
    zc_status run_pages_in_one_pass()
    {
        // the chain's words take the place of the stream sizes (one word of 8 bytes per work item: a tensor has at most
        // as many items as chunks, and two sizes of 4 bytes per chunk), its counter that of the first histogram
        uint64_t *status = reinterpret_cast<uint64_t *>(ws + w.units), *counter = reinterpret_cast<uint64_t *>(ws + w.hist);
        LAUNCH_TRY(launch_compress_pages_chained(g.S, sh.bf16 ? descs[0].period[0] : 0u, chained_hold(), q.d_descs(), q.d_list(w.fast_work), q.n_fast, chained_step(), q.d_enc(),
                                                 ws + w.blobs, (uint32_t)kBlobBytes, status, counter, (ScanOut *)(ws + w.scan), stream));
        if (no_sync) {
            for (uint32_t t = 0; t < T; t++) tensors[t].out_bytes = 0;
            return ZC_OK;
        }
        LandingLease landing((uint64_t)T * sizeof(ScanOut));
        if (!landing.ptr) return ZC_ERR_DEVICE;
        HIP_TRY(hipMemcpyAsync(landing.ptr, ws + w.scan, (uint64_t)T * sizeof(ScanOut), hipMemcpyDeviceToHost, hs));
        HIP_TRY(hipStreamSynchronize(hs));
        const ScanOut *scan = reinterpret_cast<const ScanOut *>(landing.ptr);
        zc_status st = ZC_OK;
        for (uint32_t t = 0; t < T; t++) {
            if (scan[t].total_units == 0xFFFFFFFFu) return ZC_ERR_DEVICE;      // a workgroup gave up waiting in the chain
            tensors[t].out_bytes = descs[t].payload_off + 16ull * scan[t].total_units;
            tensors[t].info.total_bytes = tensors[t].out_bytes;
            if (tensors[t].out_bytes > tensors[t].comp_capacity) st = ZC_ERR_BUFFER_TOO_SMALL;
        }
        if (scan_out) scan_out->assign(scan, scan + T);
        return st;
    }

    // a call that waits for nothing: the sizes stay in the containers' headers
    zc_status queue_encoders_without_sizes()
    {
        for (uint32_t t = 0; t < T; t++) tensors[t].out_bytes = 0;
        return q.queue_encoders();
    }

    // ---- the code is built on the device (a4): nothing between the histogram and the encoder waits for the host
    // Codes built on the device and FP8 or BF16 pages in a container with reversed payload order: the one-pass kernel takes
    // every tensor whose code turns out to suit it (decided on the device, BF16: whatever the refill period of its exponent
    // field; the others go through the generic kernels as before).  Its chain lives where the histograms were: they are dead once the codes are built.
    void choose_chained_device_path()
    {
        if (!g.reversed || (g.fmt != ZC_FMT_FP8_E4M3 && g.fmt != ZC_FMT_BF16) || g.S < 4 || g.S > 32 || stats_only) return;
        uint64_t items = 0;
        const uint32_t step = chained_step();
        for (uint32_t t = 0; t < T; t++) {
            if (!fast_shape(t) || ncs[t] == 0 || tensors[t].n_elems % g.elems_per_chunk || ncs[t] * (g.chunk_bytes / 32) >= 0x80000000ull) return;
            items += (ncs[t] + step - 1) / step;
        }
        if (items + 1 > (uint64_t)T * 3 * 256) return;
        q.chained = true; q.chain_hold = chained_hold(); q.chain_step = step; q.chain_counter = w.hist; q.chain_status = w.hist + 8;
    }

    zc_status run_with_device_codes()
    {
        choose_chained_device_path();
        std::vector<uint8_t> blobs((size_t)T * kBlobBytes, 0);
        const FieldCode no_code[3] = {};
        for (uint32_t t = 0; t < T; t++) {
            const bool fs = fast_shape(t);
            descs[t].fast_shape = (fs || sh.rows8) ? 1 : 0;
            const TensorLists L = device_code_lists(g, sh, tensors[t].n_elems, ncs[t], fs);
            append(fast_work, t, q.chained ? ListRange{0, (uint32_t)ncs[t], q.chain_step} : L.fast);
            append(whole_work, t, L.whole);
            append(other_work, t, L.other);
            append(slow_work, t, L.slow);
            // the header without what depends on the code; k_codes fills that in
            zc_info blank;
            fill_info(g, params->policy, tensors[t].d_xor_base != nullptr, tensors[t].n_elems, ncs[t], no_code, 0, &blank);
            serialize_blob(blank, &blobs[(size_t)t * kBlobBytes]);
        }
        if (!q.chained) order_for_xcds(fast_work);                 // the chain runs through the items in the list's order
        order_for_xcds(whole_work);
        order_for_xcds(other_work);
        order_for_xcds(slow_work);
        order_for_xcds(lane_hist_work);
        set_list_sizes();
        const Piece all[9] = {{w.descs, descs.data(), T * sizeof(TensorDev)},
                              {w.hist_work, hist_work.data(), hist_work.size() * sizeof(WorkItem)},
                              {w.hist_work + hist_work.size() * sizeof(WorkItem), lane_hist_work.data(), lane_hist_work.size() * sizeof(WorkItem)},
                              {w.scale_work, scale_work.data(), scale_work.size() * sizeof(WorkItem)},
                              {w.chunk_work, slow_work.data(), slow_work.size() * sizeof(WorkItem)},
                              {w.fast_work, fast_work.data(), fast_work.size() * sizeof(WorkItem)},
                              {w.whole_work, whole_work.data(), whole_work.size() * sizeof(WorkItem)},
                              {w.other_work, other_work.data(), other_work.size() * sizeof(WorkItem)},
                              {w.blobs, blobs.data(), blobs.size()}};
        zc_status st = stage_upload(ws, w.descs, w.enc, all, 9, stream);
        if (st) return st;
        st = q.queue_histogram();
        if (st) return st;
        st = q.queue_codes(params->policy);
        if (st) return st;
        st = q.queue_sizes_and_scan();
        if (st) return st;
        if (no_sync) return queue_encoders_without_sizes();
        LandingLease landing((uint64_t)T * (sizeof(ScanOut) + kBlobBytes));
        if (!landing.ptr) return ZC_ERR_DEVICE;
        st = encode_and_read_sizes(landing, ws + w.blobs, (uint64_t)T * kBlobBytes);
        // what the device decided, for the caller's zc_info
        const uint8_t *got = landing.ptr + (uint64_t)T * sizeof(ScanOut);
        for (uint32_t t = 0; t < T; t++) {
            const uint8_t *blob = got + (uint64_t)t * kBlobBytes;
            FieldCode fc[3] = {};
            for (uint32_t f = 0; f < g.nf; f++) {
                fc[f].mode = blob[32 + 4 * f]; fc[f].lmax = blob[34 + 4 * f]; fc[f].konst = blob[35 + 4 * f];
                std::memcpy(fc[f].len, blob + descs[t].table_off[f], (size_t)1 << sym_bits(g.fmt, (int)f));
            }
            fill_info(g, params->policy, tensors[t].d_xor_base != nullptr, tensors[t].n_elems, ncs[t], fc, tensors[t].out_bytes, &tensors[t].info);
        }
        return st;
    }

    // ---- the code is built on the host: a dictionary, statistics, training
    std::vector<FieldCode> codes;           // three per tensor
    std::vector<uint32_t> enc;              // 768 encode-table entries per tensor
    std::vector<uint8_t> blobs;             // header + code-length tables per tensor
    const uint64_t *hist = nullptr;         // the device histograms, landed

    // code construction on the host (a4), one tensor
    zc_status build_one(uint32_t t)
    {
        // A dictionary call gives every tensor the same code (Sec. 3.3, 5.2: K/V pages of a decoding step), so what
        // tensor 0 got is copied and only what depends on the element count is set again: for 64 tensors of a step
        // this is a third of the call's host time.  Tensors are built in order here (one thread with a dictionary).
        if (dict && t > 0 && !codes_out && tensors[t].n_elems && tensors[0].n_elems && fast_shape(t) == fast_shape(0)) {
            zc_info &info = tensors[t].info;
            info = tensors[0].info;
            info.xor_delta = tensors[t].d_xor_base != nullptr; info.n_elems = tensors[t].n_elems; info.n_chunks = (uint32_t)ncs[t];
            info.total_bytes = 0;
            layout(g.fmt, ncs[t], info.table_offset, info.index_offset, &info.payload_offset);
            uint8_t *blob = &blobs[(size_t)t * kBlobBytes];
            std::memcpy(blob, &blobs[0], kBlobBytes);
            blob[10] = (uint8_t)((info.xor_delta ? 1 : 0) | (g.reversed ? 2 : 0));
            put64(blob + 16, info.n_elems); put32(blob + 24, info.n_chunks); put64(blob + 48, 0); put64(blob + 56, info.payload_offset);
            std::memcpy(&enc[(size_t)t * 768], &enc[0], 768 * sizeof(uint32_t));
            TensorDev &d = descs[t];
            const TensorDev &d0 = descs[0];
            for (uint32_t f = 0; f < g.nf; f++) { d.mode[f] = d0.mode[f]; d.lmax[f] = d0.lmax[f]; d.konst[f] = d0.konst[f]; d.period[f] = d0.period[f]; d.kind[f] = d0.kind[f]; }
            d.route = d0.route;
            return ZC_OK;
        }
        FieldCode *fc = &codes[(size_t)t * 3];
        const zc_status s1 = dict ? codes_from_dictionary(g, tensors[t].n_elems, *dict, fc)
                                  : build_codes(g, params->policy, tensors[t].n_elems, &hist[(size_t)t * 768], fc, train);
        if (s1) return s1;
        fill_info(g, params->policy, tensors[t].d_xor_base != nullptr, tensors[t].n_elems, ncs[t], fc, 0, &tensors[t].info);
        serialize_blob(tensors[t].info, &blobs[(size_t)t * kBlobBytes]);
        TensorDev &d = descs[t];
        for (uint32_t f = 0; f < g.nf; f++) {
            d.mode[f] = (uint8_t)fc[f].mode; d.lmax[f] = (uint8_t)fc[f].lmax; d.konst[f] = (uint8_t)fc[f].konst;
            d.period[f] = (uint8_t)refill_period(run_len(g.fmt, (int)f), (int)fc[f].lmax);
            d.kind[f] = field_kind(fc[f].mode, (uint32_t)sym_bits(g.fmt, (int)f), fc[f].len);
            const int A = 1 << sym_bits(g.fmt, (int)f);
            for (int v = 0; v < A; v++)
                enc[(size_t)t * 768 + f * 256 + v] = ((uint32_t)fc[f].len[v] << 16) | reverse_bits(fc[f].code[v], fc[f].len[v]);
        }
        // FP8: the specialised kernels are written for an exponent refill period of 4 (longest code 5..8 bits) and a flat
        // or raw sign+mantissa field; their table (slot of the unused third field) maps a pair of exponents to the two
        // codes concatenated
        const bool plain_sm = d.kind[1] == 1 || d.kind[1] == 2;
        const bool fast_ok = !sh.bf16 && fast_shape(t) && fc[0].mode == ZC_MODE_HUFF && d.period[0] == 4 && plain_sm;
        if (fast_ok)
            for (uint32_t u = 0; u < 256; u++) {
                const uint32_t e0 = u & 15, e1 = u >> 4, l0 = fc[0].len[e0], l1 = fc[0].len[e1];
                enc[(size_t)t * 768 + 512 + u] = ((l0 + l1) << 16) | (enc[(size_t)t * 768 + e0] & 0xFFFFu) | ((enc[(size_t)t * 768 + e1] & 0xFFFFu) << l0);
            }
        // BF16 (and FP8 in byte symbols): the 64-lane encoder takes a table-coded exponent field next to a sign+mantissa field
        // that is flat, raw, or table coded with a refill period of 2 or 4; the BF16 page kernels want the latter flat or raw and, with two
        // exponents per refill step, no 1-bit code (the bound on their staging ring needs 4 bits per step)
        uint32_t lmin = 16;
        for (int v = 0; v < 256; v++) if (fc[0].len[v] && fc[0].len[v] < lmin) lmin = fc[0].len[v];
        // (FP8 E5M2, 16 symbols per run: both fields table coded, refill periods of at most 8)
        const bool e5m2_ok = g.fmt == ZC_FMT_FP8_E5M2 && d.kind[1] == 0 && d.period[0] <= 8 && d.period[1] >= 2 && d.period[1] <= 8;
        const bool bf16_ok = d.kind[0] == 0 &&
                             (sh.whole_shape ? (sh.rows8 && (g.fmt == ZC_FMT_FP8_E5M2 ? e5m2_ok : (plain_sm || (d.kind[1] == 0 && (d.period[1] == 2 || d.period[1] == 4)))))
                                          : (sh.bf16 && fast_shape(t) && plain_sm && (d.period[0] != 2 || lmin >= 2)));
        d.route = fast_ok ? 1 : bf16_ok ? 2 : 0;
        return ZC_OK;
    }

    zc_status run_with_host_codes()
    {
        // The histograms land in page-locked memory; what the code construction fills is allocated (and its pages
        // touched) while the histogram kernel runs.
        const uint64_t hist_bytes = dict ? 0 : (uint64_t)T * 768 * 8;
        LandingLease landing(hist_bytes);
        if (hist_bytes && !landing.ptr) return ZC_ERR_DEVICE;
        hist = reinterpret_cast<const uint64_t *>(landing.ptr);
        auto allocate_tables = [&]() {
            codes.resize((size_t)T * 3);
            enc.assign((size_t)T * 768, 0);
            blobs.assign((size_t)T * kBlobBytes, 0);
        };
        // The worker threads are started once the histogram kernel is queued and before the wait for it, so that
        // their start-up (tens of microseconds each) is hidden behind it; they sleep until run() opens the gate.
        // With a dictionary there is nothing to wait for and little to do per tensor: one thread.
        const uint32_t n_threads = (!dict && T >= 8) ? std::min<uint32_t>(std::min<uint32_t>(8, T / 2), std::max(1u, std::thread::hardware_concurrency())) : 1;
        std::optional<CodeCrew> crew;
        const auto one = [this](uint32_t t) { return build_one(t); };
        zc_status st;
        if (!dict) {
            const Piece first[3] = {{w.descs, descs.data(), T * sizeof(TensorDev)},
                                    {w.hist_work, hist_work.data(), hist_work.size() * sizeof(WorkItem)},
                                    {w.scale_work, scale_work.data(), scale_work.size() * sizeof(WorkItem)}};
            st = stage_upload(ws, w.descs, w.chunk_work, first, 3, stream);
            if (st) return st;
            set_list_sizes();
            st = q.queue_histogram();
            if (st) return st;
            HIP_TRY(hipMemcpyAsync(landing.ptr, q.d_hist(), hist_bytes, hipMemcpyDeviceToHost, hs));
            crew.emplace(T, n_threads, one);
            allocate_tables();
            HIP_TRY(hipStreamSynchronize(hs));
        } else {
            crew.emplace(T, n_threads, one);
            allocate_tables();
        }
        st = crew->run();
        if (st) return st;
        const bool chained = !pages_fit_one_workgroup() && pages_in_one_pass();
        for (uint32_t t = 0; t < T; t++) {
            // the route is known, so every chunk is listed once
            const uint64_t whole_chunks = tensors[t].n_elems / g.elems_per_chunk;
            const uint32_t n_fast = (descs[t].route == 1 || (descs[t].route == 2 && !sh.whole_shape)) ? (uint32_t)whole_chunks : 0;
            const uint32_t n_whole = (descs[t].route != 1 && sh.whole_shape) ? (uint32_t)whole_chunks : 0;
            append(fast_work, t, {0, n_fast, chained ? chained_step() : sh.fast_step});
            append(whole_work, t, {0, n_whole, sh.whole_step});
            append(slow_work, t, {n_fast + n_whole, (uint32_t)ncs[t], sh.cpi});
        }
        if (codes_out) *codes_out = codes;
        if (!chained) order_for_xcds(fast_work);                   // the chain runs through the items in the list's order
        order_for_xcds(whole_work);
        order_for_xcds(slow_work);
        set_list_sizes();
        // everything the kernels from here on read from the host, in one copy (the histogram work lists ride
        // along so that the copied range has no holes)
        const Piece all[8] = {{w.descs, descs.data(), T * sizeof(TensorDev)},
                              {w.whole_work, whole_work.data(), whole_work.size() * sizeof(WorkItem)},
                              {w.hist_work, hist_work.data(), hist_work.size() * sizeof(WorkItem)},
                              {w.scale_work, scale_work.data(), scale_work.size() * sizeof(WorkItem)},
                              {w.chunk_work, slow_work.data(), slow_work.size() * sizeof(WorkItem)},
                              {w.fast_work, fast_work.data(), fast_work.size() * sizeof(WorkItem)},
                              {w.blobs, stats_only ? nullptr : blobs.data(), stats_only ? 0 : blobs.size()},
                              {w.enc, enc.data(), enc.size() * 4}};
        st = stage_upload(ws, w.descs, w.host_end, all, 8, stream);
        if (st) return st;
        if (pages_fit_one_workgroup()) return run_fused_pages();
        if (chained) return run_pages_in_one_pass();
        st = q.queue_sizes_and_scan();
        if (st) return st;
        if (no_sync) return queue_encoders_without_sizes();
        LandingLease scan_landing((uint64_t)T * sizeof(ScanOut));
        if (!scan_landing.ptr) return ZC_ERR_DEVICE;
        st = encode_and_read_sizes(scan_landing, nullptr, 0);
        for (uint32_t t = 0; t < T; t++) tensors[t].info.total_bytes = tensors[t].out_bytes;
        return st;
    }
};

// shared by every compress-side entry point: histogram -> codes (-> sizes -> scan [-> encode])
zc_status run_compress(zc_tensor *tensors, uint32_t T, const zc_params *params, void *d_ws, uint64_t ws_bytes, void *stream,
                       bool stats_only, std::vector<FieldCode> *codes_out, std::vector<ScanOut> *scan_out,
                       const zc_info *dict = nullptr, bool train = false, bool no_sync = false)
{
    CompressCall call(tensors, T, params, d_ws, ws_bytes, stream, stats_only, codes_out, scan_out, dict, train, no_sync);
    return call.run();
}

}  // namespace

// ----------------------------------------------------------------------- C ABI

extern "C" {

uint64_t zc_workspace_bytes(const uint64_t *n_elems, uint32_t n_tensors, const zc_params *params)
{
    Geometry g;
    Workspace w;
    if (!n_elems || check_params(params, &g) || plan_workspace(g, n_elems, n_tensors, &w)) return 0;
    return w.total;
}

zc_status zc_compress_batch(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, void *d_ws, uint64_t ws_bytes, void *stream)
{
    return run_compress(tensors, n_tensors, params, d_ws, ws_bytes, stream, false, nullptr, nullptr);
}

zc_status zc_compress(const void *d_src, uint64_t n_elems, const zc_params *params, const void *d_xor_base, const void *d_scales,
                      void *d_dst, uint64_t dst_capacity, uint64_t *out_bytes, zc_info *out_info, void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!out_bytes) return ZC_ERR_INVALID_ARG;
    zc_tensor t;
    std::memset(&t, 0, sizeof(t));
    t.d_src = d_src; t.d_xor_base = d_xor_base; t.d_scales = d_scales; t.n_elems = n_elems;
    t.d_comp = d_dst; t.comp_capacity = dst_capacity;
    zc_status st = run_compress(&t, 1, params, d_ws, ws_bytes, stream, false, nullptr, nullptr);
    if (st) return st;
    *out_bytes = t.out_bytes;
    if (out_info) *out_info = t.info;
    return ZC_OK;
}

zc_status zc_train_code(const void *d_src, uint64_t n_elems, const zc_params *params, const void *d_xor_base, const void *d_scales,
                        zc_info *out_code, void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!out_code || n_elems == 0) return ZC_ERR_INVALID_ARG;
    zc_tensor t;
    std::memset(&t, 0, sizeof(t));
    t.d_src = d_src; t.d_xor_base = d_xor_base; t.d_scales = d_scales; t.n_elems = n_elems;
    std::vector<FieldCode> codes;
    zc_status st = run_compress(&t, 1, params, d_ws, ws_bytes, stream, true, &codes, nullptr, nullptr, true);
    if (st) return st;
    std::memset(out_code, 0, sizeof(*out_code));
    out_code->format = params->format; out_code->policy = params->policy;
    out_code->streams = params->streams_per_chunk ? params->streams_per_chunk : 64;
    out_code->n_fields = (uint32_t)num_fields(params->format); out_code->chunk_bytes = params->chunk_bytes;
    for (uint32_t f = 0; f < out_code->n_fields; f++) {
        out_code->mode[f] = (uint8_t)codes[f].mode; out_code->sym_bits[f] = (uint8_t)sym_bits(params->format, (int)f);
        out_code->max_len[f] = (uint8_t)codes[f].lmax;
        std::memcpy(out_code->code_len[f], codes[f].len, 256);
    }
    // what the training tensor itself costs under its dictionary: the reference point of zc_code_stale
    out_code->n_elems = n_elems; out_code->n_chunks = t.info.n_chunks;
    out_code->total_bytes = t.info.total_bytes; out_code->payload_offset = t.info.payload_offset;
    return ZC_OK;
}

zc_status zc_compress_batch_with_code(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, const zc_info *code,
                                      void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!code) return ZC_ERR_INVALID_ARG;
    return run_compress(tensors, n_tensors, params, d_ws, ws_bytes, stream, false, nullptr, nullptr, code, false);
}

zc_status zc_compress_batch_async(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, void *d_ws, uint64_t ws_bytes, void *stream)
{
    return run_compress(tensors, n_tensors, params, d_ws, ws_bytes, stream, false, nullptr, nullptr, nullptr, false, true);
}

zc_status zc_compress_batch_with_code_async(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, const zc_info *code,
                                            void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!code) return ZC_ERR_INVALID_ARG;
    return run_compress(tensors, n_tensors, params, d_ws, ws_bytes, stream, false, nullptr, nullptr, code, false, true);
}

zc_status zc_compress_with_code(const void *d_src, uint64_t n_elems, const zc_params *params, const zc_info *code,
                                const void *d_xor_base, const void *d_scales, void *d_dst, uint64_t dst_capacity,
                                uint64_t *out_bytes, zc_info *out_info, void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!out_bytes || !code) return ZC_ERR_INVALID_ARG;
    zc_tensor t;
    std::memset(&t, 0, sizeof(t));
    t.d_src = d_src; t.d_xor_base = d_xor_base; t.d_scales = d_scales; t.n_elems = n_elems;
    t.d_comp = d_dst; t.comp_capacity = dst_capacity;
    zc_status st = run_compress(&t, 1, params, d_ws, ws_bytes, stream, false, nullptr, nullptr, code, false);
    if (st) return st;
    *out_bytes = t.out_bytes;
    if (out_info) *out_info = t.info;
    return ZC_OK;
}

zc_status zc_stats(const void *d_src, uint64_t n_elems, const zc_params *params, const void *d_xor_base, const void *d_scales,
                   zc_stats_out *out, void *d_ws, uint64_t ws_bytes, void *stream)
{
    if (!out) return ZC_ERR_INVALID_ARG;
    zc_tensor t;
    std::memset(&t, 0, sizeof(t));
    t.d_src = d_src; t.d_xor_base = d_xor_base; t.d_scales = d_scales; t.n_elems = n_elems;
    std::vector<FieldCode> codes;
    std::vector<ScanOut> scan;
    zc_status st = run_compress(&t, 1, params, d_ws, ws_bytes, stream, true, &codes, &scan);
    if (st) return st;
    std::memset(out, 0, sizeof(*out));
    const uint32_t fmt = params->format;
    out->n_fields = (uint32_t)num_fields(fmt);
    out->raw_bytes = (n_elems * (uint64_t)elem_bits(fmt) + 7) / 8 + (out->n_fields == 3 ? n_elems / scale_block(fmt) : 0);
    out->container_bytes = t.out_bytes;
    uint64_t all_bits = 0;
    for (uint32_t f = 0; f < out->n_fields; f++) {
        const FieldCode &c = codes[f];
        zc_field_stats &fs = out->field[f];
        const int sb = sym_bits(fmt, (int)f);
        fs.alphabet = 1u << sb; fs.distinct = c.distinct; fs.mode = c.mode; fs.max_len = c.lmax; fs.n_symbols = c.n_symbols;
        std::memcpy(fs.hist, c.hist, sizeof(fs.hist));
        std::memcpy(fs.code_len, c.len, sizeof(fs.code_len));
        for (uint32_t v = 0; v < fs.alphabet; v++)
            if (c.hist[v]) { const double p = (double)c.hist[v] / (double)c.n_symbols; fs.entropy_bits -= p * std::log2(p); }
        fs.payload_bits = c.mode == ZC_MODE_CONST ? 0 : c.payload_bits;
        if (c.n_symbols) {
            fs.mean_code_len = (double)fs.payload_bits / (double)c.n_symbols;
            fs.ratio_payload = (double)fs.payload_bits / ((double)c.n_symbols * sb);
        }
        fs.stream_bytes = 16ull * scan[0].field_units[f];
        all_bits += fs.payload_bits;
    }
    if (out->raw_bytes) {
        out->ratio_payload_total = (double)all_bits / (8.0 * (double)out->raw_bytes);
        out->ratio_container_total = (double)out->container_bytes / (double)out->raw_bytes;
    }
    return ZC_OK;
}

}  // extern "C"
