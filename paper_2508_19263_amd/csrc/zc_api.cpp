// C ABI of the codec: argument checks, container layout, work lists, kernel launches, and the host-side code
// construction that dictionaries, statistics and ZC_HOST_CODES=1 use (a plain compress call builds its codes
// on the device).  See include/zc.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <algorithm>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <optional>
#include <thread>
#include <vector>

#include "zc_internal.h"

using namespace zc;

namespace {

struct Geometry {
    uint32_t fmt, S, nf;
    uint32_t chunk_bytes;
    uint64_t elems_per_chunk;
    int limit[kMaxFields];
};

zc_status check_params(const zc_params *p, Geometry *g)
{
    if (!p) return ZC_ERR_INVALID_ARG;
    if (p->struct_size != sizeof(zc_params)) return ZC_ERR_UNSUPPORTED;
    if (!elem_bits(p->format)) return ZC_ERR_UNSUPPORTED;
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

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// offsets of tables / indices / payload for a tensor of nc chunks
void layout(uint32_t fmt, uint64_t nc, uint64_t table_off[3], uint64_t index_off[3], uint64_t *payload_off)
{
    uint64_t off = kHeaderBytes;
    const int nf = num_fields(fmt);
    for (int f = 0; f < nf; f++) { table_off[f] = off; off += pad16(1ull << sym_bits(fmt, f)); }
    for (int f = 0; f < nf; f++) { index_off[f] = off; off += pad16(4 * (nc + 1)); }
    *payload_off = off;
}

void put32(uint8_t *p, uint32_t v) { std::memcpy(p, &v, 4); }
void put64(uint8_t *p, uint64_t v) { std::memcpy(p, &v, 8); }
uint32_t get32(const uint8_t *p) { uint32_t v; std::memcpy(&v, p, 4); return v; }
uint64_t get64(const uint8_t *p) { uint64_t v; std::memcpy(&v, p, 8); return v; }

// ---- workspace carving ------------------------------------------------------
struct Workspace {
    uint64_t descs, hist_work, scale_work, chunk_work, fast_work, whole_work, other_work, hist, enc, units, scan, blobs, lane_counts, total, host_end;
    uint32_t n_hist_work, n_scale_work, n_chunk_work;
    uint64_t n_units;
};

uint64_t align256(uint64_t x) { return (x + 255) / 256 * 256; }
constexpr uint64_t kBlobBytes = 1024;     // header + code-length tables of one tensor (<= 64 + 3*256)

// The geometry for which the histogram pass also counts exponents per chunk lane, so that the size pass need
// not read the source again (k_hist_fp8_lanes, k_sizes_fp8_counts)
bool lane_counts_shape(const Geometry &g) { return g.fmt == ZC_FMT_FP8_E4M3 && g.S == 64 && g.chunk_bytes == kHistBlockBytes; }

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
    w->total = off;
    w->n_hist_work = (uint32_t)hw; w->n_scale_work = (uint32_t)sw; w->n_chunk_work = (uint32_t)cw; w->n_units = units;
    return ZC_OK;
}

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return ZC_ERR_DEVICE; } while (0)
#define LAUNCH_TRY(expr) do { if ((expr) != 0) return ZC_ERR_DEVICE; } while (0)

// ---- pinned staging for what the host sends to the workspace ------------------
// A few page-locked buffers per process, used in turn: the pieces of an upload are packed into one at their
// workspace offsets and leave in a single asynchronous copy that needs no wait (the buffer outlives the call).
// A buffer's next user waits for the event of the copy that last left it, so calls queued back to back block
// only when more than kSlots uploads are still ahead of the device.
struct Piece { uint64_t off; const void *src; uint64_t bytes; };

class HostStage {
public:
    // copies pieces (all inside [lo, hi) of the workspace) to d_ws + lo .. d_ws + hi on `hs`
    zc_status upload(uint8_t *d_ws, uint64_t lo, uint64_t hi, const Piece *pieces, int n, hipStream_t hs)
    {
        if (hi <= lo) return ZC_OK;
        std::lock_guard<std::mutex> lock(m_);
        Slot &k = slot_[next_];
        next_ = (next_ + 1) % kSlots;
        if (k.pending && hipEventSynchronize(k.ev) != hipSuccess) return ZC_ERR_DEVICE;
        k.pending = false;
        const uint64_t need = hi - lo;
        if (need > k.cap) {
            // the first call sizes every slot that is still empty, so that the calls after it find theirs ready
            const uint64_t want = need + need / 2 + 4096;
            for (Slot &q : slot_) {
                if (&q != &k && q.buf) continue;
                if (q.buf) (void)hipHostFree(q.buf);
                q.buf = nullptr; q.cap = 0;
                if (hipHostMalloc((void **)&q.buf, want, hipHostMallocDefault) != hipSuccess) return ZC_ERR_DEVICE;
                q.cap = want;
            }
        }
        if (!k.ev && hipEventCreateWithFlags(&k.ev, hipEventDisableTiming) != hipSuccess) return ZC_ERR_DEVICE;
        for (int i = 0; i < n; i++)
            if (pieces[i].bytes) std::memcpy(k.buf + (pieces[i].off - lo), pieces[i].src, pieces[i].bytes);
        HIP_TRY(hipMemcpyAsync(d_ws + lo, k.buf, need, hipMemcpyHostToDevice, hs));
        HIP_TRY(hipEventRecord(k.ev, hs));
        k.pending = true;
        return ZC_OK;
    }
private:
    static constexpr int kSlots = 4;
    struct Slot { uint8_t *buf = nullptr; uint64_t cap = 0; hipEvent_t ev = nullptr; bool pending = false; };
    std::mutex m_;
    Slot slot_[kSlots];
    int next_ = 0;
};

HostStage &host_stage() { static HostStage s; return s; }

// ---- pinned landing buffers for what the host reads back -------------------------
// A copy into pageable memory is staged by the runtime in pieces; into page-locked memory it is one
// transfer.  Buffers are handed out one per call in flight and kept for the life of the process.
class HostLanding {
public:
    uint8_t *acquire(uint64_t bytes, uint64_t *cap)
    {
        std::lock_guard<std::mutex> lock(m_);
        for (size_t i = 0; i < free_.size(); i++)
            if (free_[i].second >= bytes) {
                uint8_t *b = free_[i].first; *cap = free_[i].second;
                free_.erase(free_.begin() + (long)i);
                return b;
            }
        if (!free_.empty()) { (void)hipHostFree(free_.back().first); free_.pop_back(); }     // too small: replace it
        uint8_t *b = nullptr;
        const uint64_t want = bytes + bytes / 2 + 4096;
        if (hipHostMalloc((void **)&b, want, hipHostMallocDefault) != hipSuccess) return nullptr;
        *cap = want;
        return b;
    }
    void release(uint8_t *b, uint64_t cap)
    {
        std::lock_guard<std::mutex> lock(m_);
        free_.push_back({b, cap});
    }
private:
    std::mutex m_;
    std::vector<std::pair<uint8_t *, uint64_t>> free_;
};

HostLanding &host_landing() { static HostLanding s; return s; }

struct LandingLease {
    uint8_t *ptr = nullptr;
    uint64_t cap = 0;
    explicit LandingLease(uint64_t bytes) { if (bytes) ptr = host_landing().acquire(bytes, &cap); }
    ~LandingLease() { if (ptr) host_landing().release(ptr, cap); }
    LandingLease(const LandingLease &) = delete;
    LandingLease &operator=(const LandingLease &) = delete;
};

// ---- a few threads for the per-tensor code construction ------------------------
// Tensors are independent, so a large set is split into contiguous ranges, one per thread; the calling
// thread takes the first range.  The destructor joins whatever was started, so an early return between
// construction and run() is safe (the workers then leave without doing anything).
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
struct FieldCode {
    uint64_t hist[256];
    uint8_t len[256];
    uint16_t code[256];
    uint32_t mode, lmax, konst, distinct;
    uint64_t n_symbols, payload_bits;
};

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

void fill_info(const Geometry &g, uint32_t policy, bool xor_delta, uint64_t n_elems, uint64_t nc, const FieldCode fc[3], uint64_t total, zc_info *info)
{
    std::memset(info, 0, sizeof(*info));
    info->format = g.fmt; info->policy = policy; info->streams = g.S; info->n_fields = g.nf;
    info->xor_delta = xor_delta; info->chunk_bytes = g.chunk_bytes; info->n_chunks = (uint32_t)nc;
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
    blob[8] = (uint8_t)info.streams; blob[9] = (uint8_t)info.n_fields; blob[10] = (uint8_t)(info.xor_delta ? 1 : 0);
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

uint32_t sub_slots_per_group(uint32_t streams, uint64_t slots);
void order_for_xcds(std::vector<WorkItem> &items);

// The code of a compress call is built on the device unless the environment says ZC_HOST_CODES=1 (read once):
// the host construction gives the same bits and is what dictionaries, statistics and training use anyway.
bool device_codes_enabled()
{
    static const bool on = [] { const char *e = std::getenv("ZC_HOST_CODES"); return !(e && e[0] == '1'); }();
    return on;
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
    Geometry g;
    Workspace w;
    uint32_t cpi = 0;                       // chunks per work item of the generic kernels
    std::vector<TensorDev> descs;
    std::vector<uint64_t> ncs;              // chunks per tensor
    std::vector<WorkItem> hist_work, scale_work;
    std::vector<WorkItem> lane_hist_work;   // whole chunks whose histogram pass also counts per lane (lanes)
    bool lanes = false;                     // the code is built on the device and the geometry is lane_counts_shape()
    bool bf16 = false;
    bool whole_shape = false;               // 64 lanes, chunks of whole 1 KiB rows: the generic encoder's whole-chunk build
    int whole_mode = 1;                     // 2: one whole chunk per work item, shared by its four wavefronts
    uint32_t whole_step = 0, fast_step = 0; // chunks per work item of the whole-chunk list and of the fast list
    bool roomy = false;                     // every destination can hold the worst case
    // Work lists of the size pass and the encoder.  fast: whole chunks for the FP8 kernels and the page kernels'
    // BF16 builds; whole: whole chunks for the generic encoder's 64-lane build (and the BF16 encoder); other: whole
    // chunks for the generic encoder where neither applies to the geometry but a specialised kernel might have taken
    // them (device-built codes only: the route is not known when the lists are written); slow: everything else (a
    // short last chunk, odd geometries).
    std::vector<WorkItem> fast_work, whole_work, other_work, slow_work;

    TensorDev *d_descs() const { return (TensorDev *)(ws + w.descs); }
    uint64_t *d_hist() const { return (uint64_t *)(ws + w.hist); }
    uint32_t *d_enc() const { return (uint32_t *)(ws + w.enc); }
    uint32_t *d_units() const { return (uint32_t *)(ws + w.units); }
    uint16_t *d_lane_counts() const { return (uint16_t *)(ws + w.lane_counts); }
    bool uses_device_codes() const { return !dict && !stats_only && !train && device_codes_enabled(); }
    const WorkItem *d_list(uint64_t off) const { return (const WorkItem *)(ws + off); }

    // Geometry the specialised FP8 size/encode kernels take: 64 lanes and chunks of whole 1 KiB rows, or 4..32
    // lanes per chunk (pages) for the sub-wavefront kernels as long as the tensor fits their 32-bit offsets.
    // The page kernels also have BF16 builds.  Whether the code suits them too is known once the code is:
    // descs[t].route.
    bool fast_shape(uint32_t t) const
    {
        if (g.fmt == ZC_FMT_BF16) return g.S >= 4 && g.S < 64 && g.chunk_bytes % (16 * g.S) == 0 && tensors[t].n_elems * 2 <= 0xF0000000ull;
        if (g.fmt != ZC_FMT_FP8_E4M3) return false;
        return g.S == 64 ? g.chunk_bytes % 1024 == 0
                         : (g.S >= 4 && g.chunk_bytes % (16 * g.S) == 0 && tensors[t].n_elems <= 0xF0000000ull);
    }

    // argument checks, workspace layout, descriptors, histogram work lists
    zc_status prepare()
    {
        if (!tensors || !ws || !aligned16(ws)) return ZC_ERR_INVALID_ARG;
        std::vector<uint64_t> counts(T);
        for (uint32_t t = 0; t < T; t++) {
            zc_tensor &x = tensors[t];
            counts[t] = x.n_elems;
            if (x.n_elems && (!x.d_src || !aligned16(x.d_src))) return ZC_ERR_INVALID_ARG;
            if (x.d_xor_base && !aligned16(x.d_xor_base)) return ZC_ERR_INVALID_ARG;
            if (g.nf == 3 && x.n_elems && (!x.d_scales || !aligned16(x.d_scales))) return ZC_ERR_INVALID_ARG;
            if (!stats_only && (!x.d_comp || !aligned16(x.d_comp))) return ZC_ERR_INVALID_ARG;
        }
        zc_status st = plan_workspace(g, counts.data(), T, &w);
        if (st) return st;
        if (ws_bytes < w.total) return ZC_ERR_BUFFER_TOO_SMALL;
        cpi = chunks_per_work_item(g.S);
        lanes = uses_device_codes() && lane_counts_shape(g);
        descs.resize(T);
        ncs.resize(T);
        uint64_t units_off = 0, all_chunks = 0;
        for (uint32_t t = 0; t < T; t++) {
            zc_tensor &x = tensors[t];
            uint64_t nc;
            check_count(g, x.n_elems, &nc);
            ncs[t] = nc;
            all_chunks += nc;
            uint64_t table_off[3] = {0, 0, 0}, index_off[3] = {0, 0, 0}, payload_off;
            layout(g.fmt, nc, table_off, index_off, &payload_off);
            if (!stats_only && x.comp_capacity < payload_off) return ZC_ERR_BUFFER_TOO_SMALL;
            TensorDev &d = descs[t];
            std::memset(&d, 0, sizeof(d));
            d.src = (const uint8_t *)x.d_src; d.base = (const uint8_t *)x.d_xor_base; d.scales = (const uint8_t *)x.d_scales;
            d.comp = stats_only ? nullptr : (uint8_t *)x.d_comp;
            d.n_elems = x.n_elems; d.n_chunks = (uint32_t)nc; d.chunk_bytes = g.chunk_bytes; d.streams = g.S;
            d.payload_off = payload_off;
            for (uint32_t f = 0; f < g.nf; f++) { d.table_off[f] = (uint32_t)table_off[f]; d.index_off[f] = (uint32_t)index_off[f]; }
            d.dst_bytes = stats_only ? 0 : x.comp_capacity;         // compress: bytes that may be written at comp
            d.units_off = (uint32_t)units_off;
            units_off += nc * g.nf;
            const uint64_t bytes = (x.n_elems * (uint64_t)elem_bits(g.fmt) + 7) / 8;
            // a histogram block is a chunk here when lanes is set: whole chunks go to the kernel that counts per lane too
            const uint64_t lane_blocks = lanes ? x.n_elems / g.elems_per_chunk : 0;
            for (uint64_t b = 0; b < lane_blocks; b++) lane_hist_work.push_back({t, (uint32_t)b});
            for (uint64_t b = lane_blocks; b * kHistBlockBytes < bytes; b++) hist_work.push_back({t, (uint32_t)b});
            if (g.nf == 3) for (uint64_t b = 0; b * kHistBlockBytes < x.n_elems / scale_block(g.fmt); b++) scale_work.push_back({t, (uint32_t)b});
        }
        bf16 = g.fmt == ZC_FMT_BF16;
        whole_shape = g.S == 64 && g.chunk_bytes % 1024 == 0;
        // FP4 elements rarely compress, so their fields are stored plainly and a chunk's rows can be shared by the four
        // wavefronts of a workgroup: one chunk per work item there
        whole_mode = is_fp4(g.fmt) ? 2 : 1;
        whole_step = whole_mode == 2 ? 1u : kWavesPerGroup;
        fast_step = g.S == 64 ? kWavesPerGroup : sub_slots_per_group(g.S, all_chunks);
        roomy = !stats_only;
        for (uint32_t t = 0; t < T && roomy; t++) roomy = tensors[t].comp_capacity >= zc_compress_bound(tensors[t].n_elems, params);
        if (no_sync && !roomy) return ZC_ERR_BUFFER_TOO_SMALL;
        return ZC_OK;
    }

    // field split + histogram (a1-a3)
    zc_status queue_histogram()
    {
        LAUNCH_TRY(launch_zero(d_hist(), (uint64_t)T * 3 * 256, stream));
        LAUNCH_TRY(launch_hist(g.fmt, d_descs(), d_list(w.hist_work), (uint32_t)hist_work.size(), 0, d_hist(), stream));
        LAUNCH_TRY(launch_hist_fp8_lanes(d_descs(), d_list(w.hist_work) + hist_work.size(), (uint32_t)lane_hist_work.size(), d_hist(), d_lane_counts(), stream));
        if (g.nf == 3) LAUNCH_TRY(launch_hist(g.fmt, d_descs(), d_list(w.scale_work), (uint32_t)scale_work.size(), (int)scale_block(g.fmt), d_hist(), stream));
        return ZC_OK;
    }

    // stream sizes (a5) and their exclusive scan into the chunk index (a6)
    zc_status queue_sizes_and_scan()
    {
        if (g.S == 64 && lanes) LAUNCH_TRY(launch_sizes_fp8_counts(d_descs(), d_list(w.fast_work), (uint32_t)fast_work.size(), d_enc(), d_lane_counts(), d_units(), stream));
        else if (g.S == 64) LAUNCH_TRY(launch_sizes_fp8(d_descs(), d_list(w.fast_work), (uint32_t)fast_work.size(), d_enc(), d_units(), stream));
        else LAUNCH_TRY(launch_encode_fp8_sub(g.S, 0, bf16, d_descs(), d_list(w.fast_work), (uint32_t)fast_work.size(), d_enc(), d_units(), fast_step, stream));
        // generic kernels: the whole-chunk list leaves route 1 to the FP8 kernels (route 2 there is the BF16 encoder,
        // whose sizes come from this pass); the list of page-shaped tensors leaves both routes to the page kernels
        LAUNCH_TRY(launch_sizes(g.fmt, whole_mode, 0x2, d_descs(), d_list(w.whole_work), (uint32_t)whole_work.size(), d_enc(), d_units(), stream));
        LAUNCH_TRY(launch_sizes(g.fmt, 0, 0x6, d_descs(), d_list(w.other_work), (uint32_t)other_work.size(), d_enc(), d_units(), stream));
        LAUNCH_TRY(launch_sizes(g.fmt, 0, 0, d_descs(), d_list(w.chunk_work), (uint32_t)slow_work.size(), d_enc(), d_units(), stream));
        LAUNCH_TRY(launch_scan(d_descs(), T, (int)g.nf, d_units(), (ScanOut *)(ws + w.scan), stats_only ? nullptr : ws + w.blobs, (uint32_t)kBlobBytes, stream));
        return ZC_OK;
    }

    // chunked encode (a7)
    zc_status queue_encoders()
    {
        if (g.S == 64) LAUNCH_TRY(launch_encode_fp8(d_descs(), d_list(w.fast_work), (uint32_t)fast_work.size(), d_enc(), stream));
        else LAUNCH_TRY(launch_encode_fp8_sub(g.S, 1, bf16, d_descs(), d_list(w.fast_work), (uint32_t)fast_work.size(), d_enc(), d_units(), fast_step, stream));
        LAUNCH_TRY(launch_encode(g.fmt, whole_mode, 0x6, d_descs(), d_list(w.whole_work), (uint32_t)whole_work.size(), d_enc(), stream));
        if (bf16) LAUNCH_TRY(launch_encode_bf16(d_descs(), d_list(w.whole_work), (uint32_t)whole_work.size(), d_enc(), stream));
        LAUNCH_TRY(launch_encode(g.fmt, 0, 0x6, d_descs(), d_list(w.other_work), (uint32_t)other_work.size(), d_enc(), stream));
        LAUNCH_TRY(launch_encode(g.fmt, 0, 0, d_descs(), d_list(w.chunk_work), (uint32_t)slow_work.size(), d_enc(), stream));
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
            const zc_status s1 = e1 == hipSuccess ? queue_encoders() : ZC_ERR_DEVICE;
            const hipError_t e2 = e1 == hipSuccess ? hipEventSynchronize(copied) : e1;
            (void)hipEventDestroy(copied);
            if (s1) return s1;
            if (e2 != hipSuccess) return ZC_ERR_DEVICE;
        } else HIP_TRY(hipStreamSynchronize(hs));
        const ScanOut *scan = reinterpret_cast<const ScanOut *>(landing.ptr);
        for (uint32_t t = 0; t < T; t++) {
            const uint64_t total = descs[t].payload_off + 16ull * scan[t].total_units;
            tensors[t].out_bytes = total;
            if (!stats_only && total > tensors[t].comp_capacity) return ZC_ERR_BUFFER_TOO_SMALL;
        }
        if (scan_out) scan_out->assign(scan, scan + T);
        if (stats_only || roomy) return ZC_OK;
        return queue_encoders();
    }

    // a call that waits for nothing: the sizes stay in the containers' headers
    zc_status queue_encoders_without_sizes()
    {
        for (uint32_t t = 0; t < T; t++) tensors[t].out_bytes = 0;
        return queue_encoders();
    }

    // ---- the code is built on the device (a4): nothing between the histogram and the encoder waits for the host
    zc_status run_with_device_codes()
    {
        std::vector<uint8_t> blobs((size_t)T * kBlobBytes, 0);
        const FieldCode no_code[3] = {};
        for (uint32_t t = 0; t < T; t++) {
            // the route is not known yet: whole chunks are listed for every kernel that may take them
            const uint64_t whole_chunks = tensors[t].n_elems / g.elems_per_chunk;
            const bool fs = fast_shape(t);
            descs[t].fast_shape = (fs || (bf16 && whole_shape)) ? 1 : 0;
            if (fs) for (uint64_t c = 0; c < whole_chunks; c += fast_step) fast_work.push_back({t, (uint32_t)c});
            if (whole_shape) for (uint64_t c = 0; c < whole_chunks; c += whole_step) whole_work.push_back({t, (uint32_t)c});
            else if (fs) for (uint64_t c = 0; c < whole_chunks; c += cpi) other_work.push_back({t, (uint32_t)c});
            for (uint64_t c = (fs || whole_shape) ? whole_chunks : 0; c < ncs[t]; c += cpi) slow_work.push_back({t, (uint32_t)c});
            // the header without what depends on the code; k_codes fills that in
            zc_info blank;
            fill_info(g, params->policy, tensors[t].d_xor_base != nullptr, tensors[t].n_elems, ncs[t], no_code, 0, &blank);
            serialize_blob(blank, &blobs[(size_t)t * kBlobBytes]);
        }
        order_for_xcds(fast_work);
        order_for_xcds(whole_work);
        order_for_xcds(other_work);
        order_for_xcds(slow_work);
        order_for_xcds(lane_hist_work);
        const Piece all[9] = {{w.descs, descs.data(), T * sizeof(TensorDev)},
                              {w.hist_work, hist_work.data(), hist_work.size() * sizeof(WorkItem)},
                              {w.hist_work + hist_work.size() * sizeof(WorkItem), lane_hist_work.data(), lane_hist_work.size() * sizeof(WorkItem)},
                              {w.scale_work, scale_work.data(), scale_work.size() * sizeof(WorkItem)},
                              {w.chunk_work, slow_work.data(), slow_work.size() * sizeof(WorkItem)},
                              {w.fast_work, fast_work.data(), fast_work.size() * sizeof(WorkItem)},
                              {w.whole_work, whole_work.data(), whole_work.size() * sizeof(WorkItem)},
                              {w.other_work, other_work.data(), other_work.size() * sizeof(WorkItem)},
                              {w.blobs, blobs.data(), blobs.size()}};
        zc_status st = host_stage().upload(ws, w.descs, w.enc, all, 9, hs);
        if (st) return st;
        st = queue_histogram();
        if (st) return st;
        CodeParams cp;
        cp.fmt = g.fmt; cp.policy = params->policy; cp.nf = g.nf; cp.blob_bytes = (uint32_t)kBlobBytes; cp.run_len = (uint32_t)run_len(g.fmt, 0);
        for (int f = 0; f < kMaxFields; f++) cp.limit[f] = f < (int)g.nf ? g.limit[f] : 0;
        LAUNCH_TRY(launch_codes(d_descs(), T, d_hist(), cp, ws + w.blobs, d_enc(), stream));
        st = queue_sizes_and_scan();
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
            blob[10] = (uint8_t)(info.xor_delta ? 1 : 0);
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
        const bool fast_ok = !bf16 && fast_shape(t) && fc[0].mode == ZC_MODE_HUFF && d.period[0] == 4 && plain_sm;
        if (fast_ok)
            for (uint32_t u = 0; u < 256; u++) {
                const uint32_t e0 = u & 15, e1 = u >> 4, l0 = fc[0].len[e0], l1 = fc[0].len[e1];
                enc[(size_t)t * 768 + 512 + u] = ((l0 + l1) << 16) | (enc[(size_t)t * 768 + e0] & 0xFFFFu) | ((enc[(size_t)t * 768 + e1] & 0xFFFFu) << l0);
            }
        // BF16: the 64-lane encoder takes a table-coded exponent field next to a sign+mantissa field that is flat, raw, or
        // table coded with a refill period of 2 or 4; the page kernels want the latter flat or raw and, with two
        // exponents per refill step, no 1-bit code (the bound on their staging ring needs 4 bits per step)
        uint32_t lmin = 16;
        for (int v = 0; v < 256; v++) if (fc[0].len[v] && fc[0].len[v] < lmin) lmin = fc[0].len[v];
        const bool bf16_ok = bf16 && d.kind[0] == 0 &&
                             (whole_shape ? (plain_sm || (d.kind[1] == 0 && (d.period[1] == 2 || d.period[1] == 4)))
                                          : (fast_shape(t) && plain_sm && (d.period[0] != 2 || lmin >= 2)));
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
            st = host_stage().upload(ws, w.descs, w.chunk_work, first, 3, hs);
            if (st) return st;
            st = queue_histogram();
            if (st) return st;
            HIP_TRY(hipMemcpyAsync(landing.ptr, d_hist(), hist_bytes, hipMemcpyDeviceToHost, hs));
            crew.emplace(T, n_threads, one);
            allocate_tables();
            HIP_TRY(hipStreamSynchronize(hs));
        } else {
            crew.emplace(T, n_threads, one);
            allocate_tables();
        }
        st = crew->run();
        if (st) return st;
        for (uint32_t t = 0; t < T; t++) {
            // the route is known, so every chunk is listed once
            const uint64_t whole_chunks = tensors[t].n_elems / g.elems_per_chunk;
            const uint64_t n_fast = (descs[t].route == 1 || (descs[t].route == 2 && !whole_shape)) ? whole_chunks : 0;
            const uint64_t n_whole = (descs[t].route != 1 && whole_shape) ? whole_chunks : 0;
            for (uint64_t c = 0; c < n_fast; c += fast_step) fast_work.push_back({t, (uint32_t)c});
            for (uint64_t c = 0; c < n_whole; c += whole_step) whole_work.push_back({t, (uint32_t)c});
            for (uint64_t c = n_fast + n_whole; c < ncs[t]; c += cpi) slow_work.push_back({t, (uint32_t)c});
        }
        if (codes_out) *codes_out = codes;
        order_for_xcds(fast_work);
        order_for_xcds(whole_work);
        order_for_xcds(slow_work);
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
        st = host_stage().upload(ws, w.descs, w.host_end, all, 8, hs);
        if (st) return st;
        st = queue_sizes_and_scan();
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
    constexpr size_t kXcds = 8;
    const size_t n = items.size(), q = n / kXcds, r = n % kXcds;
    if (n < 2 * kXcds) return;
    std::vector<WorkItem> out(n);
    for (size_t p = 0; p < n; p++) {
        const size_t k = p % kXcds, start = k * q + (k < r ? k : r);
        out[p] = items[start + p / kXcds];
    }
    items.swap(out);
}

zc_status parse_info(const uint8_t *c, uint64_t have, uint64_t comp_bytes, zc_info *out)
{
    if (have < kHeaderBytes || comp_bytes < kHeaderBytes) return ZC_ERR_CORRUPT;
    if (get32(c) != kMagic || c[4] != 1 || c[5] != 0) return ZC_ERR_CORRUPT;
    std::memset(out, 0, sizeof(*out));
    out->format = c[6]; out->policy = c[7]; out->streams = c[8]; out->n_fields = c[9]; out->xor_delta = c[10] & 1;
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

zc_status check_index(const zc_info &info, const uint8_t *d_comp, hipStream_t hs)
{
    uint32_t prev = 0;
    std::vector<uint32_t> idx((size_t)info.n_chunks + 1);
    for (uint32_t f = 0; f < info.n_fields; f++) {
        HIP_TRY(hipMemcpyAsync(idx.data(), d_comp + info.index_offset[f], idx.size() * 4, hipMemcpyDeviceToHost, hs));
        HIP_TRY(hipStreamSynchronize(hs));
        if (idx[0] != prev) return ZC_ERR_CORRUPT;
        for (size_t i = 0; i < idx.size(); i++) { if (idx[i] < prev) return ZC_ERR_CORRUPT; prev = idx[i]; }
    }
    if (info.payload_offset + 16ull * prev != info.total_bytes) return ZC_ERR_CORRUPT;
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
    if (!elem_bits(info.format) || info.total_bytes > comp_bytes || info.streams == 0) return ZC_ERR_INVALID_ARG;
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
        if (fk.ok) LAUNCH_TRY(launch_decode_fp8_fast(fk.exp_kind, fk.sm_kind, info.xor_delta != 0, nullptr, nullptr, n_fast, &d, stream));
        else {
            const bool split = s64_split_ok(info);
            LAUNCH_TRY(launch_decode_s64(info.format, rings, info.xor_delta != 0, split, nullptr, nullptr, split ? n_full : n_fast, &d, stream));
        }
        first_slot = n_full;
    }
    if (first_slot < slots) {
        const uint32_t n_work = (slots - first_slot + cpi - 1) / cpi;
        LAUNCH_TRY(launch_decode(info.format, nullptr, nullptr, n_work, cpi, &d, first_slot, stream));
    }
    return ZC_OK;
}

}  // namespace

// ----------------------------------------------------------------------- C ABI

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

uint64_t zc_workspace_bytes(const uint64_t *n_elems, uint32_t n_tensors, const zc_params *params)
{
    Geometry g;
    Workspace w;
    if (!n_elems || check_params(params, &g) || plan_workspace(g, n_elems, n_tensors, &w)) return 0;
    return w.total;
}

zc_status zc_build_code(const uint64_t *hist, uint32_t alphabet, uint32_t limit, uint8_t *len_out, uint16_t *code_out)
{
    if (!hist || !len_out || !code_out || alphabet == 0 || alphabet > 256) return ZC_ERR_INVALID_ARG;
    if (!build_code_lengths(hist, (int)alphabet, (int)limit, len_out)) return ZC_ERR_INVALID_ARG;
    assign_canonical(len_out, (int)alphabet, code_out);
    return ZC_OK;
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

int zc_code_stale(const zc_info *code, const zc_info *written, double slack)
{
    if (!code || !written || code->format != written->format || code->n_elems == 0 || written->n_elems == 0) return -1;
    if (!elem_bits(code->format) || !(slack >= 0.0)) return -1;
    auto raw = [](const zc_info *i) {
        return (double)((i->n_elems * (uint64_t)elem_bits(i->format) + 7) / 8 + (is_fp4(i->format) ? i->n_elems / scale_block(i->format) : 0));
    };
    return (double)written->total_bytes / raw(written) > (double)code->total_bytes / raw(code) + slack ? 1 : 0;
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
    const bool fast = fk.ok || rings != 0 || sub;
    uint64_t all_slots = 0;
    for (uint32_t t = 0; t < n_tensors; t++) all_slots += tensors[t].d_chunk_ids ? tensors[t].n_chunk_ids : tensors[t].info.n_chunks;
    const uint32_t spg = sub ? sub_slots_per_group(S, all_slots) : split ? 1u : kWavesPerGroup;
    std::vector<TensorDev> descs(n_tensors);
    std::vector<WorkItem> fast_work, work;
    for (uint32_t t = 0; t < n_tensors; t++) {
        const zc_tensor &x = tensors[t];
        const zc_info &info = x.info;
        if (info.format != fmt || info.streams != S) return ZC_ERR_INVALID_ARG;
        if (!x.d_comp || !aligned16(x.d_comp) || (info.n_elems && (!x.d_dst || !aligned16(x.d_dst)))) return ZC_ERR_INVALID_ARG;
        if (info.n_fields == 3 && info.n_elems && (!x.d_scales_out || !aligned16(x.d_scales_out))) return ZC_ERR_INVALID_ARG;
        if (info.xor_delta && (!x.d_xor_base || !aligned16(x.d_xor_base))) return ZC_ERR_INVALID_ARG;
        if (info.total_bytes > x.out_bytes && info.total_bytes > x.comp_capacity) return ZC_ERR_INVALID_ARG;
        descs[t] = make_desc(info);
        descs[t].comp = (uint8_t *)x.d_comp; descs[t].dst = (uint8_t *)x.d_dst; descs[t].scales_out = (uint8_t *)x.d_scales_out;
        descs[t].base = info.xor_delta ? (const uint8_t *)x.d_xor_base : nullptr;
        const uint64_t raw = (info.n_elems * (uint64_t)elem_bits(fmt) + 7) / 8;
        descs[t].ids = x.d_chunk_ids; descs[t].n_ids = x.d_chunk_ids ? x.n_chunk_ids : 0;
        descs[t].dst_bytes = x.d_chunk_ids ? (uint64_t)x.n_chunk_ids * info.chunk_bytes : raw;
        const uint32_t slots = x.d_chunk_ids ? x.n_chunk_ids : info.n_chunks;
        uint32_t first_generic = 0;
        if (fast && (sub || !x.d_chunk_ids)) {
            const uint32_t n_full = (uint32_t)(info.n_elems / ((uint64_t)info.chunk_bytes * 8 / (uint64_t)elem_bits(fmt)));
            const uint32_t n_fast = x.d_chunk_ids ? slots : n_full;        // lists reach here only when every chunk is whole
            for (uint32_t c = 0; c < n_fast; c += spg) fast_work.push_back({t, c});
            first_generic = n_fast;
        }                                                                   // an id list with 64-lane chunks goes through the generic kernel
        for (uint32_t c = first_generic; c < slots; c += cpi) work.push_back({t, c});
    }
    order_for_xcds(fast_work);
    const uint64_t descs_bytes = align256((uint64_t)n_tensors * sizeof(TensorDev));
    const uint64_t fast_bytes = align256(fast_work.size() * sizeof(WorkItem));
    if (ws_bytes < descs_bytes + fast_bytes + work.size() * sizeof(WorkItem)) return ZC_ERR_BUFFER_TOO_SMALL;
    hipStream_t hs = (hipStream_t)stream;
    uint8_t *ws = (uint8_t *)d_ws;
    // one copy from the page-locked staging buffer: no wait, the host arrays above may go away at once
    const Piece all[3] = {{0, descs.data(), descs.size() * sizeof(TensorDev)},
                          {descs_bytes, fast_work.data(), fast_work.size() * sizeof(WorkItem)},
                          {descs_bytes + fast_bytes, work.data(), work.size() * sizeof(WorkItem)}};
    const zc_status up = host_stage().upload(ws, 0, descs_bytes + fast_bytes + work.size() * sizeof(WorkItem), all, 3, hs);
    if (up) return up;
    plan->format = fmt; plan->streams = S; plan->n_tensors = n_tensors;
    plan->n_fast_work = (uint32_t)fast_work.size(); plan->n_work = (uint32_t)work.size();
    plan->fast_exp_kind = (uint32_t)fk.exp_kind; plan->fast_sm_kind = (uint32_t)fk.sm_kind; plan->xor_delta = tensors[0].info.xor_delta;
    plan->fast_kernel = fk.ok ? 1u : (rings ? (split ? 4u : 2u) : (sub ? (fmt == ZC_FMT_BF16 ? 5u : 3u) : 0u)); plan->n_rings = sub ? spg : rings;
    plan->scattered = 0;
    for (uint32_t t = 0; t < n_tensors; t++) if (tensors[t].d_chunk_ids) plan->scattered = 1;
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
        LAUNCH_TRY(launch_decode_fp8_fast((int)plan->fast_exp_kind, (int)plan->fast_sm_kind, plan->xor_delta != 0, (const TensorDev *)ws,
                                          (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && (plan->fast_kernel == 2 || plan->fast_kernel == 4))
        LAUNCH_TRY(launch_decode_s64(plan->format, plan->n_rings, plan->xor_delta != 0, plan->fast_kernel == 4, (const TensorDev *)ws,
                                     (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 3)
        LAUNCH_TRY(launch_decode_fp8_sub(plan->streams, plan->xor_delta != 0, plan->scattered != 0, (const TensorDev *)ws,
                                         (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, plan->n_rings, stream));
    else if (plan->n_fast_work && plan->fast_kernel == 5)
        LAUNCH_TRY(launch_decode_bf16_sub(plan->streams, plan->xor_delta != 0, (const TensorDev *)ws,
                                          (const WorkItem *)(ws + plan->fast_work_offset), plan->n_fast_work, nullptr, plan->n_rings, stream));
    else if (plan->n_fast_work) return ZC_ERR_INVALID_ARG;
    if (plan->n_work)
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
