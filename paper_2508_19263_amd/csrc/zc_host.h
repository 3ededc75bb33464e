// Host-side declarations shared by the files behind the C ABI: container layout and validation
// (zc_container.cpp, no HIP calls), page-locked staging (zc_staging.cpp), the compress side (zc_compress.cpp)
// and the decompress side (zc_decompress.cpp).  Not part of the C ABI.
#pragma once
#include <cstdint>
#include <cstring>
#include <vector>

#include "zc_internal.h"

namespace zc {

// ---- parameters and container layout (zc_container.cpp) -----------------------------------
struct Geometry {
    uint32_t fmt, S, nf;
    uint32_t chunk_bytes;
    uint64_t elems_per_chunk;
    int limit[kMaxFields];
    bool host_codes;            // ZC_FLAG_HOST_CODES
    bool reversed;              // ZC_FLAG_REVERSE_FIELDS: the last field's streams come first in the payload
};

zc_status check_params(const zc_params *p, Geometry *g);
zc_status check_count(const Geometry &g, uint64_t n_elems, uint64_t *n_chunks);
uint64_t field_symbols(uint32_t fmt, int f, uint64_t n_elems);
// offsets of tables / indices / payload for a tensor of nc chunks
void layout(uint32_t fmt, uint64_t nc, uint64_t table_off[3], uint64_t index_off[3], uint64_t *payload_off);

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
inline uint64_t align256(uint64_t x) { return (x + 255) / 256 * 256; }
inline void put32(uint8_t *p, uint32_t v) { std::memcpy(p, &v, 4); }
inline void put64(uint8_t *p, uint64_t v) { std::memcpy(p, &v, 8); }
inline uint32_t get32(const uint8_t *p) { uint32_t v; std::memcpy(&v, p, 4); return v; }
inline uint64_t get64(const uint8_t *p) { uint64_t v; std::memcpy(&v, p, 8); return v; }

constexpr uint64_t kBlobBytes = 1024;     // header + code-length tables of one tensor (<= 64 + 3*256)

// the code of one field as the host knows it
struct FieldCode {
    uint64_t hist[256];
    uint8_t len[256];
    uint16_t code[256];
    uint32_t mode, lmax, konst, distinct;
    uint64_t n_symbols, payload_bits;
};

// the field whose streams come k-th in the payload
inline uint32_t field_at(uint32_t k, uint32_t n_fields, bool reversed) { return reversed ? n_fields - 1 - k : k; }
void fill_info(const Geometry &g, uint32_t policy, bool xor_delta, uint64_t n_elems, uint64_t nc, const FieldCode fc[3], uint64_t total, zc_info *info);
// header + tables exactly as they sit at the start of the container
void serialize_blob(const zc_info &info, uint8_t *blob);
// how the specialised kernels treat a field: 0 table, 1 flat code, 2 raw, 3 constant
uint8_t field_kind(uint32_t mode, uint32_t sym_bits_, const uint8_t *code_len);
// the code-independent and code-dependent parts of a decode descriptor (pointers are left null)
TensorDev make_desc(const zc_info &info);
// header and tables from the first `have` bytes of a container of comp_bytes bytes
zc_status parse_info(const uint8_t *c, uint64_t have, uint64_t comp_bytes, zc_info *out);
// One field's chunk index (n_chunks + 1 entries, host memory): non-decreasing and starting at *prev, which it
// advances to the field's end
zc_status check_index_field(const uint32_t *idx, uint32_t n_chunks, uint32_t *prev);
// Workgroups are handed to the 8 XCDs in turn; reorder a work list so that every XCD walks one contiguous eighth
void order_for_xcds(std::vector<WorkItem> &items);
// slots one workgroup of the sub-wavefront (page) kernels takes
uint32_t sub_slots_per_group(uint32_t streams, uint64_t slots);

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return ZC_ERR_DEVICE; } while (0)
#define LAUNCH_TRY(expr) do { if ((expr) != 0) return ZC_ERR_DEVICE; } while (0)

// ---- page-locked staging (zc_staging.cpp) ---------------------------------------------------
struct Piece { uint64_t off; const void *src; uint64_t bytes; };
// Copies pieces (all inside [lo, hi) of the workspace) to d_ws + lo .. d_ws + hi on `stream`, through one of a few
// page-locked buffers of the library's that are used in turn: one asynchronous copy that needs no wait (the
// buffer outlives the call).
zc_status stage_upload(uint8_t *d_ws, uint64_t lo, uint64_t hi, const Piece *pieces, int n, void *stream);
// a page-locked buffer for one call's read-backs, returned to the library's pool by the destructor
struct LandingLease {
    uint8_t *ptr = nullptr;
    uint64_t cap = 0;
    explicit LandingLease(uint64_t bytes);
    ~LandingLease();
    LandingLease(const LandingLease &) = delete;
    LandingLease &operator=(const LandingLease &) = delete;
};

// ---- the kernel sequence of a compress call (zc_compress.cpp) ---------------------------------
// where everything lives in the workspace of a compress-side call
struct Workspace {
    uint64_t descs, hist_work, scale_work, chunk_work, fast_work, whole_work, other_work, hist, enc, units, scan, blobs, lane_counts, total, host_end;
    uint32_t n_hist_work, n_scale_work, n_chunk_work;
    uint64_t n_units;
};
zc_status plan_workspace(const Geometry &g, const uint64_t *n_elems, uint32_t T, Workspace *w);

// what the geometry of a call decides, the same for every tensor of it
struct CompressShape {
    bool lanes;                 // the code is built on the device and the histogram pass also counts exponents per chunk lane
    bool lanes8;                // the same for the formats of 8-bit symbols (BF16, FP8 in byte symbols): both fields' symbols per chunk lane
    bool lanes_e5m2;            // the same for FP8 E5M2: 32 exponent and 8 sign+mantissa counts per chunk lane
    bool bf16;
    bool rows8;                 // 64 lanes, whole rows, 8 or 16 symbols of 8 bits per run and field (BF16, FP8 in byte symbols, FP8 E5M2): the 64-lane encoder written for BF16
    bool whole_shape;           // 64 lanes, chunks of whole 1 KiB rows: the generic encoder's whole-chunk build
    int whole_mode;             // 2: one whole chunk per work item, shared by its four wavefronts
    uint32_t whole_step, fast_step, cpi;    // chunks per work item of the whole-chunk list, the fast list, the generic kernels
};
CompressShape compress_shape(const Geometry &g, bool device_codes, uint64_t all_chunks);
bool compress_fast_shape(const Geometry &g, uint64_t n_elems, uint64_t bound_bytes);

// work items first, first + step, ... below end
struct ListRange {
    uint32_t first, end, step;
    uint32_t count() const { return (step && end > first) ? (end - first + step - 1) / step : 0u; }
};
// Work lists of one tensor.  hist / lane_hist / scale: histogram blocks.  fast: whole chunks for the FP8 kernels and
// the page kernels' BF16 builds; whole: whole chunks for the generic encoder's 64-lane build (and the BF16 encoder);
// other: whole chunks for the generic encoder where neither applies to the geometry but a specialised kernel might
// have taken them; slow: everything else (a short last chunk, odd geometries).
struct TensorLists { ListRange hist, lane_hist, scale, fast, whole, other, slow; };
TensorLists device_code_lists(const Geometry &g, const CompressShape &sh, uint64_t n_elems, uint64_t nc, bool fast_shape);

// the launches of a compress-side call, given a workspace that holds descriptors and work lists
struct CompressQueue {
    Geometry g;
    Workspace w;
    CompressShape sh;
    uint8_t *ws;
    void *stream;
    uint32_t T;
    bool stats_only;
    uint32_t n_hist, n_lane_hist, n_scale, n_fast, n_whole, n_other, n_slow;     // entries of the work lists
    // pages in one pass (containers with reversed payload order): the fast list is in natural order, chain_step pages per
    // item, and one kernel sizes, places and encodes the tensors whose code suits it; the chain's words and its counter
    // lie at these offsets of the workspace
    bool chained = false;
    uint32_t chain_hold = 0;                                   // words of LDS per page where that kernel keeps the exponent streams, else 0
    uint32_t chain_step = 0;
    uint64_t chain_status = 0, chain_counter = 0;

    TensorDev *d_descs() const { return (TensorDev *)(ws + w.descs); }
    uint64_t *d_hist() const { return (uint64_t *)(ws + w.hist); }
    uint32_t *d_enc() const { return (uint32_t *)(ws + w.enc); }
    uint32_t *d_units() const { return (uint32_t *)(ws + w.units); }
    uint16_t *d_lane_counts() const { return (uint16_t *)(ws + w.lane_counts); }
    const WorkItem *d_list(uint64_t off) const { return (const WorkItem *)(ws + off); }

    zc_status queue_histogram() const;
    zc_status queue_codes(uint32_t policy) const;
    zc_status queue_sizes_and_scan() const;
    zc_status queue_encoders() const;
};

// argument checks of one tensor of a compress-side call
zc_status check_compress_tensor(const Geometry &g, const zc_tensor &x, bool stats_only);
// the compress-side descriptor of one tensor without what depends on its code; false: the destination cannot even
// hold the container's prologue
bool compress_desc(const Geometry &g, const zc_tensor &x, uint64_t nc, uint64_t units_off, bool stats_only, TensorDev *out);

}  // namespace zc
