// Internal declarations shared by the host side (zc_container.cpp, zc_compress.cpp, zc_decompress.cpp,
// zc_codebook.cpp) and the kernels (*.hip) of the HIP library.  Not part of the C ABI.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include "../../include/zc.h"

namespace zc {

constexpr uint32_t kMagic = 0x0031435Au;   // "ZC1\0"
constexpr uint32_t kHeaderBytes = 64;
constexpr int kMaxFields = 3;

// ---- format geometry -------------------------------------------------------
// element format of a (possibly byte-grouped) format, and field values per coded symbol
inline uint32_t base_format(uint32_t fmt)
{
    if (fmt == ZC_FMT_FP4_E2M1_NV) return ZC_FMT_FP4_E2M1_MX;      // same elements, other scales
    return fmt == ZC_FMT_FP8_E4M3_BYTES ? ZC_FMT_FP8_E4M3 : fmt == ZC_FMT_FP4_E2M1_MX_BYTES ? ZC_FMT_FP4_E2M1_MX : fmt;
}
// elements that share one scale byte (0: the format has no scales)
inline uint32_t scale_block(uint32_t fmt) { return fmt == ZC_FMT_FP4_E2M1_NV ? 16 : (fmt == ZC_FMT_FP4_E2M1_MX || fmt == ZC_FMT_FP4_E2M1_MX_BYTES) ? 32 : 0; }
inline int group_of(uint32_t fmt) { return fmt == ZC_FMT_FP8_E4M3_BYTES ? 2 : fmt == ZC_FMT_FP4_E2M1_MX_BYTES ? 4 : 1; }
inline bool is_fp4(uint32_t fmt) { return base_format(fmt) == ZC_FMT_FP4_E2M1_MX; }
inline int elem_bits(uint32_t fmt)
{
    fmt = base_format(fmt);
    return fmt == ZC_FMT_BF16 ? 16 : (fmt == ZC_FMT_FP8_E4M3 || fmt == ZC_FMT_FP8_E5M2) ? 8 : fmt == ZC_FMT_FP4_E2M1_MX ? 4 : 0;
}
inline int num_fields(uint32_t fmt) { return is_fp4(fmt) ? 3 : 2; }
inline int sym_bits(uint32_t fmt, int f)
{
    if (f == 2 || group_of(fmt) > 1 || fmt == ZC_FMT_FP8_E5M2) return 8;
    return fmt == ZC_FMT_BF16 ? 8 : fmt == ZC_FMT_FP8_E4M3 ? 4 : 2;
}
// symbols per 16-byte run of the field's plain array
inline int run_len(uint32_t fmt, int f) { return f == 2 ? 16 : 128 / elem_bits(fmt) / group_of(fmt); }
inline uint64_t pad16(uint64_t x) { return (x + 15) / 16 * 16; }
// refill period of a field's stream: symbols between two refill steps
inline int refill_period(int G, int lmax)
{
    int r = 1;
    if (lmax < 1) lmax = 1;
    while (2 * r * lmax <= 32) r *= 2;
    return r < G ? r : G;
}

// ---- per-tensor descriptor handed to every kernel --------------------------
struct alignas(16) TensorDev {
    const uint8_t *src;       // compress: elements
    const uint8_t *base;      // XOR base or null
    const uint8_t *scales;    // compress, FP4: scale bytes
    uint8_t *comp;            // container
    uint8_t *dst;             // decompress: elements out
    uint8_t *scales_out;      // decompress, FP4
    const uint32_t *ids;      // decompress: chunk id list (slot i decodes chunk ids[i]) or null (slot i = chunk i)
    uint64_t dst_bytes;       // decompress: bytes that may be written at dst; compress: at comp
    uint64_t n_elems;
    uint64_t total_bytes;     // decompress: container size (bounds for reads)
    uint64_t payload_off;
    uint32_t n_chunks;
    uint32_t chunk_bytes;
    uint32_t table_off[kMaxFields];
    uint32_t index_off[kMaxFields];
    uint32_t n_ids;           // decompress: entries of ids
    uint32_t units_off;       // compress: first entry of this tensor in the units array (field-major, n_chunks each)
    uint32_t streams;         // S
    uint8_t mode[4], lmax[4], konst[4], period[4];
    uint8_t kind[4];          // how the specialised kernels treat the field (0 table, 1 flat code, 2 raw, 3 constant)
    uint8_t fast_shape;       // compress: the tensor's geometry suits the specialised size/encode kernels of its format
    uint8_t route;            // compress: who takes the whole chunks.  0 = the generic kernels; 1 = the FP8 size and encode
                              // kernels; 2 = BF16: with 64 lanes per chunk the generic size pass and the BF16 encoder, with
                              // fewer the BF16 builds of the page size/encode kernel
    uint8_t pad_[6];
};

struct WorkItem { uint32_t tensor, first; };   // `first`: first chunk / block of the item

#ifdef __HIPCC__
#define ZC_HOST_DEVICE __host__ __device__
#else
#define ZC_HOST_DEVICE
#endif
// Workgroups are handed to the 8 XCDs (each with an L2 of its own) in turn, so workgroup p runs on XCD p % 8.
// Work lists are ordered so that every XCD walks one contiguous eighth of the list: position p of the ordered list
// holds the item at this position of the natural list of n items.
ZC_HOST_DEVICE inline uint64_t xcd_order_source(uint64_t p, uint64_t n)
{
    constexpr uint64_t kXcds = 8;
    if (n < 2 * kXcds) return p;
    const uint64_t q = n / kXcds, r = n % kXcds, k = p % kXcds;
    return k * q + (k < r ? k : r) + p / kXcds;
}

// histogram block: bytes of input handled by one workgroup pass
constexpr uint32_t kHistBlockBytes = 256 * 1024;
// chunks (or chunk slots) handled by one workgroup of the chunk kernels
constexpr uint32_t kWavesPerGroup = 4;

// per-tensor scratch written by the scan kernel and read back by the host
struct ScanOut { uint32_t field_units[kMaxFields]; uint32_t total_units; };

// ---- host-side code construction (zc_codebook.cpp) --------------------------
// Length-limited canonical Huffman code; returns false if 2^limit < used symbols.
bool build_code_lengths(const uint64_t *hist, int alphabet, int limit, uint8_t *len_out);
void assign_canonical(const uint8_t *len, int alphabet, uint16_t *code_out);

// ---- code construction on the device (zc_codes.hip) ---------------------------
struct CodeParams {
    uint32_t fmt, policy, nf;
    int32_t limit[kMaxFields];
    uint32_t blob_bytes;      // stride of the per-tensor header blobs
    uint32_t run_len;         // symbols per 16-byte run of an element field
};
// histograms (768 counters per tensor, as k_hist leaves them) -> encode tables, the code-dependent bytes of the
// header blobs and of the descriptors (mode, lmax, konst, period, kind, route)
int launch_codes(TensorDev *d_descs, uint32_t n_tensors, const uint64_t *d_hist, const CodeParams &cp, uint8_t *d_blobs, uint32_t *d_enc, void *stream);

// ---- kernel launchers (zc_kernels.hip); all return a hipError_t as int ------
int launch_hist(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                int scales_view, uint64_t *d_hist, void *stream);
int launch_zero(uint64_t *d_words, uint64_t n_words, void *stream);
int launch_copy(const void *d_src, void *d_dst, uint64_t bytes, void *stream);
int launch_copy_chunked(const void *d_src, void *d_dst, uint64_t bytes, uint32_t chunk_bytes, void *stream);
// skip_routes: bit r set = leave tensors of route r to the specialised kernel that takes their whole chunks
// whole: 0 = any chunks, 1 = up to four whole 64-lane chunks per work item, 2 = one such chunk per work item, shared
// by the workgroup's four wavefronts
int launch_sizes(uint32_t fmt, int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                 const uint32_t *d_enc_tables, uint32_t *d_units, void *stream);
// d_blobs: per tensor the header and code-length tables to put at the start of its container (blob_bytes apart), or null
int launch_scan(const TensorDev *d_descs, uint32_t n_tensors, int n_fields, bool reversed, int skip_routes, const uint32_t *d_units, ScanOut *d_out, const uint8_t *d_blobs,
                uint32_t blob_bytes, void *stream);
int launch_encode(uint32_t fmt, int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                  const uint32_t *d_enc_tables, void *stream);
int launch_decode(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint32_t chunks_per_item,
                  const TensorDev *single, uint32_t first_slot, void *stream);
// specialised FP8 decode of full chunks (zc_decode_fast.hip); exp_kind 0 = single, 1 = pair lookups; sm_kind 0 = flat, 1 = raw
int launch_decode_fp8_fast(int exp_kind, int sm_kind, bool xor_delta, bool with_ids, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, void *stream);
// FP8, fewer than 64 lanes per chunk (pages), optional id list (zc_decode_fast.hip)
int launch_decode_fp8_sub(uint32_t streams, bool xor_delta, bool scattered, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                          const TensorDev *single, uint32_t slots_per_group, void *stream);
// BF16, fewer than 64 lanes per chunk (pages), exponent field table decoded, sign+mantissa flat or raw, optional id list
int launch_decode_bf16_sub(uint32_t streams, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, uint32_t slots_per_group, void *stream);
// any format, 64 lanes per chunk, full chunks (zc_decode_fast.hip); n_rings = element fields that are table decoded (1..2)
int launch_decode_s64(uint32_t fmt, uint32_t n_rings, bool xor_delta, bool split, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                      const TensorDev *single, void *stream);
int launch_decode_s64_tail(uint32_t fmt, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev *single,
                           uint32_t first_slot, bool skip_whole, void *stream);
// BF16, 64 lanes per chunk, full chunks, exponent field table decoded (refill period 2, 4 or 8), sign+mantissa field table
// decoded on the same period, flat coded, raw or constant (zc_decode_fast.hip)
int launch_decode_bf16_s64(uint32_t n_rings, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, void *stream);
// FP8 E5M2, 64 lanes per chunk, full chunks, exponent field table decoded (refill period 2, 4 or 8), sign+mantissa field
// coded with the flat 3-bit code over the values 0..7 (zc_decode_fast.hip)
int launch_decode_e5m2(bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev *single, void *stream);
// FP8, 64 lanes, full chunks, exponent codes <= 8 bits, sign+mantissa flat or raw (zc_encode_fast.hip)
int launch_sizes_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream);
// FP8, 64 lanes, chunks of kHistBlockBytes: the histogram pass that also counts exponents per chunk lane (one work
// item per whole chunk; 16 u16 per lane, 2 KiB per chunk, at lane_counts[(units_off / 2 + chunk) * 1024]), and the
// size pass that reads those counts instead of the source (same work list as launch_sizes_fp8) (zc_hist_lanes.hip).
// e5m2: the E5M2 layout instead, 32 exponent and 8 sign+mantissa counts per lane (40 u16, 5 KiB per chunk, at
// lane_counts[(units_off / 2 + chunk) * 2560]), read by launch_sizes_e5m2_counts (work list of the generic whole-chunk
// size pass, which it replaces for every tensor)
int launch_hist_fp8_lanes(bool e5m2, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint16_t *d_lane_counts, void *stream);
int launch_sizes_e5m2_counts(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, const uint16_t *d_lane_counts,
                             uint32_t *d_units, void *stream);
// BF16 / FP8 in byte symbols, 64 lanes, chunks of kHistBlockBytes: the same for fields of 8-bit symbols (256 counts
// of 16 bits per lane and field, 64 KiB per chunk, at lane_counts + (units_off / 2 + chunk) * 16384 words), and the size pass of
// the tensors of route 2 from those counts (zc_hist_lanes.hip)
int launch_hist_rows8_lanes(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint32_t *d_lane_counts, void *stream);
int launch_sizes_rows8_counts(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc,
                              const uint32_t *d_lane_counts, uint32_t *d_units, void *stream);
// Two-field formats, 64 lanes: stream sizes of the chunks of a generic work list (up to kWavesPerGroup chunks per item)
// from the closed form over the lanes' bit totals; meant for the short last chunks of tensors (zc_hist_lanes.hip)
int launch_sizes_tail(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream);
int launch_sizes_fp8_counts(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, const uint16_t *d_lane_counts,
                            uint32_t *d_units, void *stream);
int launch_encode_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream);
// BF16 (FP8 in byte symbols, FP8 E5M2), 64 lanes, full chunks, exponent field table coded, sign+mantissa flat, raw or table coded;
// work items as for the generic whole-chunk build (zc_encode_fast.hip)
int launch_encode_bf16(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream);
// K/V pages, 4 to 32 lanes per chunk (zc_encode_pages.hip)
int launch_compress_pages_fused(uint32_t streams, uint32_t bf16_periods, bool reversed, const TensorDev *d_descs, uint32_t n_tensors, const uint32_t *d_enc,
                                const uint8_t *d_blobs, uint32_t blob_bytes, ScanOut *d_out, void *stream);
uint32_t compress_pages_fused_limit();      // most pages per tensor the fused kernel takes
// pages in one pass over the source: containers with their fields in reverse order, dictionary calls; see the kernel
int launch_compress_pages_chained(uint32_t streams, uint32_t bf16_period, uint32_t hold, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                                  uint32_t slots_per_item, const uint32_t *d_enc, const uint8_t *d_blobs, uint32_t blob_bytes, uint64_t *d_status,
                                  uint64_t *d_counter, ScanOut *d_out, void *stream);
uint32_t compress_pages_chained_limit();    // most pages per work item of that kernel
uint32_t compress_pages_held_words();       // words of LDS for the exponent streams of a work item in its `hold` build
int launch_encode_fp8_sub(uint32_t streams, int write, bool bf16, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc,
                          uint32_t *d_units, uint32_t slots_per_group, void *stream);
uint32_t chunks_per_work_item(uint32_t streams);

}  // namespace zc
