/*
 * zc.h -- C ABI of the field-split Huffman tensor codec for MI355X (gfx950).
 *
 * Method: Heilper & Singer, "Lossless Compression of Neural Network Components:
 * Weights, Checkpoints, and K/V Caches in Low-Precision Formats" (2025).
 * Every value of a BF16 / FP8 (E4M3, E5M2) / FP4 E2M1 tensor is split into its exponent
 * bits and its sign+mantissa bits (Sec. 3.1, 3.2, 3.4, Fig. 5); each field is
 * histogrammed over the tensor and Huffman coded on its own (Sec. 3.1, 3.2, 4);
 * FP4 block scales form a third field (Sec. 3.4, 4.4); a checkpoint delta is the
 * bitwise XOR against a base tensor (Sec. 3.1, 4.1); a field that does not
 * compress may be stored as is (Sec. 3.1, 4.3); data is cut into fixed-size
 * chunks that decode independently (Sec. 3.1), which also serves paged K/V
 * caches (Sec. 3.3, 4.3, 5.2).  The result is lossless (Sec. 1, 2.2).
 *
 * Conventions for every entry point
 *   - "device" pointers are GPU memory of the current HIP device, 16-byte
 *     aligned, owned by the caller; "host" pointers are ordinary memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued on it.  Calls that must read results back (noted
 *     below) synchronise that stream before returning.
 *   - The library never allocates or frees device memory: scratch space comes in
 *     through `d_ws`.  The only state it keeps between calls is page-locked host
 *     memory: a few buffers through which descriptors, work lists and tables are
 *     uploaded (used in turn, so that calls queued back to back do not wait for each
 *     other's copies) and a few through which sizes and headers are read back (allocated
 *     on first use, grown when needed, held until zc_release_host_buffers() or the end of
 *     the process).  No environment variable is read.
 *   - HIP graphs: only zc_decompress_batch_run may be recorded by stream capture (it
 *     launches kernels and nothing else).  Every other entry point that takes a stream
 *     copies from or to the library's page-locked buffers, may wait on an event and may
 *     allocate page-locked memory, none of which a capture allows; a captured copy would
 *     also replay whatever a later call left in the buffer.
 *   - Errors are returned as zc_status; nothing is thrown.  On error the
 *     destination contents are unspecified but nothing is written outside the
 *     capacities given.
 *   - Element layout: BF16 little-endian u16; FP8 one byte; FP4 two elements per
 *     byte, element 2i in the low nibble, with one scale byte per 32 (MX: E8M0) or
 *     16 (NV: E4M3) consecutive elements in a separate array.
 */
#ifndef ZC_H
#define ZC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZC_OK = 0,
    ZC_ERR_INVALID_ARG = 1,      /* bad pointer, size, alignment or parameter value */
    ZC_ERR_UNSUPPORTED = 2,      /* unknown format / struct size */
    ZC_ERR_BUFFER_TOO_SMALL = 3, /* destination or workspace capacity */
    ZC_ERR_CORRUPT = 4,          /* container fails validation */
    ZC_ERR_DEVICE = 5            /* a HIP call failed */
} zc_status;

typedef enum {
    ZC_FMT_BF16 = 1,        /* fields: 8-bit exponent, 8-bit sign+mantissa (Sec. 3.1) */
    ZC_FMT_FP8_E4M3 = 2,    /* fields: 4-bit exponent, 4-bit sign+mantissa (Sec. 3.2) */
    ZC_FMT_FP4_E2M1_MX = 3, /* fields: 2-bit exponent, 2-bit sign+mantissa, 8-bit E8M0 scale (Sec. 3.4) */
    /* The same elements and fields as formats 2 and 3, coded in byte-sized groups (Sec. 3.2 with Fig. 7:
     * FP8 exponents, and sign+mantissa values, paired into bytes; Sec. 3.4: four 2-bit FP4 values per
     * byte): one Huffman symbol is one byte of the packed field array, i.e. 2 (FP8) or 4 (FP4)
     * consecutive field values with the first in the low bits, so every field has a 256-symbol alphabet.
     * A last group that runs past the tensor is filled with zero values. */
    ZC_FMT_FP8_E4M3_BYTES = 4,
    ZC_FMT_FP4_E2M1_MX_BYTES = 5,
    /* NVFP4 (Sec. 3.4): the E2M1 elements of format 3 with one FP8 (E4M3) scale byte per 16 elements
     * (d_scales holds n_elems / 16 bytes); fields as format 3, the scale bytes coded as 8-bit symbols. */
    ZC_FMT_FP4_E2M1_NV = 6,
    /* The other FP8 variant of Sec. 3.2, E5M2 (s eeeee mm): a 5-bit exponent and a 3-bit sign+mantissa
     * value per element, each held in an 8-bit symbol (alphabets of 256 of which 32 and 8 can occur), so
     * that a lane's run of 16 elements is 16 symbols in both fields.  zc_field_stats.ratio_payload of
     * this format is relative to those 8 bits. */
    ZC_FMT_FP8_E5M2 = 7
} zc_format;

typedef enum {
    ZC_POLICY_HUFF_ALL = 0, /* every field with >= 2 distinct symbols is Huffman coded */
    ZC_POLICY_AUTO = 1      /* a field is stored raw unless Huffman saves >= 1/16 (Sec. 3.1) */
} zc_policy;

typedef enum { ZC_MODE_EMPTY = 0, ZC_MODE_HUFF = 1, ZC_MODE_RAW = 2, ZC_MODE_CONST = 3 } zc_mode;

typedef struct {
    uint32_t struct_size;       /* = sizeof(zc_params): the struct may grow at its end, older sizes stay valid */
    uint32_t format;            /* zc_format */
    uint32_t chunk_bytes;       /* element bytes per chunk; multiple of 16 (FP4: of 256) */
    uint32_t max_code_len[3];   /* per field, 1..16 with 2^L >= alphabet; 0 = 16 for 8-bit symbols, else 8 */
    uint32_t streams_per_chunk; /* lanes per chunk: 1,2,4,...,64; 0 = 64 */
    uint32_t policy;            /* zc_policy */
    uint32_t flags;             /* ZC_FLAG_* bits; absent (read as 0) when struct_size is the 32 bytes of the first layout */
} zc_params;

/* Choosing the geometry.  Every geometry above gives a valid container; these give the fast kernels:
 *   - 64 lanes: chunk_bytes a multiple of 1024 (whole rows of 16 bytes per lane).  Other chunk sizes are compressed
 *     by the generic kernels (1.25 x slower) and decode about 1.35 x slower on MI355X (48 KiB + 16 against 48 KiB);
 *     the short last chunk of a tensor costs a set of tensors a second, small launch (1.1 x for 224 tensors).
 *   - chunks below 16 KiB (K/V pages, Sec. 3.3): 4 to 32 lanes with chunk_bytes a multiple of 16 * lanes.  A
 *     wavefront then decodes 64 / lanes chunks at once; with 64 lanes it decodes one small chunk at a time (a 2 KiB
 *     page: 2.3 x slower from an id list) and every lane's look-ahead words eat the gain (ratio 1.00 against 0.86).
 *   - max_code_len of the exponent field: up to 8 keeps four symbols per refill step for FP8 (the default); 9 to 16
 *     halves the step and costs about 40 % of decode speed for 0.2 % of size on FP8 weights.  For BF16 and for byte
 *     symbols a limit of 11 keeps every code inside the decoders' lookup index (5 to 7 % faster, 0.5 % larger).
 * Where the tensors lie: measured on MI355X, a decode call whose output tensors all lie within one stretch of a few tens
 * of GiB of device memory that was allocated in one go runs about 14 % slower than the same call with its outputs in
 * two such stretches (2.5 - 2.6 against 2.2 ms for 7 GB of FP8 weights); a plain linear copy shows no such difference.
 * Nothing in the addresses tells which is which; outputs spread over more of the memory (a larger model, or two
 * buffers allocated far apart) get the faster case. */

/* zc_params.flags.  HOST_CODES: the compress calls build their codes on the host instead of on the device: the
 * same containers, one more wait per call (the histogram is read back).  What statistics and dictionary
 * training do anyway; meant for checking one construction against the other.
 * REVERSE_FIELDS: the container keeps its fields in reverse order in the payload (the streams of the last field first;
 * tables and indices stay where they are; header flag bit 1, zc_info.payload_order = 1).  The paper fixes no arrangement
 * of the streams (Sec. 3.1 asks only that blocks can be reached at random).  With the sign+mantissa streams of FP8 and
 * BF16 pages in front (they have one fixed size when flat or raw), the place of an exponent stream depends on the
 * exponent streams before it alone, and a dictionary call compresses K/V pages in ONE pass over them (Sec. 5.2: that
 * compression is on the critical path) instead of a size pass, a scan and an encoder.  Every decode entry point takes
 * both orders. */
enum { ZC_FLAG_HOST_CODES = 1, ZC_FLAG_REVERSE_FIELDS = 2 };

/* Parsed, validated container header plus the code-length tables: everything the
 * host needs to launch a decode.  Filled by zc_compress / zc_read_info; may be
 * cached by the caller for as long as the container bytes do not change. */
typedef struct {
    uint32_t format, policy, streams, n_fields, xor_delta, chunk_bytes;
    uint32_t n_chunks, payload_order;   /* payload_order: 0 = field 0's streams first, 1 = the last field's first */
    uint64_t n_elems;
    uint64_t total_bytes;       /* size of the container */
    uint64_t payload_offset;
    uint64_t table_offset[3];   /* code-length table of each field */
    uint64_t index_offset[3];   /* chunk index of each field */
    uint8_t mode[3], sym_bits[3], max_len[3], const_symbol[3];
    uint8_t code_len[3][256];
} zc_info;

typedef struct {
    uint32_t alphabet, distinct, mode, max_len;
    uint64_t n_symbols;
    uint64_t hist[256];
    uint8_t code_len[256];
    double entropy_bits;        /* -sum p log2 p, bits per symbol */
    double mean_code_len;       /* payload_bits / n_symbols */
    uint64_t payload_bits;      /* sum f*len (HUFF), n*sym_bits (RAW), 0 (CONST) */
    uint64_t stream_bytes;      /* bytes of this field's chunk streams in the container */
    double ratio_payload;       /* payload_bits / (n_symbols*sym_bits); "ratio" as in Sec. 4: coded/original */
} zc_field_stats;

typedef struct {
    uint32_t n_fields, reserved;
    uint64_t raw_bytes;         /* element bytes + scale bytes */
    uint64_t container_bytes;
    double ratio_payload_total;
    double ratio_container_total;
    zc_field_stats field[3];
} zc_stats_out;

/* One tensor of a batched call (host array).  Inputs are set by the caller;
 * `out_bytes` and `info` are filled by zc_compress_batch and read by zc_decompress_batch. */
typedef struct {
    const void *d_src;          /* compress: elements (device) */
    const void *d_xor_base;     /* device, same shape as the tensor, or NULL (Sec. 3.1 delta) */
    const void *d_scales;       /* compress, FP4 only: one scale byte per 32 (MX) or 16 (NV) elements (device) */
    uint64_t n_elems;
    void *d_comp;               /* container (device): written by compress, read by decompress */
    uint64_t comp_capacity;     /* compress: bytes available at d_comp */
    void *d_dst;                /* decompress: elements out (device) */
    void *d_scales_out;         /* decompress, FP4 only */
    const uint32_t *d_chunk_ids;/* decompress: device list of chunk ids to decode densely into d_dst (chunk
                                   ids[i] -> d_dst + i*chunk_bytes), or NULL for the whole tensor */
    uint32_t n_chunk_ids, reserved;
    uint64_t out_bytes;         /* container size */
    zc_info info;
} zc_tensor;

/* Worst-case container size for n_elems (0 if the parameters are invalid).  Host only. */
uint64_t zc_compress_bound(uint64_t n_elems, const zc_params *params);

/* Scratch bytes a call on these tensors needs in d_ws (compress, stats and the
 * batched decompress).  n_elems: host array of n_tensors element counts.  A few hundred bytes per chunk and a few KB
 * per tensor, except for 64 lanes with chunks of 256 KiB, where the histogram pass leaves symbol counts per chunk lane
 * for the size pass (so that the source is read twice, not three times): 2 KiB per chunk for FP8 E4M3, 5 KiB for
 * FP8 E5M2, and 64 KiB per chunk, a quarter of the tensor, for BF16 and FP8 in byte symbols. */
uint64_t zc_workspace_bytes(const uint64_t *n_elems, uint32_t n_tensors, const zc_params *params);

/* Compress one tensor: field split (+ XOR delta) and per-field histogram over the tensor,
 * length-limited canonical Huffman code per field, per-chunk stream sizes, exclusive scan
 * into the chunk index, chunked encode (Sec. 3.1, 3.2, 3.4, 4).
 * d_src/d_xor_base/d_scales/d_dst/d_ws: device.  out_bytes, out_info (may be NULL): host.
 * dst_capacity must hold the result (zc_compress_bound always suffices), else
 * ZC_ERR_BUFFER_TOO_SMALL.  The code is built on the device from the device histogram, so the
 * whole sequence is queued without a wait in between; the call then waits once, for the sizes
 * (and for nothing but them when dst_capacity >= zc_compress_bound: the encoder is queued
 * first).  n_elems == 0 gives a header-only container. */
zc_status zc_compress(const void *d_src, uint64_t n_elems, const zc_params *params,
                      const void *d_xor_base, const void *d_scales,
                      void *d_dst, uint64_t dst_capacity, uint64_t *out_bytes, zc_info *out_info,
                      void *d_ws, uint64_t ws_bytes, void *stream);

/* Same over a host array of tensors sharing one zc_params: one launch sequence for the set. */
zc_status zc_compress_batch(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params,
                            void *d_ws, uint64_t ws_bytes, void *stream);
/* zc_compress_batch without any wait on the stream: histogram, code construction, size pass, scan and
 * encoder are queued and the call returns.  Every comp_capacity must be at least
 * zc_compress_bound(n_elems) (else ZC_ERR_BUFFER_TOO_SMALL, nothing queued).  out_bytes and info are not
 * filled in: once the stream has reached this point each container's header holds its size and its
 * code, and zc_read_info or the decompress entry points read them from there.  d_ws must stay
 * untouched until then. */
zc_status zc_compress_batch_async(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params,
                                  void *d_ws, uint64_t ws_bytes, void *stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  zc_compress_batch_async for ONE tensor without a workspace argument and without any allocation,
 * copy or wait: the call launches kernels on `stream` and nothing else (no hipMalloc, hipHostMalloc or hipFree,
 * no page-locked staging, no heap memory).  The scratch that the other compress calls take through d_ws is a
 * file-scope device array of ZC_NOALLOC_SCRATCH_BYTES inside the library (every GPU the library runs on holds
 * its own copy until the process ends), and descriptor, header and work lists are written into it by a kernel
 * from its arguments.  Codes are built on the device; the container is byte for byte what zc_compress writes.
 * Limits: zc_workspace_bytes(&n_elems, 1, params) must not exceed ZC_NOALLOC_SCRATCH_BYTES (which admits e.g.
 * 504 MiB of FP8 in 256 KiB chunks or 901 MiB of FP8 K/V pages of 2 KiB in one call) and dst_capacity
 * must be at least zc_compress_bound(n_elems, params), else ZC_ERR_BUFFER_TOO_SMALL and nothing is queued;
 * ZC_FLAG_HOST_CODES is refused (ZC_ERR_INVALID_ARG).  out size and code are not returned: once the stream has
 * reached this point the container's header holds them (zc_read_info).  All calls on one GPU share that GPU's
 * array: a second call may be queued behind the first on the SAME stream (stream order keeps them apart), but
 * calls on different streams, or from threads that do not order their work, race on it. */
#define ZC_NOALLOC_SCRATCH_BYTES (4u << 20)
zc_status zc_compress_noalloc(const void *d_src, uint64_t n_elems, const zc_params *params,
                              const void *d_xor_base, const void *d_scales,
                              void *d_dst, uint64_t dst_capacity, void *stream);

/* Static dictionaries (Sec. 3.3, 5.2: a code computed ahead of time on representative data and
 * reused while the exponent distribution stays stable, e.g. across K/V-cache time steps).
 * zc_train_code builds a dictionary from a representative tensor: its per-field histogram with
 * every count raised by one (so that any symbol can be coded later), then the usual code
 * construction and raw/Huffman decision.  In *out_code, format, policy, mode[], sym_bits[],
 * max_len[] and code_len[][] describe the dictionary; n_elems, n_chunks, payload_offset and
 * total_bytes are those of the training tensor's container under it (nothing is written).
 * Synchronises.
 * zc_compress_with_code / zc_compress_batch_with_code code every tensor with that dictionary:
 * no histogram pass and no code construction.  The container is an ordinary one (it carries the dictionary's length tables), so
 * every decompress entry point reads it.  A dictionary whose Huffman fields do not form a
 * complete prefix code over the whole alphabet is rejected with ZC_ERR_INVALID_ARG.
 * K/V pages (FP8 or BF16, 4 to 32 lanes, every tensor whole pages): a call whose tensors have at most 512 pages each runs as
 * one kernel, one workgroup per tensor; with ZC_FLAG_REVERSE_FIELDS a call over tensors of any number of pages runs as
 * one kernel that reads the pages once (on MI355X 1.4 against 1.7 ms for 2.1 GB of FP8 pages; fastest for FP8 pages of
 * at most 2 KiB and BF16 pages of at most 4 KiB, whose coded exponents wait on chip for their place, and with a
 * dictionary that suits the data: a page whose coded exponents are longer than the plain ones is coded twice);
 * otherwise a size pass, a scan and an encoder are queued.  The containers are the same whichever way they were written.
 * zc_code_stale (host arithmetic only) is the refresh test of Sec. 3.3: 1 when the container
 * described by *written (from a *_with_code call) is larger, as a fraction of its raw size, than
 * the training tensor's was by more than `slack` (absolute, e.g. 0.02), 0 when not, -1 on
 * arguments that do not fit together. */
zc_status zc_train_code(const void *d_src, uint64_t n_elems, const zc_params *params,
                        const void *d_xor_base, const void *d_scales, zc_info *out_code,
                        void *d_ws, uint64_t ws_bytes, void *stream);
zc_status zc_compress_with_code(const void *d_src, uint64_t n_elems, const zc_params *params, const zc_info *code,
                                const void *d_xor_base, const void *d_scales,
                                void *d_dst, uint64_t dst_capacity, uint64_t *out_bytes, zc_info *out_info,
                                void *d_ws, uint64_t ws_bytes, void *stream);
zc_status zc_compress_batch_with_code(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, const zc_info *code,
                                      void *d_ws, uint64_t ws_bytes, void *stream);
/* zc_compress_batch_with_code without any wait on the stream, for compression on the critical path of a
 * decoding step (Sec. 5.2): every kernel is queued and the call returns.  Every comp_capacity must be at
 * least zc_compress_bound(n_elems) (else ZC_ERR_BUFFER_TOO_SMALL, nothing queued).  out_bytes and
 * info.total_bytes are left 0: once the stream has reached this point the container's header holds its
 * size, and zc_read_info or the decompress entry points read it from there.  d_ws must stay untouched
 * until then. */
zc_status zc_compress_batch_with_code_async(zc_tensor *tensors, uint32_t n_tensors, const zc_params *params, const zc_info *code,
                                            void *d_ws, uint64_t ws_bytes, void *stream);
int zc_code_stale(const zc_info *code, const zc_info *written, double slack);

/* Read and validate a container's header and tables (blocking copy of at most 1 KiB from
 * the device; with check_index != 0 also the chunk index).  d_comp: device; out: host. */
zc_status zc_read_info(const void *d_comp, uint64_t comp_bytes, int check_index, zc_info *out, void *stream);

/* The same validation for a container held in HOST memory; no device is touched.  host_bytes: the first
 * have_bytes bytes of a container of container_bytes bytes (have_bytes <= container_bytes; the header and the
 * code-length tables lie in the first 1 KiB, the chunk index ends at payload_offset).  Checked: magic, version,
 * format and geometry, the layout offsets, a total size that is at most container_bytes, every field's mode,
 * symbol width and code-length table (a complete prefix code whose longest length is the one recorded), and
 * with check_index != 0 that the chunk index of every field is non-decreasing, continues where the field before
 * ended and ends at the container's size.  ZC_ERR_CORRUPT when any of it fails (Sec. 3.1: the per-chunk
 * metadata is what decoding relies on); ZC_ERR_INVALID_ARG when check_index is asked for and have_bytes does
 * not reach the end of the index. */
zc_status zc_validate_container(const void *host_bytes, uint64_t have_bytes, uint64_t container_bytes, int check_index, zc_info *out);

/* Wait for the uploads still in flight from the library's page-locked buffers, then free those buffers and
 * the read-back buffers no call holds.  The next call that needs one allocates it again.  Must not run
 * concurrently with other calls into the library on the streams it waits for. */
zc_status zc_release_host_buffers(void);

/* Decompress a whole tensor (the inverse of Sec. 3.1 / 3.2 / 3.4's split-and-code, exact as Sec. 1 and
 * 2.2 require; Sec. 5.1, 5.2: paid on every load, so it is the path to keep fast): per chunk,
 * table-driven decode of every field and re-interleave into the original bit patterns (XORed
 * with the base for a delta container, Sec. 3.1 / 4.1).  info: host, from zc_compress / zc_read_info, or NULL (then the header is
 * read with a blocking copy first).  Does not synchronise when info is given.
 * d_scales_out: FP4 only.  d_xor_base: required iff the container is a delta.
 * A zc_info whose sizes cannot belong to a container (total_bytes below payload_offset or above
 * comp_bytes, chunk_bytes 0, a chunk count that does not follow from n_elems) is refused with
 * ZC_ERR_INVALID_ARG; this includes the zc_info the *_async compress calls leave behind, whose
 * total_bytes is 0 until zc_read_info has filled it in. */
zc_status zc_decompress(const void *d_comp, uint64_t comp_bytes, const zc_info *info,
                        void *d_dst, uint64_t dst_capacity, void *d_scales_out,
                        const void *d_xor_base, void *stream);

/* Random-access decode (Sec. 3.1: chunks decode independently; Sec. 4.3 / 5.2: K/V pages):
 * chunk d_chunk_ids[i] is written to d_dst + i*chunk_bytes (and its scales to
 * d_scales_out + i * the scale bytes of a whole chunk: chunk_bytes/16 for MX, chunk_bytes/8 for NV).  A short last chunk leaves the rest of its slot
 * untouched.  d_chunk_ids: device array of n_ids u32, each < n_chunks (ids out of range
 * are skipped).  Delta containers: d_xor_base is the whole base tensor. */
zc_status zc_decompress_chunks(const void *d_comp, uint64_t comp_bytes, const zc_info *info,
                               const uint32_t *d_chunk_ids, uint32_t n_ids,
                               void *d_dst, uint64_t dst_capacity, void *d_scales_out,
                               const void *d_xor_base, void *stream);

/* Whole-set decode in one launch: every tensor's d_comp/info/d_dst (and d_xor_base,
 * d_scales_out) must be set.  All tensors must share format and streams.  A tensor with
 * d_chunk_ids set decodes only those chunks, densely (random-access page decode of a whole
 * K/V cache in one launch).  The per-tensor descriptors and the work list go to d_ws in a copy
 * queued on the stream ahead of the kernels; the call never waits.  Every info must describe a
 * written container (see zc_decompress): one left by an *_async compress call is refused with
 * ZC_ERR_INVALID_ARG until zc_read_info has filled it in. */
zc_status zc_decompress_batch(const zc_tensor *tensors, uint32_t n_tensors,
                              void *d_ws, uint64_t ws_bytes, void *stream);

/* The two halves of zc_decompress_batch, for callers that decode the same set more than
 * once: _plan validates, queues the upload of the descriptors and the work lists to d_ws on the
 * stream (from a page-locked buffer of the library's: no wait) and fills *plan (host); _run only
 * enqueues the decode kernels on d_ws as left by _plan, on the same stream or one ordered after it
 * (never synchronises; it makes kernel launches and nothing else, so it may be recorded into a HIP
 * graph by stream capture and replayed, _plan having completed before the capture).  The plan is
 * plain data; it stays valid while d_ws, the containers and the destination pointers are unchanged. */
typedef struct {
    uint32_t format, streams, n_tensors;
    uint32_t n_fast_work, n_work;               /* work items of the specialised / generic kernel */
    uint32_t fast_kernel;                       /* 0 none, 1 FP8 specialised, 2 64-lane full-chunk kernel, 3 FP8 small chunks,
                                                   4 = 2 with every chunk shared by four wavefronts (no table-decoded element field),
                                                   5 BF16 small chunks, 6 BF16 with 64 lanes (table-decoded exponents),
                                                   7 FP8 E5M2 with 64 lanes (table-decoded exponents, flat 3-bit sign+mantissa code) */
    uint32_t fast_exp_kind, fast_sm_kind, n_rings /* kernels 3, 5: slots per workgroup */, xor_delta;
    uint32_t scattered;                         /* some tensor decodes an id list */
    uint32_t tail_kernel;                       /* the second work list (chunks that are not whole rows, id lists with 64 lanes):
                                                   0 generic kernel, 1 the 64-lane kernel's build for such chunks (two-field formats),
                                                   2 = 1 leaving whole chunks to the FP8 kernel's build for id lists */
    uint64_t fast_work_offset, work_offset;     /* byte offsets of the two work lists in d_ws */
} zc_batch_plan;
zc_status zc_decompress_batch_plan(const zc_tensor *tensors, uint32_t n_tensors, void *d_ws, uint64_t ws_bytes,
                                   zc_batch_plan *plan, void *stream);
zc_status zc_decompress_batch_run(const zc_batch_plan *plan, const void *d_ws, void *stream);

/* Per-field histogram, entropy, code lengths, payload bits, stream and container bytes
 * and the ratios of Sec. 4, without producing the container.  out: host.  Synchronises. */
zc_status zc_stats(const void *d_src, uint64_t n_elems, const zc_params *params,
                   const void *d_xor_base, const void *d_scales, zc_stats_out *out,
                   void *d_ws, uint64_t ws_bytes, void *stream);

/* Measurement aid, not part of the method: a plain copy of `bytes` bytes (a multiple of 16) from d_src to d_dst
 * (device, 16-byte aligned, not overlapping), 16 bytes per lane.  chunk_bytes == 0: linear through memory, the
 * best this machine gives a kernel that only moves bytes.  chunk_bytes != 0 (a multiple of 1024 that divides
 * `bytes`): one wavefront per chunk of that size, each walking through its own chunk 1 KiB at a time, which is how
 * the 64-lane decoders and encoders touch memory: the ceiling of that access pattern.  Queued on the stream, never
 * waits.  Benchmarks report the codec's traffic next to these, and counter runs use the linear copy as the kernel
 * of known traffic. */
zc_status zc_copy_reference(const void *d_src, void *d_dst, uint64_t bytes, uint32_t chunk_bytes, void *stream);

/* Length-limited canonical Huffman code for one histogram (host only; exposed so that the
 * code construction can be checked without a GPU).  hist: `alphabet` counts;
 * len_out/code_out: `alphabet` entries.  Returns ZC_ERR_INVALID_ARG if 2^limit < number of
 * used symbols.  A single used symbol gets length 1. */
zc_status zc_build_code(const uint64_t *hist, uint32_t alphabet, uint32_t limit,
                        uint8_t *len_out, uint16_t *code_out);

const char *zc_status_string(zc_status s);

#ifdef __cplusplus
}
#endif
#endif /* ZC_H */
