// The 64-lane decoders for whole chunks of any format (k_decode_s64), and the kernels cut down for BF16 and for FP8 E5M2.
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_decode_device.h"

namespace zc {

// split: the workgroup's four wavefronts share ONE chunk, each taking a quarter of its rows (the first also the
// block scales).  Only for chunks whose element fields are both stored plainly (flat code, raw or constant):
// their rows do not depend on each other, and four times the wavefronts hide four times the memory latency,
// which is what a small set (few chunks per SIMD) is bound by.
//
// TAIL: the launch is over chunks that need not be whole rows: the short last chunk of a tensor, every chunk of a
// tensor whose chunk size is not a multiple of 1 KiB, or the chunks a list of ids names (which may include either).
// Their whole rows are decoded as above; the row after them, in which a lane owns a whole run, part of one or
// nothing, takes its stream words by the same rule with the lanes that own nothing left out, and is stored byte by
// byte where a run is cut.  Formats with two fields only.  skip_whole: leave whole chunks to the kernel that has them.
template <int FMT, bool XOR, bool SPLIT, bool TAIL>
__global__ __launch_bounds__(256) void k_decode_s64(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single, uint32_t first_slot,
                                                    uint32_t skip_whole)
{
    constexpr bool split = SPLIT;
    using F_ = Fmt<FMT>;
    static_assert(!TAIL || (F_::NF == 2 && !SPLIT), "the tail build has no scale field and no shared chunks");
    extern __shared__ __attribute__((aligned(16))) uint32_t rings[];     // [ring][wave][kRing2Words], sized by the host
    __shared__ FieldTab tab[F_::NF];
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = first_slot + blockIdx.x * (split ? 1u : kWavesPerGroup); }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    uint32_t kind[F_::NF];
    for (int f = 0; f < F_::NF; f++) {
        kind[f] = uniform32(d.kind[f]);
        if (kind[f] == KIND_HUFF && !(SPLIT && f < 2)) build_field_tab(tab[f], d.comp + d.table_off[f], 1 << (f == 2 ? 8 : F_::SB), d.lmax[f]);
    }
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t slot = uniform32(it.first + (split ? 0u : wave));
    uint32_t chunk = slot;
    if (TAIL) {
        // a list of chunk ids: slot i of the output takes chunk ids[i]; an id out of range leaves its slot alone
        const uint32_t *ids = reinterpret_cast<const uint32_t *>(uniform64((uint64_t)d.ids));
        if (ids) {
            if (slot >= uniform32(d.n_ids)) return;
            chunk = uniform32(ids[slot]);
        }
    }
    const uint32_t cb = uniform32(d.chunk_bytes);
    const uint32_t E = cb * 8 / F_::EB;
    const uint64_t n_elems = uniform64(d.n_elems);
    const uint32_t n_full = (uint32_t)(n_elems / E);
    if (TAIL ? chunk >= uniform32(d.n_chunks) : chunk >= n_full) return;
    if (TAIL && skip_whole && chunk < n_full && cb % 1024 == 0) return;        // a specialised kernel took the whole chunks of this launch
    // this chunk's elements and bytes: all of cb unless it is the tensor's short last chunk
    const uint64_t before = (uint64_t)chunk * E;
    const uint32_t n = (!TAIL || n_elems - before >= E) ? E : (uint32_t)(n_elems - before);
    const uint32_t nbytes = n * F_::EB / 8;                   // two-field formats have whole bytes per element
    if (TAIL && n_elems <= before) return;
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    const uint8_t *sp[F_::NF];
    uint32_t sb[F_::NF];
    for (int f = 0; f < F_::NF; f++)
        if (!stream_range(d, comp, f, chunk, payload, total, sp[f], sb[f])) return;      // damaged index: leave the chunk alone
    const __amdgpu_buffer_rsrc_t r0 = make_rsrc(sp[0], sb[0]), r1 = make_rsrc(sp[1], sb[1]);
    uint8_t *const dst_chunk = reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)) + (uint64_t)slot * cb;       // slot == chunk without an id list
    const uint8_t *const base_chunk = XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) + (uint64_t)chunk * cb : comp;
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(dst_chunk, nbytes);
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(base_chunk, XOR ? nbytes : 0);
    // the row after the whole rows: symbols of this lane's run in it (0 in every lane when the chunk is whole rows)
    const uint32_t whole_rows = nbytes / 1024;
    uint32_t tail_sym = 0, tail_bytes = 0;
    if (TAIL) {
        const uint32_t at = whole_rows * 1024 + lane * 16;
        tail_bytes = nbytes > at ? (nbytes - at < 16u ? nbytes - at : 16u) : 0u;
        tail_sym = (tail_bytes * 8 / F_::EB + F_::GRP - 1) / F_::GRP;         // a last partial group of values is one symbol
    }
    const uint32_t p0 = uniform32(d.period[0]), p1 = uniform32(d.period[1]);
    const uint64_t K0 = splat(uniform32(d.konst[0]), F_::SB), K1 = splat(uniform32(d.konst[1]), F_::SB);

    // rings: the workgroup has 8 KiB.  One table-decoded element field: 512 words per wavefront; two: 256 words per
    // wavefront and field, field 0's in the first half.  The scale field, decoded after the elements, takes over the
    // wavefront's first ring as it is (the other wavefronts may still be using theirs).
    const bool two = kind[0] == KIND_HUFF && kind[1] == KIND_HUFF;
    const uint32_t rw = two ? 256u : kRing2Words;
    char *ring0 = reinterpret_cast<char *>(rings) + wave * (rw * 4), *ring1 = ring0 + (two ? kWavesPerGroup * 256 * 4 : 0);
    HuffStream H0, H1;
    const bool first = !TAIL || whole_rows > 0 || tail_sym > 0;                  // does this lane own a symbol at step 0?
    if (!SPLIT && kind[0] == KIND_HUFF) huff_open(H0, tab[0], r0, ring0, lane, rw, first);
    if (!SPLIT && kind[1] == KIND_HUFF) huff_open(H1, tab[1], r1, ring1, lane, rw, first);

    const uint32_t rows = TAIL ? whole_rows : cb / 1024;      // 64 lanes x 16 bytes per row
    if (split && (kind[0] == KIND_HUFF || kind[1] == KIND_HUFF)) return;          // the host never asks for this
    uint32_t row_begin = 0, row_end = rows;
    if (split) shared_chunk_rows(rows, F_::NF == 3 ? E / F_::SCALE / 1024 : 0u, wave, row_begin, row_end);
    // what a row takes from global memory besides its stream words (plainly stored fields, the base of a delta) is asked
    // for one row ahead
    constexpr int WPR = F_::G * F_::SB / 32;
    uint32_t w0_next[WPR] = {}, w1_next[WPR] = {};
    u32x4 base_next = {0, 0, 0, 0};
    if (row_begin < row_end) {
        if (SPLIT || kind[0] != KIND_HUFF) plain_fetch<F_::SB, F_::G>(kind[0], r0, row_begin, lane, w0_next);
        if (SPLIT || kind[1] != KIND_HUFF) plain_fetch<F_::SB, F_::G>(kind[1], r1, row_begin, lane, w1_next);
        if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), (int)(row_begin * 1024), 0);
    }
    for (uint32_t row = row_begin; row < row_end; row++) {
        uint64_t P0 = 0, P1 = 0, Q0 = 0, Q1 = 0;       // Q: symbols 8..15 of a run of 16 symbols of 8 bits
        uint32_t w0[WPR], w1[WPR];
#pragma unroll
        for (int h = 0; h < WPR; h++) { w0[h] = w0_next[h]; w1[h] = w1_next[h]; }
        const u32x4 base = base_next;
        if (SPLIT || kind[0] != KIND_HUFF) plain_fetch<F_::SB, F_::G>(kind[0], r0, row + 1, lane, w0_next);
        if (SPLIT || kind[1] != KIND_HUFF) plain_fetch<F_::SB, F_::G>(kind[1], r1, row + 1, lane, w1_next);
        // (the scalar offset of a buffer access is not range checked: the row after the last is the last again)
        if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), (int)((row + 1 < rows ? row + 1 : row) * 1024), 0);
        // the words a lane takes at the end of a row are for its next run: after the last whole row, the tail's
        const uint32_t next_sym = (TAIL && row + 1 == rows) ? tail_sym : (uint32_t)F_::G;
        if (!SPLIT && kind[0] == KIND_HUFF) huff_run<F_::SB, F_::G>(H0, tab[0], p0, P0, Q0, lane, F_::G, next_sym);
        else plain_finish<F_::SB, F_::G>(kind[0], w0, K0, P0, Q0);
        if (!SPLIT && kind[1] == KIND_HUFF) huff_run<F_::SB, F_::G>(H1, tab[1], p1, P1, Q1, lane, F_::G, next_sym);
        else plain_finish<F_::SB, F_::G>(kind[1], w1, K1, P1, Q1);
        const uint4 j = join_run4<FMT>(P0, Q0, P1, Q1);
        u32x4 v = {j.x, j.y, j.z, j.w};
        if (XOR) v ^= base;
        // (a whole row of the output, written once: stored with the non-temporal hint so that it does not displace the streams' lines in the L2)
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 2);
    }
    if (TAIL && nbytes % 1024) {
        uint64_t P0 = 0, P1 = 0, Q0 = 0, Q1 = 0;
        if (kind[0] == KIND_HUFF) huff_run<F_::SB, F_::G>(H0, tab[0], p0, P0, Q0, lane, tail_sym, 0u);
        else plain_tail<F_::SB, F_::G>(kind[0], r0, whole_rows, lane, tail_sym, K0, P0, Q0);
        if (kind[1] == KIND_HUFF) huff_run<F_::SB, F_::G>(H1, tab[1], p1, P1, Q1, lane, tail_sym, 0u);
        else plain_tail<F_::SB, F_::G>(kind[1], r1, whole_rows, lane, tail_sym, K1, P1, Q1);
        if (tail_bytes) {
            const uint32_t at = whole_rows * 1024 + lane * 16;
            uint4 v = join_run4<FMT>(P0, Q0, P1, Q1);
            if (XOR) v = xor4(v, load_run(base_chunk + at, tail_bytes));
            store_run(dst_chunk + at, v, tail_bytes);
        }
    }

    if (F_::NF == 3 && !(split && wave != 0)) {
        // block scales: one byte per 32 elements, 16 per run, the chunk's E/32 scales in rows of 1024
        constexpr int F2 = F_::NF - 1;
        const uint32_t n_sc = E / F_::SCALE;
        const __amdgpu_buffer_rsrc_t r2 = make_rsrc(sp[F2], sb[F2]);
        const __amdgpu_buffer_rsrc_t ss = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.scales_out)) + (uint64_t)chunk * n_sc, n_sc);
        const uint32_t p2 = uniform32(d.period[F2]);
        const uint64_t K2 = splat(uniform32(d.konst[F2]), 8);
        HuffStream H2;
        if (kind[F2] == KIND_HUFF) huff_open(H2, tab[F2], r2, ring0, lane, rw);      // this wavefront's first element ring is free again
        for (uint32_t row = 0; row < n_sc / 1024; row++) {
            uint64_t P0 = 0, P1 = 0;
            if (kind[F2] == KIND_HUFF) huff_run<8, 16>(H2, tab[F2], p2, P0, P1, lane);
            else plain_run<8, 16>(kind[F2], r2, row, lane, K2, P0, P1);
            const u32x4 v = {(uint32_t)P0, (uint32_t)(P0 >> 32), (uint32_t)P1, (uint32_t)(P1 >> 32)};
            __builtin_amdgcn_raw_buffer_store_b128(v, ss, (int)(lane * 16), (int)(row * 1024), 0);
        }
    }
}

template <int FMT>
static int launch_s64_x(bool xor_delta, int split, uint32_t lds_bytes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single, hipStream_t st)
{
    if (split) {
        if (xor_delta) hipLaunchKernelGGL((k_decode_s64<FMT, true, true, false>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, 0u, 0u);
        else hipLaunchKernelGGL((k_decode_s64<FMT, false, true, false>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, 0u, 0u);
    } else {
        if (xor_delta) hipLaunchKernelGGL((k_decode_s64<FMT, true, false, false>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, 0u, 0u);
        else hipLaunchKernelGGL((k_decode_s64<FMT, false, false, false>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, 0u, 0u);
    }
    return (int)hipGetLastError();
}

template <int FMT>
static int launch_s64_tail_x(bool xor_delta, uint32_t lds_bytes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single,
                             uint32_t first_slot, uint32_t skip_whole, hipStream_t st)
{
    if (xor_delta) hipLaunchKernelGGL((k_decode_s64<FMT, true, false, true>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, first_slot, skip_whole);
    else hipLaunchKernelGGL((k_decode_s64<FMT, false, false, true>), dim3(n_work), dim3(256), lds_bytes, st, d_descs, d_work, s, use_single, first_slot, skip_whole);
    return (int)hipGetLastError();
}

// n_rings: 1 or 2 rings per wavefront (2 only when both element fields are table decoded); split: one chunk per
// work item, its rows shared by the four wavefronts (both element fields stored plainly)
int launch_decode_s64(uint32_t fmt, uint32_t n_rings, bool xor_delta, bool split, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                      const TensorDev *single, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    // the rings of a workgroup take 8 KiB whether one or two fields are table decoded (see huff_open)
    (void)n_rings;
    const uint32_t lds = kWavesPerGroup * kRing2Words * 4;
    switch (fmt) {
    case ZC_FMT_BF16: return launch_s64_x<ZC_FMT_BF16>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP8_E4M3: return launch_s64_x<ZC_FMT_FP8_E4M3>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP4_E2M1_MX: return launch_s64_x<ZC_FMT_FP4_E2M1_MX>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP8_E4M3_BYTES: return launch_s64_x<ZC_FMT_FP8_E4M3_BYTES>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP4_E2M1_MX_BYTES: return launch_s64_x<ZC_FMT_FP4_E2M1_MX_BYTES>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP4_E2M1_NV: return launch_s64_x<ZC_FMT_FP4_E2M1_NV>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    case ZC_FMT_FP8_E5M2: return launch_s64_x<ZC_FMT_FP8_E5M2>(xor_delta, split ? 1 : 0, lds, d_descs, d_work, n_work, s, use_single, st);
    default: return 1;
    }
}

// The tail build over work items of up to four chunks each (64 lanes, two-field formats), chunks that need not be whole
// rows.  single: one tensor, work items from chunk first_slot on.  skip_whole: leave whole chunks alone (a specialised
// kernel with an id list has taken them; only what it leaves, a short last chunk, is decoded here).
int launch_decode_s64_tail(uint32_t fmt, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev *single,
                           uint32_t first_slot, bool skip_whole, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    const uint32_t lds = kWavesPerGroup * kRing2Words * 4;
    switch (fmt) {
    case ZC_FMT_BF16: return launch_s64_tail_x<ZC_FMT_BF16>(xor_delta, lds, d_descs, d_work, n_work, s, use_single, first_slot, skip_whole ? 1u : 0u, st);
    case ZC_FMT_FP8_E4M3: return launch_s64_tail_x<ZC_FMT_FP8_E4M3>(xor_delta, lds, d_descs, d_work, n_work, s, use_single, first_slot, skip_whole ? 1u : 0u, st);
    case ZC_FMT_FP8_E4M3_BYTES: return launch_s64_tail_x<ZC_FMT_FP8_E4M3_BYTES>(xor_delta, lds, d_descs, d_work, n_work, s, use_single, first_slot, skip_whole ? 1u : 0u, st);
    case ZC_FMT_FP8_E5M2: return launch_s64_tail_x<ZC_FMT_FP8_E5M2>(xor_delta, lds, d_descs, d_work, n_work, s, use_single, first_slot, skip_whole ? 1u : 0u, st);
    default: return 1;
    }
}

// ---------------------------------------------------------------------------------------
// BF16 with 64 lanes per chunk and whole chunks, exponent field table decoded and the sign+mantissa field either
// table decoded on the same refill period (checkpoint deltas, Sec. 3.1 / 4.1) or stored plainly (weights): the
// same streams and rings as above with the per-symbol work cut down for this format.
//   - Table entries are laid out so that a value is assembled without shifting fields around: an exponent entry is
//     (e << 7) | length, a sign+mantissa entry (s << 15) | (length << 8) | mantissa.  Two entries packed into one
//     register are the two halves of an output word, and one bit-field insert with the exponent mask 0x7F80 per
//     half merges the fields; the lengths sit in bits the insert drops.
//   - With two symbols per refill step the lookups index from the window shifted left by one (entries are 2 bytes),
//     so a lookup is an AND and a load; a step's lengths are added to the bit position with one three-operand add.
constexpr uint32_t kExpMask2 = 0x7F807F80u;            // the exponent bits of both halves of an output word

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }   // v_bfi_b32

// shift amount taken from byte 1 of `by` (the hardware uses its low 5 bits)
__device__ __forceinline__ uint32_t shr_by_byte1(uint32_t v, uint32_t by)
{
    uint32_t r;
    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(r) : "v"(by), "v"(v));
    return r;
}
__device__ __forceinline__ uint32_t add_byte1(uint32_t a, uint32_t b)      // a + byte 1 of b
{
    uint32_t r;
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// FieldTab::lut entries (length | symbol << 8) rewritten for this path, in place; 0 (a code longer than the index) stays 0
template <int FIELD>
__device__ __forceinline__ uint32_t bf16_entry(uint32_t e)
{
    const uint32_t len = e & 31u, sym = e >> 8;
    if (FIELD == 0) return (sym << 7) | len;
    return ((sym & 0x80u) << 8) | (len << 8) | (sym & 0x7Fu);
}
template <int FIELD>
__device__ void bf16_relayout(FieldTab &T)
{
    const uint32_t n = T.mask + 1;
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) T.lut[i] = (uint16_t)bf16_entry<FIELD>(T.lut[i]);
    __syncthreads();
}

// The stream ring of huff_open / huff_ring_service / huff_refill with its size as a parameter: RW words per wavefront
// and field, refilled SEG = RW / 4 words at a time (SEG / 64 words per lane).  A segment that has been asked for is
// written into the ring only when the next one is asked for, i.e. once a whole segment has been consumed since:
// that is the time its load has to arrive.  Invariant when ring_service is called: words [wbase, wbase + RW) are in
// the ring except the newest SEG, which may still be in flight or in registers; wpos - wbase < 2 * SEG, and at
// most SEG words are handed out before the next call, so every word asked for is below wbase + 3 * SEG: present.
template <uint32_t RW>
__device__ __forceinline__ void ring_open(HuffStream &H, const FieldTab &T, __amdgpu_buffer_rsrc_t rs, char *ring, uint32_t lane)
{
    constexpr uint32_t SEG = RW / 4, B = SEG / 16;       // bytes per lane and segment: 4 or 8
    static_assert(B == 4 || B == 8, "one 4- or 8-byte load per lane and segment");
    H.rs = rs; H.ring = ring;
#pragma unroll
    for (int i = 0; i < 4; i++) H.lim[i] = uniform32(T.limit[kLutBits + 1 + i]);
#pragma unroll
    for (uint32_t q = 0; q < 4; q++) {
        if (B == 8) *reinterpret_cast<u32x2 *>(ring + q * SEG * 4 + lane * 8) = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(lane * 8 + q * SEG * 4), 0, 0);
        else *reinterpret_cast<uint32_t *>(ring + q * SEG * 4 + lane * 4) = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(lane * 4 + q * SEG * 4), 0, 0);
    }
    H.W = (uint64_t)(*reinterpret_cast<const uint32_t *>(ring + lane * 4)) << 32;   // step 0: word `lane`
    H.c = 32; H.wpos = 64; H.wbase = 0; H.pslot = 0; H.pending = false;
    H.pv = u32x2{0, 0};
}

template <uint32_t RW>
__device__ __forceinline__ void ring_service(HuffStream &H, uint32_t lane)
{
    constexpr uint32_t SEG = RW / 4, B = SEG / 16;
    if (H.wpos - H.wbase >= SEG) {                       // the oldest segment is used up: its place takes the segment after the newest
        if (H.pending) {
            if (B == 8) *reinterpret_cast<u32x2 *>(H.ring + H.pslot * 4 + lane * 8) = H.pv;
            else *reinterpret_cast<uint32_t *>(H.ring + H.pslot * 4 + lane * 4) = H.pv.x;
        }
        // the newest segment [wbase + 3 SEG, wbase + 4 SEG) is complete now; the one asked for goes where the oldest was
        if (B == 8) H.pv = __builtin_amdgcn_raw_buffer_load_b64(H.rs, (int)(lane * 8 + (H.wbase + RW) * 4), 0, 0);
        else H.pv.x = __builtin_amdgcn_raw_buffer_load_b32(H.rs, (int)(lane * 4 + (H.wbase + RW) * 4), 0, 0);
        H.pslot = H.wbase & (RW - 1);
        H.wbase += SEG;
        H.pending = true;
    }
}

template <uint32_t RW>
__device__ __forceinline__ void ring_refill(HuffStream &H)
{
    const bool need = H.c >= 32;
    const uint64_t bm = __ballot(need);
    const uint32_t w = *reinterpret_cast<const uint32_t *>(H.ring + ((prefix_count64(bm) * 4 + H.wpos * 4) & (RW * 4 - 1)));
    H.W = need ? ((H.W >> 32) | ((uint64_t)w << 32)) : H.W;
    H.c = need ? H.c - 32 : H.c;
    H.wpos += (uint32_t)__popcll(bm);
}

// One refill period of R symbols of field FIELD: the entries of symbols 2i and 2i+1, packed into out[first / 2 + i].
template <int FIELD, int R, bool LONG, uint32_t RW>
__device__ __forceinline__ void bf16_period(HuffStream &H, const FieldTab &T, const char *lut, uint32_t mask2, int first, uint32_t out[4])
{
    static_assert(!LONG || R == 2, "codes beyond the lookup index come with a refill period of 2 only");
    const uint32_t x = (uint32_t)(H.W >> H.c);             // the next 32 unread bits
    uint32_t e[R];
    if (R == 2) {
        // entries are two bytes: index from the window shifted left once; bits [1..] of (y >> n) are bits [0..] of (x >> n)
        uint32_t y = x << 1;
        e[0] = *reinterpret_cast<const uint16_t *>(lut + (y & mask2));
        y = FIELD == 0 ? y >> (e[0] & 31u) : shr_by_byte1(y, e[0]);
        e[1] = *reinterpret_cast<const uint16_t *>(lut + (y & mask2));
        if (LONG) {
            // an empty entry stands for a code longer than the index; it shifts by nothing, so the entry after it is
            // empty too and the last one tells
            if (__any(e[1] == 0)) {
                uint32_t x1 = x;
                if (e[0] == 0) {
                    e[0] = bf16_entry<FIELD>(long_code(T, H, x));
                    x1 = FIELD == 0 ? x >> (e[0] & 31u) : shr_by_byte1(x, e[0]);
                    e[1] = *reinterpret_cast<const uint16_t *>(lut + ((x1 << 1) & mask2));
                } else x1 = FIELD == 0 ? x >> (e[0] & 31u) : shr_by_byte1(x, e[0]);
                if (e[1] == 0) e[1] = bf16_entry<FIELD>(long_code(T, H, x1));
            }
        }
    } else {
        uint32_t xx = x;
#pragma unroll
        for (int j = 0; j < R; j++) {
            e[j] = *reinterpret_cast<const uint16_t *>(lut + ((xx << 1) & mask2));
            xx = FIELD == 0 ? xx >> (e[j] & 31u) : shr_by_byte1(xx, e[j]);
        }
    }
    // the lengths: bits 4..0 of an exponent entry (the exponents above them leave the low 7 bits of a sum alone),
    // byte 1 of a sign+mantissa entry (the sign above the length leaves the low 7 bits of a sum alone); a period's
    // lengths add up to 32 at most and c was 32 at most
    uint32_t c = H.c;
#pragma unroll
    for (int j = 0; j < R; j += 2) {
        if (FIELD == 0) c = c + e[j] + e[j + 1];
        else c = add_byte1(add_byte1(c, e[j]), e[j + 1]);
        out[(first + j) / 2] = __builtin_amdgcn_perm(e[j + 1], e[j], 0x05040100u);       // low halves of both
    }
    H.c = c & 0x7Fu;
    ring_refill<RW>(H);
}

// The rows of one chunk.  R: refill period of the exponent field (and of the sign+mantissa field when PAIR).
// PAIR: the sign+mantissa field is table decoded on the same period; else it is flat coded, raw or constant.
template <int R, bool LONG, bool PAIR, bool XOR>
__device__ __forceinline__ void bf16_rows(const FieldTab *tab, uint32_t kind1, uint32_t konst1, __amdgpu_buffer_rsrc_t r0, __amdgpu_buffer_rsrc_t r1,
                                          __amdgpu_buffer_rsrc_t ds, __amdgpu_buffer_rsrc_t bs, char *ring0, char *ring1, uint32_t rows, uint32_t lane)
{
    // two table-decoded fields: rings of 256 words, serviced at every refill step, so that eight workgroups fit a
    // compute unit's LDS; one field: 512 words, serviced every other step
    constexpr uint32_t RW = PAIR ? 256u : 512u;
    HuffStream A, B;
    ring_open<RW>(A, tab[0], r0, ring0, lane);
    if (PAIR) ring_open<RW>(B, tab[1], r1, ring1, lane);
    const char *la = reinterpret_cast<const char *>(tab[0].lut), *lb = reinterpret_cast<const char *>(tab[1].lut);
    const uint32_t ma2 = uniform32(tab[0].mask) << 1, mb2 = PAIR ? uniform32(tab[1].mask) << 1 : 0u;
    const uint32_t k1 = konst1 | (konst1 << 8) | (konst1 << 16) | (konst1 << 24);
    // What a row takes from global memory besides its stream words (plain sign+mantissa bytes, the base of a delta)
    // is asked for one row ahead, so that the loads are in flight while the row before is decoded.  Row offsets go
    // into the scalar operand of the loads, which the hardware does not range check, so they never leave the chunk.
    auto fetch_m = [&](uint32_t row, uint32_t m[2]) {
        m[0] = k1; m[1] = k1;
        if (kind1 == KIND_FLAT) {
#pragma unroll
            for (int h = 0; h < 2; h++) m[h] = __builtin_amdgcn_raw_buffer_load_b32(r1, (int)(lane * 4), (int)((row * 2 + h) * 256), 0);
        } else if (kind1 == KIND_RAW) {
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r1, (int)(lane * 8), (int)(row * 512), 0);
            m[0] = v.x; m[1] = v.y;
        }
    };
    uint32_t m_next[2] = {0, 0};
    u32x4 base_next = {0, 0, 0, 0};
    if (!PAIR) fetch_m(0, m_next);
    if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), 0, 0);
    for (uint32_t row = 0; row < rows; row++) {
        uint32_t ea[4], mb[4];
        const uint32_t m[2] = {m_next[0], m_next[1]};
        const u32x4 base = base_next;
        const uint32_t ahead = row + 1 < rows ? row + 1 : row;      // the row after the last is the last again
        if (!PAIR) fetch_m(ahead, m_next);
        if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), (int)(ahead * 1024), 0);
#pragma unroll
        for (int g = 0; g < 8 / R; g++) {
            if (PAIR || (g & 1) == 0) { ring_service<RW>(A, lane); if (PAIR) ring_service<RW>(B, lane); }
            bf16_period<0, R, LONG, RW>(A, tab[0], la, ma2, g * R, ea);
            if (PAIR) bf16_period<1, R, LONG, RW>(B, tab[1], lb, mb2, g * R, mb);
        }
        if (!PAIR) {
            // eight sign+mantissa bytes of the lane (a flat code is the byte, most significant bit first), then two per
            // output word: byte b -> (s << 15) | ... | m (bits 14..7 are dropped by the insert)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t mm = kind1 == KIND_FLAT ? reverse_in_groups<8>(m[i / 2]) : m[i / 2];
                const uint32_t t = __builtin_amdgcn_perm(0, mm, (i & 1) ? 0x0C030C02u : 0x0C010C00u);      // bytes 2i, 2i+1 into bytes 0 and 2
                mb[i] = t | (t << 8);
            }
        }
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; i++) v[i] = bfi(kExpMask2, ea[i], mb[i]);
        if (XOR) v ^= base;
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 2);
    }
}


// One wavefront per whole chunk, four chunks per workgroup, as k_decode_s64; the host sends a set of tensors here
// only when every one of them has the shape bf16_rows is written for.
template <bool XOR>
__global__ __launch_bounds__(256) void k_decode_bf16_s64(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t rings[];     // [ring][wave][kRing2Words], sized by the host
    __shared__ FieldTab tab[2];
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = blockIdx.x * kWavesPerGroup; }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    const uint32_t kind0 = uniform32(d.kind[0]), kind1 = uniform32(d.kind[1]);
    const uint32_t p0 = uniform32(d.period[0]), p1 = uniform32(d.period[1]);
    const bool pair = kind1 == KIND_HUFF;
    if (kind0 != KIND_HUFF || (p0 != 2 && p0 != 4 && p0 != 8) || (pair && p1 != p0)) return;       // whole workgroup; the host never asks for this
    build_field_tab(tab[0], d.comp + d.table_off[0], 256, d.lmax[0]);
    bf16_relayout<0>(tab[0]);
    if (pair) {
        build_field_tab(tab[1], d.comp + d.table_off[1], 256, d.lmax[1]);
        bf16_relayout<1>(tab[1]);
    }
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t chunk = uniform32(it.first + wave);
    const uint32_t cb = uniform32(d.chunk_bytes);
    const uint32_t n_full = (uint32_t)(uniform64(d.n_elems) / (cb / 2));
    if (chunk >= n_full) return;
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    const uint8_t *sp[2];
    uint32_t sb[2];
    for (int f = 0; f < 2; f++)
        if (!stream_range(d, comp, f, chunk, payload, total, sp[f], sb[f])) return;      // damaged index: leave the chunk alone
    // a plainly stored sign+mantissa field takes a byte per value; its rows are addressed through the scalar offset,
    // which is not range checked, so a stream shorter than that (a damaged index) must not be read at all
    if ((kind1 == KIND_FLAT || kind1 == KIND_RAW) && sb[1] < cb / 2) return;
    const __amdgpu_buffer_rsrc_t r0 = make_rsrc(sp[0], sb[0]), r1 = make_rsrc(sp[1], sb[1]);
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)) + (uint64_t)chunk * cb, cb);
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) + (uint64_t)chunk * cb : comp, XOR ? cb : 0);
    // one field: 512 words per wavefront; two: 256 words per wavefront and field (the same 8 KiB per workgroup)
    char *ring0 = reinterpret_cast<char *>(rings) + wave * (pair ? 1024 : 2048), *ring1 = ring0 + kWavesPerGroup * 1024;
    const uint32_t rows = cb / 1024, konst1 = uniform32(d.konst[1]);
    const bool any_long = uniform32(tab[0].lmax) > (uint32_t)kLutBits || (pair && uniform32(tab[1].lmax) > (uint32_t)kLutBits);
    switch (p0 * 4 + (pair ? 2 : 0) + ((any_long && p0 == 2) ? 1 : 0)) {
    case 2 * 4 + 0: bf16_rows<2, false, false, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 2 * 4 + 1: bf16_rows<2, true, false, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 2 * 4 + 2: bf16_rows<2, false, true, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 2 * 4 + 3: bf16_rows<2, true, true, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 4 * 4 + 0: bf16_rows<4, false, false, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 4 * 4 + 2: bf16_rows<4, false, true, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    case 8 * 4 + 0: bf16_rows<8, false, false, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    default: bf16_rows<8, false, true, XOR>(tab, kind1, konst1, r0, r1, ds, bs, ring0, ring1, rows, lane); break;
    }
}

// n_rings: 1, or 2 when some tensor's sign+mantissa field is table decoded too
int launch_decode_bf16_s64(uint32_t n_rings, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev *single, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    const uint32_t lds = kWavesPerGroup * 2048;
    (void)n_rings;
    if (xor_delta) hipLaunchKernelGGL((k_decode_bf16_s64<true>), dim3(n_work), dim3(256), lds, st, d_descs, d_work, s, use_single);
    else hipLaunchKernelGGL((k_decode_bf16_s64<false>), dim3(n_work), dim3(256), lds, st, d_descs, d_work, s, use_single);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// FP8 E5M2 (s eeeee mm) with 64 lanes per chunk and whole chunks, in the shape weights take: the exponent field
// table decoded (16 symbols per run), the sign+mantissa field coded with the flat 3-bit code that its eight nearly
// equally likely values get (lengths 3 for the values 0..7, nothing else in the table).  The exponent stream goes
// through the ring and huff_run_r as in k_decode_s64, with table entries that hold the exponent at its place in the
// output byte.  The sign+mantissa stream needs no table and no refill logic: every lane takes 24 bits per refill
// step, so all lanes ask for words at the same steps, the stream is rounds of 64 words in lane order, and a lane's
// bits are its words of every round one after the other: a row (16 values, 48 bits) starts at bit 48 * row of
// them.  What a row takes from global memory is asked for one row ahead.

// 32-bit word whose bytes are the next four 3-bit codes of v (first code in bits 2..0): a code is s, m1, m0 with the
// sign first in stream order, a byte of the result is s << 7 | m1 << 1 | m0
__device__ __forceinline__ uint32_t e5m2_sm_bytes(uint32_t v)
{
    const uint32_t a = (v & 0x7u) | ((v & 0x38u) << 5) | ((v & 0x1C0u) << 10) | ((v & 0xE00u) << 15);      // one code per byte
    return ((a << 7) & 0x80808080u) | (a & 0x02020202u) | ((a >> 2) & 0x01010101u);
}

template <int R, bool LONG, bool XOR>
__device__ __forceinline__ void e5m2_rows(const FieldTab &T, __amdgpu_buffer_rsrc_t r0, __amdgpu_buffer_rsrc_t r1, __amdgpu_buffer_rsrc_t ds,
                                          __amdgpu_buffer_rsrc_t bs, char *ring, uint32_t rows, uint32_t lane)
{
    HuffStream H;
    huff_open(H, T, r0, ring, lane);
    // sign+mantissa words of the lane: word q of the lane is word 64 * q + lane of the stream; two rows take three
    auto fetch_sm = [&](uint32_t pair, uint32_t w[3]) {
#pragma unroll
        for (int k = 0; k < 3; k++) w[k] = __builtin_amdgcn_raw_buffer_load_b32(r1, (int)(lane * 4 + (pair * 3 + k) * 256), 0, 0);   // range checked
    };
    uint32_t sm_next[3];
    u32x4 base_next = {0, 0, 0, 0};
    fetch_sm(0, sm_next);
    if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), 0, 0);
    uint32_t sm[3] = {0, 0, 0};
    for (uint32_t row = 0; row < rows; row++) {
        if ((row & 1) == 0) {
            sm[0] = sm_next[0]; sm[1] = sm_next[1]; sm[2] = sm_next[2];
            fetch_sm(row / 2 + 1, sm_next);                     // past the stream's end the loads return zeros (checked offsets)
        }
        const u32x4 base = base_next;
        // (the scalar offset of a buffer access is not range checked: the row after the last is the last again)
        if (XOR) base_next = __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), (int)((row + 1 < rows ? row + 1 : row) * 1024), 0);
        uint64_t P = 0, Q = 0;
        huff_run_r<8, 16, R, LONG>(H, T, P, Q, lane);          // bytes: exponent << 2
        // the row's 48 sign+mantissa bits: an even row starts at bit 0 of the pair's three words, an odd one at bit 48
        const uint32_t lo = (row & 1) ? __builtin_amdgcn_alignbit(sm[2], sm[1], 16) : sm[0];
        const uint32_t hi = (row & 1) ? sm[2] >> 16 : sm[1];
        u32x4 v;
        v[0] = e5m2_sm_bytes(lo) | (uint32_t)P;
        v[1] = e5m2_sm_bytes(lo >> 12) | (uint32_t)(P >> 32);
        v[2] = e5m2_sm_bytes(__builtin_amdgcn_alignbit(hi, lo, 24)) | (uint32_t)Q;
        v[3] = e5m2_sm_bytes(hi >> 4) | (uint32_t)(Q >> 32);
        if (XOR) v ^= base;
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 2);
    }
}

template <bool XOR>
__global__ __launch_bounds__(256) void k_decode_e5m2(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single)
{
    __shared__ __attribute__((aligned(16))) uint32_t rings[kWavesPerGroup * kRing2Words];
    __shared__ FieldTab tab;
    __shared__ TensorDev dsh;
    __shared__ uint32_t flat3;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = blockIdx.x * kWavesPerGroup; }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) { dsh = use_single ? single : descs[it.tensor]; flat3 = 1; }
    __syncthreads();
    const TensorDev &d = dsh;
    const uint32_t p0 = uniform32(d.period[0]);
    // the sign+mantissa table must be the flat 3-bit code
    if (d.comp[d.table_off[1] + threadIdx.x] != (threadIdx.x < 8 ? 3 : 0)) flat3 = 0;
    build_field_tab(tab, d.comp + d.table_off[0], 256, d.lmax[0]);
    if (uniform32(d.kind[0]) != KIND_HUFF || uniform32(d.mode[1]) != ZC_MODE_HUFF || !flat3 || (p0 != 2 && p0 != 4 && p0 != 8)) return;      // whole workgroup; the host never asks for this
    // entries: the symbol byte becomes the exponent at its place in the output byte
    for (uint32_t i = threadIdx.x; i <= tab.mask; i += blockDim.x) { const uint32_t e = tab.lut[i]; tab.lut[i] = (uint16_t)((e & 0xFFu) | ((e >> 8) << 10)); }
    if (threadIdx.x < 32) tab.sorted[threadIdx.x] = (uint8_t)(tab.sorted[threadIdx.x] << 2);       // what a code beyond the index resolves to (at most 32 exponents are coded)
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t chunk = uniform32(it.first + wave);
    const uint32_t cb = uniform32(d.chunk_bytes);
    const uint32_t n_full = (uint32_t)(uniform64(d.n_elems) / cb);
    if (chunk >= n_full) return;
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    const uint8_t *sp[2];
    uint32_t sb[2];
    for (int f = 0; f < 2; f++)
        if (!stream_range(d, comp, f, chunk, payload, total, sp[f], sb[f])) return;      // damaged index: leave the chunk alone
    if (sb[1] < cb / 8 * 3) return;                         // a flat 3-bit stream of this chunk cannot be shorter
    const __amdgpu_buffer_rsrc_t r0 = make_rsrc(sp[0], sb[0]), r1 = make_rsrc(sp[1], sb[1]);
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)) + (uint64_t)chunk * cb, cb);
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) + (uint64_t)chunk * cb : comp, XOR ? cb : 0);
    char *ring = reinterpret_cast<char *>(rings) + wave * (kRing2Words * 4);
    const uint32_t rows = cb / 1024;
    const bool any_long = uniform32(tab.lmax) > (uint32_t)kLutBits;
    if (p0 == 2 && any_long) e5m2_rows<2, true, XOR>(tab, r0, r1, ds, bs, ring, rows, lane);
    else if (p0 == 2) e5m2_rows<2, false, XOR>(tab, r0, r1, ds, bs, ring, rows, lane);
    else if (p0 == 4) e5m2_rows<4, false, XOR>(tab, r0, r1, ds, bs, ring, rows, lane);
    else e5m2_rows<8, false, XOR>(tab, r0, r1, ds, bs, ring, rows, lane);
}

int launch_decode_e5m2(bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev *single, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    if (xor_delta) hipLaunchKernelGGL((k_decode_e5m2<true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    else hipLaunchKernelGGL((k_decode_e5m2<false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    return (int)hipGetLastError();
}

}  // namespace zc
