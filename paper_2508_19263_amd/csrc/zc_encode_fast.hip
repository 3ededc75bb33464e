// Specialised stream-size and encode kernels for the common FP8 E4M3 container shape:
// 64 lanes per chunk, full chunks, longest exponent code 5..8 bits (refill period 4), sign+mantissa field
// stored raw or with the flat 4-bit code.  Everything else goes through k_encode in
// zc_kernels.hip; both produce the same bytes.
//
// A refill period of 4 symbols is one 32-bit word of source, so a group is handled as two
// exponent pairs: the two exponents of adjacent bytes index a 256-entry table (built on the
// host from the tensor's code) that holds the two codes already concatenated and their total
// length, halving the table lookups and the shift/or work per symbol.
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_encode_device.h"

namespace zc {

// stream sizes of full chunks: per lane only arithmetic on code lengths, no stream positions
__global__ __launch_bounds__(256) void k_sizes_fp8(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables, uint32_t *units)
{
    __shared__ uint32_t pair[256];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (!dp->route) return;                                      // whole workgroup: the code does not suit this kernel
    pair[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + 512 + threadIdx.x];
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = uni32(it.first + (threadIdx.x >> 6));
    const uint32_t E = uni32(dp->chunk_bytes);
    const uint64_t n_elems = uni64(dp->n_elems);
    if (chunk >= (uint32_t)(n_elems / E)) return;
    const bool has_base = uni64((uint64_t)dp->base) != 0;
    const __amdgpu_buffer_rsrc_t src = rsrc_of(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + (uint64_t)chunk * E, E);
    const __amdgpu_buffer_rsrc_t bas = rsrc_of(has_base ? reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + (uint64_t)chunk * E : nullptr, has_base ? E : 0);
    const char *pair_lut = reinterpret_cast<const char *>(pair);
    const uint32_t two = 2;
    int32_t k = 0;              // unread bits the decoder would hold
    uint32_t q = 0;             // words this lane's decoder asks for
    const uint32_t rows = E / 1024;
    for (uint32_t row = 0; row < rows; row++) {
        u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(src, (int)(lane * 16), (int)(row * 1024), 0);
        if (has_base) v ^= __builtin_amdgcn_raw_buffer_load_b128(bas, (int)(lane * 16), (int)(row * 1024), 0);
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const bool req = k <= 32;
            q += req ? 1u : 0u;
            k += req ? 32 : 0;
            uint32_t code, len;
            group_code(v[g], pair_lut, two, code, len);
            k -= (int32_t)len;
        }
    }
    // words of the chunk's exponent stream = sum over the lanes
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
    if (lane == 0) {
        uint32_t *my = units + uni32(dp->units_off);
        const uint32_t nc = uni32(dp->n_chunks);
        my[chunk] = (q + 3) / 4;
        my[nc + chunk] = E / 32;                            // 4 bits per element, 16-byte units (flat code and raw alike)
    }
}

__global__ __launch_bounds__(256) void k_encode_fp8(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables)
{
    constexpr uint32_t kSeg = 256, kRing = 2048;                // words: 16 bytes per lane; 32 words per lane
    __shared__ uint32_t pair[256];
    __shared__ __attribute__((aligned(16))) uint32_t stage[kWavesPerGroup * kRing];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (!dp->route) return;                                      // whole workgroup: the code does not suit this kernel
    pair[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + 512 + threadIdx.x];
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = uni32(it.first + (threadIdx.x >> 6));
    const uint32_t E = uni32(dp->chunk_bytes);
    const uint64_t n_elems = uni64(dp->n_elems);
    if (chunk >= (uint32_t)(n_elems / E)) return;
    const bool has_base = uni64((uint64_t)dp->base) != 0;
    const bool sm_raw = uni32(dp->kind[1]) == 2;
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    const uint64_t payload = uni64(dp->payload_off);
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[0]));
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[1]));
    const uint64_t a0 = uni32(index0[chunk]), b0 = uni32(index0[chunk + 1]), a1 = uni32(index1[chunk]), b1 = uni32(index1[chunk + 1]);
    if (a0 > b0 || a1 > b1 || (b0 - a0) * 16 > 0x7FFFFFFFull || (b1 - a1) * 16 != (uint64_t)E / 2) return;   // index not as the size pass left it
    const __amdgpu_buffer_rsrc_t src = rsrc_of(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + (uint64_t)chunk * E, E);
    const __amdgpu_buffer_rsrc_t bas = rsrc_of(has_base ? reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + (uint64_t)chunk * E : nullptr, has_base ? E : 0);
    const __amdgpu_buffer_rsrc_t es = rsrc_of(comp + payload + 16 * a0, (uint32_t)((b0 - a0) * 16));
    const __amdgpu_buffer_rsrc_t ms = rsrc_of(comp + payload + 16 * a1, E / 2);
    const char *pair_lut = reinterpret_cast<const char *>(pair);
    uint32_t *const ring = stage + (threadIdx.x >> 6) * kRing;
    const uint32_t two = 2;

    // What a lane keeps of its stream.  The decoder it mirrors asks for a word whenever it holds k <= 32 unread
    // bits; the word's position is fixed then, its content is complete later.  Words asked for and not yet
    // written number (k + nacc) / 32: never above 2 (a request needs k <= 32 and nacc < 32).  So one position is
    // due (p0) and at most one more is waiting (p1): a request sets p1, and p0 too when nothing is owed (k == 0:
    // at the start, and after a group that took exactly the 32 bits the decoder held); a write moves p1 to p0.
    uint32_t lo = 0;            // bits not yet written, next free bit = nacc (< 32 between groups)
    uint32_t nacc = 0;
    int32_t k = 0;              // unread bits the decoder would hold at this point
    uint32_t p0 = 0, p1 = 0;
    uint32_t wpos = 0;          // words of the stream handed out so far
    uint32_t flushed = 0;       // words of the stream that have left the ring
    const uint32_t rows = E / 1024;
    // the source (and the base of a delta) is fetched two rows ahead, into two register sets used in turn
    auto fetch = [&](uint32_t row, u32x4 &x, u32x4 &y) {
        row = row < rows ? row : rows - 1;
        x = __builtin_amdgcn_raw_buffer_load_b128(src, (int)(lane * 16), (int)(row * 1024), 0);
        if (has_base) y = __builtin_amdgcn_raw_buffer_load_b128(bas, (int)(lane * 16), (int)(row * 1024), 0);
    };
    auto encode_row = [&](const u32x4 &v, uint32_t row) {
        // ---- sign+mantissa nibbles of the run
        if (sm_raw) {
            // symbol j at bits 4j: nibbles of the even and of the odd bytes of two words, gathered with byte permutes
            uint32_t m[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t x0 = ((v[2 * h] >> 4) & 0x08080808u) | (v[2 * h] & 0x07070707u);
                const uint32_t x1 = ((v[2 * h + 1] >> 4) & 0x08080808u) | (v[2 * h + 1] & 0x07070707u);
                const uint32_t even = __builtin_amdgcn_perm(x1, x0, 0x06040200u), odd = __builtin_amdgcn_perm(x1, x0, 0x07050301u);
                m[h] = even | (odd << 4);
            }
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{m[0], m[1]}, ms, (int)(lane * 8), (int)(row * 512), 0);
        } else {
            // flat code: each symbol most significant bit first, one word per 8 symbols, rows of 64 words.  A bit
            // reversal of the source word puts s, m2, m1, m0 of every byte in this order already (bits 0, 5, 6, 7
            // of the reversed byte) and reverses the bytes, which the permutes undo.
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t r0 = __brev(v[2 * h]), r1 = __brev(v[2 * h + 1]);
                const uint32_t x0 = ((r0 >> 4) & 0x0E0E0E0Eu) | (r0 & 0x01010101u);       // bytes: symbols 3, 2, 1, 0
                const uint32_t x1 = ((r1 >> 4) & 0x0E0E0E0Eu) | (r1 & 0x01010101u);       // bytes: symbols 7, 6, 5, 4
                const uint32_t even = __builtin_amdgcn_perm(x1, x0, 0x05070103u), odd = __builtin_amdgcn_perm(x1, x0, 0x04060002u);
                __builtin_amdgcn_raw_buffer_store_b32(even | (odd << 4), ms, (int)(lane * 4), (int)((row * 2 + h) * 256), 0);
            }
        }
        // ---- exponent: one refill step of the decoder, then the four codes of a source word
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const bool req = k <= 32;
            const uint64_t bm = __ballot(req);
            const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(bm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bm, wpos));
            p0 = k == 0 ? pos : p0;
            p1 = req ? pos : p1;
            k += req ? 32 : 0;
            wpos += (uint32_t)__popcll(bm);
            uint32_t code, len;
            group_code(v[g], pair_lut, two, code, len);
            const uint64_t placed = (uint64_t)code << nacc;       // nothing is left above bit nacc
            lo |= (uint32_t)placed;
            nacc += len;
            k -= (int32_t)len;
            if (nacc >= 32) {
                ring[p0 & (kRing - 1)] = lo;
                lo = (uint32_t)(placed >> 32); nacc -= 32; p0 = p1;
            }
        }
        // Whole segments that are complete leave the ring, 16 bytes per lane: all of them, so that after every
        // row the ring starts at the segment of the oldest word still owed.  A word is owed for at most 16 steps
        // (64 bits at one bit per symbol), in which at most 1024 positions are handed out; with the segment
        // rounding and the 256 positions of the next row the ring never holds more than 1536 words.
#pragma unroll 1
        for (int guard = 0; guard < (int)(kRing / kSeg); guard++) {
            if (wpos < flushed + kSeg || __ballot(k + (int32_t)nacc >= 32 && p0 < flushed + kSeg) != 0) break;
            const u32x4 w = *reinterpret_cast<const u32x4 *>(ring + ((flushed + 4 * lane) & (kRing - 1)));
            __builtin_amdgcn_raw_buffer_store_b128(w, es, (int)((flushed + 4 * lane) * 4), 0, 0);
            flushed += kSeg;
        }
    };
    u32x4 xa, ya = {0, 0, 0, 0}, xb, yb = {0, 0, 0, 0};
    fetch(0, xa, ya);
    fetch(1, xb, yb);
    uint32_t row = 0;
    for (; row + 1 < rows; row += 2) {
        const u32x4 va = xa ^ ya;
        fetch(row + 2, xa, ya);
        encode_row(va, row);
        const u32x4 vb = xb ^ yb;
        fetch(row + 3, xb, yb);
        encode_row(vb, row + 1);
    }
    if (row < rows) encode_row(xa ^ ya, row);
    // the words still owed to the decoder (a partial word and look-ahead words) and the zero padding of the
    // last 16-byte unit go into the ring too; then everything left in it leaves in 16-byte pieces
    const uint32_t pend = ((uint32_t)k + nacc) >> 5;
    if (pend > 0) ring[p0 & (kRing - 1)] = lo;
    if (pend > 1) ring[p1 & (kRing - 1)] = 0;
    if (lane < ((4 - (wpos & 3)) & 3)) ring[(wpos + lane) & (kRing - 1)] = 0;
    const uint32_t end = (wpos + 3) & ~3u;                      // words of the stream with its padding
#pragma unroll 1
    for (uint32_t at = flushed + 4 * lane; __any(at < end); at += kSeg) {
        const u32x4 w = *reinterpret_cast<const u32x4 *>(ring + (at & (kRing - 1)));
        __builtin_amdgcn_raw_buffer_store_b128(w, es, (int)(at < end ? at * 4 : 0xFFFFFFF0u), 0, 0);
    }
}

// ---------------------------------------------------------------------------------------
// BF16 with 64 lanes per chunk and chunks of whole 1 KiB rows, exponent field table coded, sign+mantissa field
// flat coded, raw or table coded too: the shape of model weights, checkpoints and checkpoint deltas (Sec. 3.1,
// 4.1).  The generic encoder spends 240 (one coded field) to 360 (two) vector instructions on such a row of 8
// values per lane and is bound by them; here the row's eight exponent and eight sign+mantissa bytes are pulled
// out of the four source words with byte permutes, the R codes of a refill period (R = 2, 4 or 8 for longest
// codes of 9..16, 5..8 or at most 4 bits) are concatenated in 32 bits before they enter the 64-bit accumulator,
// and the source is fetched two rows ahead.  Sizes come from the generic size pass (it runs at the speed of its
// reads already); this kernel only writes.

// What an encoding lane keeps of one table-coded stream; the decoder it mirrors is in lock step with it.  That
// decoder asks for a word whenever it holds k <= 32 unread bits; the word's position is fixed then, its content
// is complete later.  Words asked for and not yet written number (k + nacc) / 32: never above 2 (a request
// needs k <= 32 and nacc < 32).  So one position is due (p0) and at most one more is waiting (p1): a request
// sets p1, and p0 too when nothing is owed (k == 0: at the start, and after a period that took exactly the 32
// bits the decoder held); a write moves p1 to p0.
struct LaneStream {
    uint32_t lo;                // bits not yet written, next free bit = nacc (< 32 between periods)
    uint32_t nacc;
    int32_t k;                  // unread bits the decoder would hold at this point
    uint32_t p0, p1;            // where the word in progress goes, and the one after it
    uint32_t wpos;              // words of the stream handed out so far (the same in all lanes)
    __device__ LaneStream() : lo(0), nacc(0), k(0), p0(0), p1(0), wpos(0) {}
};

// one refill step of the decoder, then the R codes of a period: bytes first .. first+R-1 of the 8 symbol bytes in w
template <int R>
__device__ __forceinline__ void code_period(LaneStream &L, const uint32_t w[2], int first, const char *lut, __amdgpu_buffer_rsrc_t out)
{
    const bool req = L.k <= 32;
    const uint64_t bm = __ballot(req);
    const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(bm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bm, L.wpos));
    L.p0 = L.k == 0 ? pos : L.p0;
    L.p1 = req ? pos : L.p1;
    L.k += req ? 32 : 0;
    L.wpos += (uint32_t)__popcll(bm);
    uint32_t code, len;
    codes_of_period<R>(w, first, lut, code, len);
    const uint64_t placed = (uint64_t)code << L.nacc;             // nothing is left above bit nacc
    L.lo |= (uint32_t)placed;
    L.nacc += len;
    L.k -= (int32_t)len;
    if (L.nacc >= 32) {
        __builtin_amdgcn_raw_buffer_store_b32(L.lo, out, (int)(L.p0 * 4), 0, 0);
        L.lo = (uint32_t)(placed >> 32); L.nacc -= 32; L.p0 = L.p1;
    }
}

// the words still owed to the decoder (a partial word and a look-ahead word), then zero padding of the last unit
__device__ __forceinline__ void close_stream(LaneStream &L, __amdgpu_buffer_rsrc_t out, uint32_t lane)
{
    const uint32_t owed = ((uint32_t)L.k + L.nacc) >> 5;
    if (owed > 0) __builtin_amdgcn_raw_buffer_store_b32(L.lo, out, (int)(L.p0 * 4), 0, 0);
    if (owed > 1) __builtin_amdgcn_raw_buffer_store_b32(0u, out, (int)(L.p1 * 4), 0, 0);
    if (lane < ((4 - (L.wpos & 3)) & 3)) __builtin_amdgcn_raw_buffer_store_b32(0u, out, (int)((L.wpos + lane) * 4), 0, 0);
}

// R0: refill period of the exponent field; R1: of the sign+mantissa field when it is table coded, 0 when it is flat or raw.
// KIND: what the source is.  kSrcBf16: BF16, 8 values per run.  kSrcFp8Pairs: FP8 coded in byte symbols (Sec. 3.2, Fig. 7:
// the exponents of two consecutive values in one byte, their sign+mantissa values in another), 16 values per run.  Either
// way a run is 8 symbols of 8 bits in each field, which is all the rest of the kernel knows.  kSrcE5m2: FP8 E5M2, whose
// 5-bit exponents and 3-bit sign+mantissa values are symbols of 8 bits each: 16 symbols per run and field, coded as two
// halves of 8 one after the other (both fields table coded; a refill period is at most 8 symbols here).
constexpr int kSrcBf16 = 0, kSrcFp8Pairs = 1, kSrcE5m2 = 2;
template <int R0, int R1, int KIND>
__device__ __forceinline__ void encode_bf16_chunk(const TensorDev *dp, const WorkItem &it, const uint32_t *enc)
{
    static_assert(KIND != kSrcE5m2 || R1 != 0, "E5M2: both fields table coded");
    constexpr bool BYTES = KIND == kSrcFp8Pairs;
    constexpr int kHalves = KIND == kSrcE5m2 ? 2 : 1;           // groups of 8 symbols per field in a 16-byte run
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = uni32(it.first + (threadIdx.x >> 6));
    const uint32_t cb = uni32(dp->chunk_bytes);
    const uint64_t n_elems = uni64(dp->n_elems);
    if (chunk >= (uint32_t)(n_elems / (KIND == kSrcBf16 ? cb / 2 : cb))) return;
    const bool has_base = uni64((uint64_t)dp->base) != 0;
    const bool sm_raw = uni32(dp->kind[1]) == 2;
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    const uint64_t payload = uni64(dp->payload_off);
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[0]));
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[1]));
    const uint64_t a0 = uni32(index0[chunk]), b0 = uni32(index0[chunk + 1]), a1 = uni32(index1[chunk]), b1 = uni32(index1[chunk + 1]);
    // the index must be as the size pass left it
    if (a0 > b0 || a1 > b1 || (b0 - a0) * 16 > 0x7FFFFFFFull || (b1 - a1) * 16 > 0x7FFFFFFFull) return;
    if (R1 == 0 && (b1 - a1) * 16 != (uint64_t)cb / 2) return;
    const __amdgpu_buffer_rsrc_t src = rsrc_of(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + (uint64_t)chunk * cb, cb);
    const __amdgpu_buffer_rsrc_t bas = rsrc_of(has_base ? reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + (uint64_t)chunk * cb : nullptr, has_base ? cb : 0);
    const __amdgpu_buffer_rsrc_t es = rsrc_of(comp + payload + 16 * a0, (uint32_t)((b0 - a0) * 16));
    const __amdgpu_buffer_rsrc_t ms = rsrc_of(comp + payload + 16 * a1, (uint32_t)((b1 - a1) * 16));
    const char *lut0 = reinterpret_cast<const char *>(enc), *lut1 = reinterpret_cast<const char *>(enc + 256);

    LaneStream E, M;
    const uint32_t rows = cb / 1024;
    // The source and the base are read with the non-temporal hint (cache policy bit 1): the exponent words leave as single
    // 4-byte stores that fill a cache line over several rows, and lines that the streaming reads push out of the L2 half
    // written are written to memory twice (the delta's containers: 1.49 times their bytes written without the hint).
    auto fetch = [&](uint32_t row, u32x4 &x, u32x4 &y) {
        row = row < rows ? row : rows - 1;
        x = __builtin_amdgcn_raw_buffer_load_b128(src, (int)(lane * 16), (int)(row * 1024), 2);
        if (has_base) y = __builtin_amdgcn_raw_buffer_load_b128(bas, (int)(lane * 16), (int)(row * 1024), 2);
    };
    auto encode_row = [&](const u32x4 &v, uint32_t row) {
        if (KIND == kSrcE5m2) {
            // a value is s eeeee mm, four per word: words 2b, 2b + 1 hold the symbols 8b .. 8b + 7 of either field
#pragma unroll
            for (int b = 0; b < kHalves; b++) {
                const uint32_t ex[2] = {(v[2 * b] >> 2) & 0x1F1F1F1Fu, (v[2 * b + 1] >> 2) & 0x1F1F1F1Fu};
                const uint32_t sm[2] = {((v[2 * b] >> 5) & 0x04040404u) | (v[2 * b] & 0x03030303u), ((v[2 * b + 1] >> 5) & 0x04040404u) | (v[2 * b + 1] & 0x03030303u)};
#pragma unroll
                for (int g = 0; g < 8 / R0; g++) code_period<R0>(E, ex, g * R0, lut0, es);
#pragma unroll
                for (int g = 0; g < 8 / (R1 ? R1 : 8); g++) code_period<(R1 ? R1 : 8)>(M, sm, g * R1, lut1, ms);
            }
            return;
        }
        // ---- the eight exponents (bits 14..7 of a value) and sign+mantissa bytes (bit 15, bits 6..0), four per word
        uint32_t ex[2], sm[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const uint32_t lo = v[2 * h], hi = v[2 * h + 1];            // BF16: values 4h, 4h+1 | 4h+2, 4h+3; FP8: 8h .. 8h+3 | 8h+4 .. 8h+7
            if (BYTES) {
                // a value is s eeee mmm: the exponent nibbles and the sign+mantissa nibbles of the even and of the odd
                // bytes, gathered with byte permutes, make the pair symbols (first value in the low four bits)
                const uint32_t e0 = (lo >> 3) & 0x0F0F0F0Fu, e1 = (hi >> 3) & 0x0F0F0F0Fu;
                ex[h] = __builtin_amdgcn_perm(e1, e0, 0x06040200u) | (__builtin_amdgcn_perm(e1, e0, 0x07050301u) << 4);
                const uint32_t m0 = ((lo >> 4) & 0x08080808u) | (lo & 0x07070707u), m1 = ((hi >> 4) & 0x08080808u) | (hi & 0x07070707u);
                sm[h] = __builtin_amdgcn_perm(m1, m0, 0x06040200u) | (__builtin_amdgcn_perm(m1, m0, 0x07050301u) << 4);
            } else {
                const uint32_t el = lo >> 7, eh = hi >> 7;                    // exponents in byte 0 and byte 2
                ex[h] = __builtin_amdgcn_perm(eh, el, 0x06040200u);          // bytes: el.b0, el.b2, eh.b0, eh.b2
                const uint32_t ml = ((lo >> 8) & 0x00800080u) | (lo & 0x007F007Fu), mh = ((hi >> 8) & 0x00800080u) | (hi & 0x007F007Fu);
                sm[h] = __builtin_amdgcn_perm(mh, ml, 0x06040200u);
            }
        }
        if (R1 == 0) {
            if (sm_raw) __builtin_amdgcn_raw_buffer_store_b64(u32x2{sm[0], sm[1]}, ms, (int)(lane * 8), (int)(row * 512), 0);
            else {
                // flat code: every byte most significant bit first, one word per 4 symbols, rows of 64 words
#pragma unroll
                for (int h = 0; h < 2; h++)
                    __builtin_amdgcn_raw_buffer_store_b32(reverse_in_groups<8>(sm[h]), ms, (int)(lane * 4), (int)((row * 2 + h) * 256), 0);
            }
        }
#pragma unroll
        for (int g = 0; g < 8 / R0; g++) code_period<R0>(E, ex, g * R0, lut0, es);
        if (R1 != 0) {
#pragma unroll
            for (int g = 0; g < 8 / (R1 ? R1 : 8); g++) code_period<(R1 ? R1 : 8)>(M, sm, g * R1, lut1, ms);
        }
    };
    u32x4 xa, ya = {0, 0, 0, 0}, xb, yb = {0, 0, 0, 0};
    fetch(0, xa, ya);
    fetch(1, xb, yb);
    uint32_t row = 0;
    for (; row + 1 < rows; row += 2) {
        const u32x4 va = xa ^ ya;
        fetch(row + 2, xa, ya);
        encode_row(va, row);
        const u32x4 vb = xb ^ yb;
        fetch(row + 3, xb, yb);
        encode_row(vb, row + 1);
    }
    if (row < rows) encode_row(xa ^ ya, row);
    close_stream(E, es, lane);
    if (R1 != 0) close_stream(M, ms, lane);
}

template <int KIND>
__global__ __launch_bounds__(256) void k_encode_bf16(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables)
{
    __shared__ uint32_t enc[512];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (dp->route != 2) return;                                  // whole workgroup: the generic encoder takes this tensor
    enc[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + threadIdx.x];
    enc[256 + threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + 256 + threadIdx.x];
    __syncthreads();
    const uint32_t r0 = uni32(dp->period[0]), r1 = uni32(dp->kind[1]) == 0 ? uni32(dp->period[1]) : 0u;
    if (KIND == kSrcE5m2) {
        switch (r0 * 16 + r1) {
        case 0x22: encode_bf16_chunk<2, 2, KIND>(dp, it, enc); break;
        case 0x42: encode_bf16_chunk<4, 2, KIND>(dp, it, enc); break;
        case 0x82: encode_bf16_chunk<8, 2, KIND>(dp, it, enc); break;
        case 0x24: encode_bf16_chunk<2, 4, KIND>(dp, it, enc); break;
        case 0x44: encode_bf16_chunk<4, 4, KIND>(dp, it, enc); break;
        case 0x84: encode_bf16_chunk<8, 4, KIND>(dp, it, enc); break;
        case 0x28: encode_bf16_chunk<2, 8, KIND>(dp, it, enc); break;
        case 0x48: encode_bf16_chunk<4, 8, KIND>(dp, it, enc); break;
        case 0x88: encode_bf16_chunk<8, 8, KIND>(dp, it, enc); break;
        default: break;                                          // the route is only given for these combinations
        }
        return;
    }
    constexpr int K = KIND == kSrcE5m2 ? kSrcBf16 : KIND;         // (the combinations below do not exist for E5M2)
    switch (r0 * 16 + r1) {
    case 0x20: encode_bf16_chunk<2, 0, K>(dp, it, enc); break;
    case 0x40: encode_bf16_chunk<4, 0, K>(dp, it, enc); break;
    case 0x80: encode_bf16_chunk<8, 0, K>(dp, it, enc); break;
    case 0x22: encode_bf16_chunk<2, 2, K>(dp, it, enc); break;
    case 0x42: encode_bf16_chunk<4, 2, K>(dp, it, enc); break;
    case 0x82: encode_bf16_chunk<8, 2, K>(dp, it, enc); break;
    case 0x24: encode_bf16_chunk<2, 4, K>(dp, it, enc); break;
    case 0x44: encode_bf16_chunk<4, 4, K>(dp, it, enc); break;
    case 0x84: encode_bf16_chunk<8, 4, K>(dp, it, enc); break;
    default: break;                                              // the route is only given for these combinations
    }
}

// fmt: ZC_FMT_BF16, ZC_FMT_FP8_E4M3_BYTES (the same encoder over FP8 values split into byte symbols) or ZC_FMT_FP8_E5M2
int launch_encode_bf16(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream)
{
    if (n_work == 0) return 0;
    if (fmt == ZC_FMT_FP8_E4M3_BYTES) hipLaunchKernelGGL(k_encode_bf16<kSrcFp8Pairs>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc);
    else if (fmt == ZC_FMT_FP8_E5M2) hipLaunchKernelGGL(k_encode_bf16<kSrcE5m2>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc);
    else hipLaunchKernelGGL(k_encode_bf16<kSrcBf16>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc);
    return (int)hipGetLastError();
}

int launch_sizes_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_sizes_fp8, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_units);
    return (int)hipGetLastError();
}

int launch_encode_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_encode_fp8, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc);
    return (int)hipGetLastError();
}

}  // namespace zc
