// Size pass, encoder and the one-launch compressions of chunks with fewer than 64 lanes: K/V-cache pages (Sec. 3.3, 5.2).
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_encode_device.h"

namespace zc {

// ---------------------------------------------------------------------------------------
// what encode_pages does with the exponent streams: count their words, write them through a ring, or keep them in LDS
constexpr int kPagesSize = 0, kPagesWrite = 1, kPagesHold = 2;
// words of LDS a workgroup has for the exponent streams it keeps until their places are known (the memory of its rings)
constexpr uint32_t kHeldWords = kWavesPerGroup * 64 * 32;

// The same shape with fewer than 64 lanes per chunk (small chunks such as K/V-cache pages, whose
// compression sits on the critical path of a decoding step: Sec. 5.2): a wavefront handles 64/S chunks
// at once, one per S-lane group.  Ballots are masked to the group, stream positions are per group, and
// the buffer resources span the tensor and the container's payload with the group's offsets in the
// vector offset; a lane with nothing to write aims past the end of the resource, where the hardware
// drops the store.  MODE: the size pass; the encoder; or the encoder for callers that learn a page's place only after
// it is coded (kPagesHold): the sign+mantissa stream goes to chunk * chunk_bytes / 2 of the payload (reverse field
// order), the exponent stream of the workgroup's i-th chunk stays in words [i * hold, (i + 1) * hold) of `stage`
// (slots_per_group * hold <= kHeldWords), its units go to `my` as in the size pass, and the result is non-zero in
// the lanes of a group whose stream did not fit (the caller then codes the pages again with kPagesWrite).
// A workgroup takes slots_per_group chunks in passes of 4 wavefronts x 64/S.
//
// The words of the exponent stream are not stored one by one (a lane's word goes to a position that was
// handed out earlier, so such stores are scattered 4-byte writes): they are collected in a ring of 32*S
// words per group in LDS and leave it in whole segments of 4*S words, 16 bytes per lane.  A segment is
// complete when every position in it has been handed out and no lane still owes a word inside it.  A lane
// that asks for a word has at most 64 more bits to produce before it writes that word (the decoder it
// mirrors held at most 32 unread bits and the word adds 32), i.e. at most 16 steps of four symbols of at
// least one bit each, during which the group hands out at most 16*S positions; with the segment rounding
// and the 4*S positions of the row in progress the ring never holds more than 24*S words.
//
// BF: 0 = FP8 as described.  2, 4, 8 = BF16 with that refill period of the exponent field (longest code 9..16,
// 5..8, at most 4 bits): a row is then 8 values per lane, 8 exponent bytes coded in 8/BF periods through the
// 256-entry table of the field, and the same 8 bytes of sign+mantissa per lane as FP8 has, so everything but the
// field split and the period is shared.  The bound on the ring needs at least 4 bits per step; with two symbols
// per step (BF = 2) that takes a shortest code of 2 bits, which the host (or k_codes_finish) checks before it
// gives a tensor to this kernel.
// The chunks [first, first + slots_per_group) of one tensor, by one workgroup.  pair: the field's table in LDS; stage,
// pairs_of_rows: the workgroup's staging memory (WRITE only); index0, index1: the chunk index of both fields (WRITE:
// read; in the container, or wherever the caller keeps it); my: where the sizes go (!WRITE), field 0's at my[chunk],
// field 1's at my[my_stride + chunk] unless my_stride is 0.  rel: what is subtracted from a chunk's number where it indexes index0, index1 and my
// (0 for arrays over the whole tensor, first_chunk for arrays over this call's chunks).
template <int S, int MODE, int BF>
__device__ __forceinline__ uint32_t encode_pages(const TensorDev *dp, uint32_t first_chunk, uint32_t slots_per_group, const uint32_t *pair, uint32_t *stage,
                                                 uint32_t *pairs_of_rows, const uint32_t *index0, const uint32_t *index1, uint32_t *my, uint32_t my_stride,
                                                 uint32_t rel = 0, uint32_t hold = 0)
{
    static_assert(S >= 4 && S <= 32, "the zero padding of a stream's last unit takes up to 3 lanes of the group");
    static_assert(BF == 0 || BF == 2 || BF == 4 || BF == 8, "FP8, or BF16 with a refill period of 2, 4 or 8");
    static_assert(MODE == kPagesSize || MODE == kPagesWrite || MODE == kPagesHold, "size pass, encoder, or encoder that keeps the exponent streams in LDS");
    constexpr bool WRITE = MODE != kPagesSize, HOLD = MODE == kPagesHold;
    constexpr int kPeriods = BF ? 8 / (BF ? BF : 1) : 4;      // refill steps per row
    constexpr uint32_t kGroups = 64 / S;
    constexpr uint32_t kNowhere = 0xFFFFFFF0u;
    constexpr uint32_t kSeg = 4 * S, kRing = 32 * S;             // words per group
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t s = lane & (S - 1), grp = lane / S;
    const uint64_t gmask = ((1ull << S) - 1) << (lane - s);
    const uint32_t cb = uni32(dp->chunk_bytes);                  // FP8: one element per byte; BF16: two bytes per element
    const uint64_t n_elems = uni64(dp->n_elems) * (BF ? 2 : 1);  // in bytes
    const uint32_t n_full = (uint32_t)(n_elems / cb);
    const bool has_base = uni64((uint64_t)dp->base) != 0;
    const bool sm_raw = uni32(dp->kind[1]) == 2;
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    const uint64_t payload = uni64(dp->payload_off), cap = uni64(dp->dst_bytes);
    if (n_elems > 0xFFFFFFF0ull) return 0;                       // the host never launches this
    const __amdgpu_buffer_rsrc_t src = rsrc_of(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)), (uint32_t)n_elems);
    const __amdgpu_buffer_rsrc_t bas = rsrc_of(has_base ? reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) : nullptr, has_base ? (uint32_t)n_elems : 0u);
    const uint64_t pay_cap = (WRITE && cap > payload) ? (cap - payload > 0xFFFFFFF0ull ? 0xFFFFFFF0ull : cap - payload) : 0;
    const __amdgpu_buffer_rsrc_t ps = rsrc_of(WRITE ? comp + payload : nullptr, (uint32_t)pay_cap);
    const char *pair_lut = reinterpret_cast<const char *>(pair);
    const uint32_t two = 2;
    const uint32_t rows = cb / (16 * S);
    uint32_t *ring = stage + (WRITE && !HOLD ? (wave * kGroups + grp) * kRing : 0);
    constexpr uint32_t kRingMask = HOLD ? 0xFFFFFFFFu : kRing - 1;  // kept streams do not wrap: words beyond their memory are dropped
    uint32_t did_not_fit = 0;
    uint32_t *const two_rows = pairs_of_rows + (WRITE ? wave * 256 + grp * 4 * S : 0);

    for (uint32_t pass = 0; pass * kWavesPerGroup * kGroups < slots_per_group; pass++) {
        const uint32_t local = (pass * kWavesPerGroup + wave) * kGroups + grp;
        if (HOLD) ring = stage + (local < slots_per_group ? local : 0) * hold;
        const uint32_t chunk = first_chunk + local;
        bool alive = local < slots_per_group && chunk < n_full;  // a short last chunk goes to the generic kernel
        uint32_t e_off = kNowhere, e_len = 0, m_off = kNowhere;
        if (HOLD && alive) {
            m_off = chunk * (cb / 2);
            if ((uint64_t)m_off + cb / 2 > pay_cap) alive = false;
        } else if (WRITE && alive) {
            const uint32_t at = chunk - rel;
            const uint64_t a0 = index0[at], b0 = index0[at + 1], a1 = index1[at], b1 = index1[at + 1];
            // the index must be as the size pass left it, and inside the 32-bit offset space of the payload
            if (a0 <= b0 && a1 <= b1 && 16 * b1 <= pay_cap && 16 * b0 <= pay_cap && (b1 - a1) * 16 == cb / 2) {
                e_off = (uint32_t)(16 * a0); e_len = (uint32_t)(16 * (b0 - a0)); m_off = (uint32_t)(16 * a1);
            } else alive = false;
        }
        const uint32_t in_off = alive ? chunk * cb : kNowhere;
        const uint32_t lim = HOLD && alive ? hold : 0u;         // kept streams: a group without a page writes nothing

        // the lane's stream: as in the 64-lane encoders, one position due (p0) and at most one more waiting (p1);
        // words asked for and not yet written number (k + nacc) / 32
        uint32_t lo = 0;            // bits not yet written, next free bit = nacc (< 32 between groups)
        uint32_t nacc = 0;
        int32_t k = 0;              // unread bits the decoder would hold at this point
        uint32_t p0 = 0, p1 = 0;
        uint32_t wpos = 0, q = 0;
        uint32_t flushed = 0;       // words of the stream that have left the ring
        // whole segments that are complete leave the ring, 16 bytes per lane
        auto flush_segments = [&]() {
#pragma unroll 1
            for (int guard = 0; guard < 8; guard++) {
                const bool owes = k + (int32_t)nacc >= 32 && p0 < flushed + kSeg;
                const bool ready = wpos >= flushed + kSeg && (__ballot(owes) & gmask) == 0;
                if (!__any(ready)) break;
                if (ready) {
                    const u32x4 w = *reinterpret_cast<const u32x4 *>(ring + ((flushed + 4 * s) & (kRing - 1)));
                    const uint32_t to = (alive && (flushed + 4 * s) * 4 + 16 <= e_len) ? e_off + (flushed + 4 * s) * 4 : kNowhere;
                    __builtin_amdgcn_raw_buffer_store_b128(w, ps, (int)to, 0, 0);
                    flushed += kSeg;
                }
            }
        };
        // the source (and the base of a delta) is fetched two rows ahead, into two register sets used in turn
        auto fetch = [&](uint32_t row, u32x4 &x, u32x4 &y) {
            row = row < rows ? row : rows - 1;
            const uint32_t at = alive ? in_off + (row * S + s) * 16 : kNowhere;
            x = __builtin_amdgcn_raw_buffer_load_b128(src, (int)at, 0, 0);
            if (has_base) y = __builtin_amdgcn_raw_buffer_load_b128(bas, (int)at, 0, 0);
        };
        auto encode_row = [&](const u32x4 &v, uint32_t row) {
            uint32_t ex[2] = {0, 0};                                // BF16: the row's eight exponent bytes
            if (BF) {
#pragma unroll
                for (int h = 0; h < 2; h++) ex[h] = __builtin_amdgcn_perm(v[2 * h + 1] >> 7, v[2 * h] >> 7, 0x06040200u);
            }
            if (WRITE) {
                // m: the row's sign+mantissa symbols (FP8: nibble j at bits 4j; BF16: bytes), or, when the field has a
                // flat code, w: every symbol most significant bit first.  FP8 gathers the nibbles of the even and of
                // the odd bytes of two words with byte permutes; for the flat code it starts from the bit-reversed
                // words, whose bytes hold s, m2, m1, m0 in this order already (bits 0, 5, 6, 7) and come reversed.
                uint32_t m[2], w[2];
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    if (BF) {
                        const uint32_t lo2 = v[2 * h], hi2 = v[2 * h + 1];
                        const uint32_t ml = ((lo2 >> 8) & 0x00800080u) | (lo2 & 0x007F007Fu), mh = ((hi2 >> 8) & 0x00800080u) | (hi2 & 0x007F007Fu);
                        m[h] = __builtin_amdgcn_perm(mh, ml, 0x06040200u);
                        w[h] = reverse_in_groups<8>(m[h]);
                    } else if (sm_raw) {
                        const uint32_t x0 = ((v[2 * h] >> 4) & 0x08080808u) | (v[2 * h] & 0x07070707u);
                        const uint32_t x1 = ((v[2 * h + 1] >> 4) & 0x08080808u) | (v[2 * h + 1] & 0x07070707u);
                        m[h] = __builtin_amdgcn_perm(x1, x0, 0x06040200u) | (__builtin_amdgcn_perm(x1, x0, 0x07050301u) << 4);
                        w[h] = 0;
                    } else {
                        const uint32_t r0 = __brev(v[2 * h]), r1 = __brev(v[2 * h + 1]);
                        const uint32_t x0 = ((r0 >> 4) & 0x0E0E0E0Eu) | (r0 & 0x01010101u);       // bytes: symbols 3, 2, 1, 0
                        const uint32_t x1 = ((r1 >> 4) & 0x0E0E0E0Eu) | (r1 & 0x01010101u);       // bytes: symbols 7, 6, 5, 4
                        w[h] = __builtin_amdgcn_perm(x1, x0, 0x05070103u) | (__builtin_amdgcn_perm(x1, x0, 0x04060002u) << 4);
                        m[h] = 0;
                    }
                }
                if (sm_raw) {
                    // the packed symbols as they are: 8 bytes per lane
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{m[0], m[1]}, ps, (int)(alive ? m_off + (row * S + s) * 8 : kNowhere), 0, 0);
                } else {
                    // flat code: one word per 8 (BF16: 4) symbols, rows of S words.  Two source rows make 4*S words of
                    // the stream: they are exchanged through LDS so that every lane stores 16 contiguous bytes; an
                    // odd last row is stored word by word.
                    if ((row & 1) == 0 && row + 1 == rows) {
#pragma unroll
                        for (int h = 0; h < 2; h++)
                            __builtin_amdgcn_raw_buffer_store_b32(w[h], ps, (int)(alive ? m_off + ((row * 2 + h) * S + s) * 4 : kNowhere), 0, 0);
                    } else {
                        two_rows[((row & 1) * 2 + 0) * S + s] = w[0];
                        two_rows[((row & 1) * 2 + 1) * S + s] = w[1];
                        if (row & 1) {
                            const u32x4 t = *reinterpret_cast<const u32x4 *>(two_rows + 4 * s);
                            __builtin_amdgcn_raw_buffer_store_b128(t, ps, (int)(alive ? m_off + ((row - 1) * 2 * S + 4 * s) * 4 : kNowhere), 0, 0);
                        }
                    }
                }
            }
#pragma unroll
            for (int g = 0; g < kPeriods; g++) {
                const bool req = k <= 32;
                if (WRITE) {
                    const uint64_t bm = __ballot(req) & gmask;
                    const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(bm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bm, wpos));
                    p0 = k == 0 ? pos : p0;              // nothing owed: the word asked for is the one due
                    p1 = req ? pos : p1;
                    wpos += (uint32_t)__popcll(bm);
                } else q += req ? 1u : 0u;
                k += req ? 32 : 0;
                uint32_t code = 0, len = 0;
                if (BF) codes_of_period<(BF ? BF : 2)>(ex, g * BF, pair_lut, code, len);
                else group_code(v[g & 3], pair_lut, two, code, len);
                k -= (int32_t)len;
                if (WRITE) {
                    const uint64_t placed = (uint64_t)code << nacc;       // nothing is left above bit nacc
                    lo |= (uint32_t)placed;
                    nacc += len;
                    const bool full = nacc >= 32;
                    if (full && (!HOLD || p0 < lim)) ring[p0 & kRingMask] = lo;
                    lo = full ? (uint32_t)(placed >> 32) : lo;
                    nacc &= 31u;                         // nacc < 64: minus 32 where a word was written
                    p0 = full ? p1 : p0;
                }
            }
            if (WRITE && !HOLD) flush_segments();
        };
        // Four register sets used in turn, each refilled four rows ahead: a page is a few rows, a row a few hundred
        // cycles of work, and the wavefront shares its SIMD with three others at most (the staging rings fill
        // the LDS), so a load issued two rows ahead was not back in time.
        u32x4 x[4], y[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
#pragma unroll
        for (uint32_t k = 0; k < 4; k++) fetch(k, x[k], y[k]);
        uint32_t row = 0;
        for (; row + 3 < rows; row += 4) {
#pragma unroll
            for (uint32_t k = 0; k < 4; k++) {
                const u32x4 v = x[k] ^ y[k];
                fetch(row + 4 + k, x[k], y[k]);
                encode_row(v, row + k);
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < 3; k++)
            if (row + k < rows) encode_row(x[k] ^ y[k], row + k);
        if (HOLD) {
            // the words still owed to the decoder and the zero padding of the last 16-byte unit, as below
            const uint32_t owed = ((uint32_t)k + nacc) >> 5;
            if (owed > 0 && p0 < lim) ring[p0] = lo;
            if (owed > 1 && p1 < lim) ring[p1] = 0;
            if (s < ((4 - (wpos & 3)) & 3) && wpos + s < lim) ring[wpos + s] = 0;
            const uint32_t end = alive ? (wpos + 3) & ~3u : 0u;  // words of the stream with its padding
            if (end > hold) did_not_fit = 1;
            if (local < slots_per_group && s == 0) my[chunk - rel] = end / 4;
        } else if (WRITE) {
            // the words still owed to the decoder (a partial word and look-ahead words) and the zero padding of
            // the last 16-byte unit go into the ring too; then everything left in it leaves in 16-byte pieces
            const uint32_t owed = ((uint32_t)k + nacc) >> 5;
            if (owed > 0) ring[p0 & (kRing - 1)] = lo;
            if (owed > 1) ring[p1 & (kRing - 1)] = 0;
            if (s < ((4 - (wpos & 3)) & 3)) ring[(wpos + s) & (kRing - 1)] = 0;
            const uint32_t end = alive ? (wpos + 3) & ~3u : 0u;  // words of the stream with its padding
#pragma unroll 1
            for (uint32_t at = flushed + 4 * s; __any(at < end); at += kSeg) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(ring + (at & (kRing - 1)));
                const uint32_t to = (alive && at < end && at * 4 + 16 <= e_len) ? e_off + at * 4 : kNowhere;
                __builtin_amdgcn_raw_buffer_store_b128(w, ps, (int)to, 0, 0);
            }
        } else {
            // words of the chunk's exponent stream = sum over the lanes of the group
#pragma unroll
            for (int o = S / 2; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
            if (alive && s == 0) {
                my[chunk - rel] = (q + 3) / 4;
                if (my_stride) my[my_stride + chunk - rel] = cb / 32;    // 4 bits per element, 16-byte units (flat code and raw alike)
            }
        }
    }
    return did_not_fit;
}

// The same for a kernel whose BF16 tensors may differ in the refill period of their exponent field (BF == kAnyBf16: the period
// is the tensor's, 2, 4 or 8).
constexpr int kAnyBf16 = 16;
template <int S, int MODE, int BF>
__device__ __forceinline__ uint32_t encode_pages_of(uint32_t period, const TensorDev *dp, uint32_t first_chunk, uint32_t slots_per_group, const uint32_t *pair,
                                                    uint32_t *stage, uint32_t *pairs_of_rows, const uint32_t *index0, const uint32_t *index1, uint32_t *my,
                                                    uint32_t my_stride, uint32_t rel, uint32_t hold)
{
    if (BF != kAnyBf16) return encode_pages<S, MODE, (BF == kAnyBf16 ? 2 : BF)>(dp, first_chunk, slots_per_group, pair, stage, pairs_of_rows, index0, index1, my, my_stride, rel, hold);
    switch (period) {
    case 2: return encode_pages<S, MODE, 2>(dp, first_chunk, slots_per_group, pair, stage, pairs_of_rows, index0, index1, my, my_stride, rel, hold);
    case 4: return encode_pages<S, MODE, 4>(dp, first_chunk, slots_per_group, pair, stage, pairs_of_rows, index0, index1, my, my_stride, rel, hold);
    default: return encode_pages<S, MODE, 8>(dp, first_chunk, slots_per_group, pair, stage, pairs_of_rows, index0, index1, my, my_stride, rel, hold);
    }
}

template <int S, bool WRITE, int BF>
__global__ __launch_bounds__(256) void k_encode_fp8_sub(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables, uint32_t *units,
                                                        uint32_t slots_per_group)
{
    constexpr uint32_t kGroups = 64 / S, kRing = 32 * S;
    __shared__ uint32_t pair[256];
    __shared__ __attribute__((aligned(16))) uint32_t stage[WRITE ? kWavesPerGroup * kGroups * kRing : 4];
    __shared__ __attribute__((aligned(16))) uint32_t pairs_of_rows[WRITE ? kWavesPerGroup * 256 : 4];   // 4*S words per group
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (dp->route != (BF ? 2 : 1) || (BF && dp->period[0] != BF)) return;      // whole workgroup: not this kernel's tensor
    pair[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + (BF ? 0 : 512) + threadIdx.x];
    __syncthreads();
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    const uint32_t *index0 = WRITE ? reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[0])) : nullptr;
    const uint32_t *index1 = WRITE ? reinterpret_cast<const uint32_t *>(comp + uni32(dp->index_off[1])) : nullptr;
    encode_pages<S, WRITE ? kPagesWrite : kPagesSize, BF>(dp, it.first, slots_per_group, pair, stage, pairs_of_rows, index0, index1, units + uni32(dp->units_off), uni32(dp->n_chunks));
}

// Stream sizes, their scan into the chunk index and the encoder in ONE launch, one workgroup per tensor, for tensors of
// so few pages that a workgroup holds all their sizes: the K/V pages a decoding step appends (Sec. 5.2: their
// compression sits on the critical path), coded with a dictionary, so that the code and with it the route are known
// when the call is made.  A page's sign+mantissa stream lies behind ALL exponent streams of its tensor, which keeps
// workgroups from placing streams before every page of the tensor is sized; inside one workgroup that is a barrier.
// The source is read twice, the second time from the cache.  Writes what k_scan writes: the container's prologue
// from the tensor's blob, both chunk indices, the total size, and the totals for the host.
constexpr uint32_t kFusedMaxPages = 512;

// BF as in the page encoder: 0 = FP8, else BF16 with that refill period of the exponent field (a workgroup whose
// tensor has another one returns at once: the host launches one build per period that occurs in the call).
template <int S, int BF>
__global__ __launch_bounds__(256) void k_compress_pages_fused(const TensorDev *descs, const uint32_t *enc_tables, const uint8_t *blobs, uint32_t blob_bytes,
                                                              ScanOut *out, int reversed)
{
    constexpr uint32_t kGroups = 64 / S, kRing = 32 * S, kPerPass = kWavesPerGroup * kGroups;
    __shared__ uint32_t pair[256];
    __shared__ __attribute__((aligned(16))) uint32_t stage[kWavesPerGroup * kGroups * kRing];
    __shared__ __attribute__((aligned(16))) uint32_t pairs_of_rows[kWavesPerGroup * 256];
    __shared__ uint32_t sizes[2 * kFusedMaxPages];               // field 0's at [chunk], field 1's at [n_chunks + chunk]
    __shared__ uint32_t idx0[kFusedMaxPages + 1], idx1[kFusedMaxPages + 1];
    const TensorDev *dp = descs + blockIdx.x;
    const uint32_t nc = uni32(dp->n_chunks), tid = threadIdx.x;
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    // whole workgroup; the host sends only tensors of the page kernels' route with 1 .. kFusedMaxPages whole pages here
    if (dp->route != (BF ? 2 : 1) || (BF && dp->period[0] != BF) || nc == 0 || nc > kFusedMaxPages || !comp) return;
    if (uni64(dp->n_elems) * (BF ? 2 : 1) != (uint64_t)nc * uni32(dp->chunk_bytes)) return;
    pair[tid] = enc_tables[(uint64_t)blockIdx.x * 768 + (BF ? 0 : 512) + tid];
    const uint32_t i0 = uni32(dp->index_off[0]), i1 = uni32(dp->index_off[1]);
    {
        // the prologue (header and code-length tables) as prepared in the blob, and zeros behind both indices
        const uint32_t *src = reinterpret_cast<const uint32_t *>(blobs + (uint64_t)blockIdx.x * blob_bytes);
        uint32_t *dst = reinterpret_cast<uint32_t *>(comp);
        for (uint32_t i = tid; i < i0 / 4; i += 256) dst[i] = src[i];
        if (tid < 8) {
            const uint32_t w = nc + 1 + (tid & 3);
            if (w < ((nc + 1 + 3) & ~3u)) dst[(tid < 4 ? i0 : i1) / 4 + w] = 0;
        }
    }
    __syncthreads();
    const uint32_t slots = (nc + kPerPass - 1) / kPerPass * kPerPass;
    encode_pages<S, kPagesSize, BF>(dp, 0, slots, pair, stage, pairs_of_rows, nullptr, nullptr, sizes, nc);
    __syncthreads();
    if (tid < 64) {
        // exclusive scan of up to 512 sizes per field by one wavefront, eight consecutive chunks per lane
        uint32_t carry = 0;
        for (int k = 0; k < 2; k++) {
            const int f = reversed ? 1 - k : k;              // the payload's order of the two fields
            uint32_t *idx = f ? idx1 : idx0;
            uint32_t v[8], t = 0;
#pragma unroll
            for (uint32_t j = 0; j < 8; j++) { v[j] = tid * 8 + j < nc ? sizes[f * nc + tid * 8 + j] : 0u; t += v[j]; }
            uint32_t x = t;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t y = __shfl_up(x, o, 64);
                if (tid >= (uint32_t)o) x += y;
            }
            uint32_t at = carry + x - t;
#pragma unroll
            for (uint32_t j = 0; j < 8; j++) { if (tid * 8 + j < nc) idx[tid * 8 + j] = at; at += v[j]; }
            carry += __shfl(x, 63, 64);
            if (tid == 0) idx[nc] = carry;
        }
    }
    __syncthreads();
    {
        uint32_t *g0 = reinterpret_cast<uint32_t *>(comp + i0), *g1 = reinterpret_cast<uint32_t *>(comp + i1);
        for (uint32_t c = tid; c <= nc; c += 256) { g0[c] = idx0[c]; g1[c] = idx1[c]; }
        if (tid == 0) {
            const uint32_t total = reversed ? idx0[nc] : idx1[nc];
            ScanOut o = {{idx0[nc] - idx0[0], idx1[nc] - idx1[0], 0}, total};
            out[blockIdx.x] = o;
            *reinterpret_cast<uint64_t *>(comp + 48) = uni64(dp->payload_off) + 16ull * total;
        }
    }
    encode_pages<S, kPagesWrite, BF>(dp, 0, slots, pair, stage, pairs_of_rows, idx0, idx1, nullptr, 0);
}

template <int S>
static void launch_fused_s(uint32_t bf16_periods, const TensorDev *d_descs, uint32_t n_tensors, const uint32_t *d_enc, const uint8_t *d_blobs, uint32_t blob_bytes,
                           ScanOut *d_out, int rev, hipStream_t st)
{
    if (!bf16_periods) { hipLaunchKernelGGL((k_compress_pages_fused<S, 0>), dim3(n_tensors), dim3(256), 0, st, d_descs, d_enc, d_blobs, blob_bytes, d_out, rev); return; }
    if (bf16_periods & 2) hipLaunchKernelGGL((k_compress_pages_fused<S, 2>), dim3(n_tensors), dim3(256), 0, st, d_descs, d_enc, d_blobs, blob_bytes, d_out, rev);
    if (bf16_periods & 4) hipLaunchKernelGGL((k_compress_pages_fused<S, 4>), dim3(n_tensors), dim3(256), 0, st, d_descs, d_enc, d_blobs, blob_bytes, d_out, rev);
    if (bf16_periods & 8) hipLaunchKernelGGL((k_compress_pages_fused<S, 8>), dim3(n_tensors), dim3(256), 0, st, d_descs, d_enc, d_blobs, blob_bytes, d_out, rev);
}

// streams: 4, 8, 16 or 32; one workgroup per tensor.  bf16_periods: 0 for FP8 tensors (route 1); for BF16 tensors (route 2)
// the refill periods of the exponent field that occur among them, or-ed together (2, 4, 8): one launch per period.
int launch_compress_pages_fused(uint32_t streams, uint32_t bf16_periods, bool reversed, const TensorDev *d_descs, uint32_t n_tensors, const uint32_t *d_enc,
                                const uint8_t *d_blobs, uint32_t blob_bytes, ScanOut *d_out, void *stream)
{
    const int rev = reversed ? 1 : 0;
    if (n_tensors == 0) return 0;
    if (bf16_periods & ~14u) return 1;
    hipStream_t st = (hipStream_t)stream;
    switch (streams) {
    case 4: launch_fused_s<4>(bf16_periods, d_descs, n_tensors, d_enc, d_blobs, blob_bytes, d_out, rev, st); break;
    case 8: launch_fused_s<8>(bf16_periods, d_descs, n_tensors, d_enc, d_blobs, blob_bytes, d_out, rev, st); break;
    case 16: launch_fused_s<16>(bf16_periods, d_descs, n_tensors, d_enc, d_blobs, blob_bytes, d_out, rev, st); break;
    case 32: launch_fused_s<32>(bf16_periods, d_descs, n_tensors, d_enc, d_blobs, blob_bytes, d_out, rev, st); break;
    default: return 1;
    }
    return (int)hipGetLastError();
}

uint32_t compress_pages_fused_limit() { return kFusedMaxPages; }

// ---------------------------------------------------------------------------------------
// K/V pages in ONE pass over the source (Sec. 5.2: their compression is on the critical path), for containers that
// keep their fields in reverse order in the payload (ZC_FLAG_REVERSE_FIELDS) and dictionary calls, so that code and
// route are known at the launch.  The sign+mantissa streams of pages are flat or raw, cb / 32 units each, and lie in
// front: page c's at c * cb / 32.  The exponent stream of page c then starts at n_chunks * cb / 32 plus the units of
// the exponent streams of the pages before it: a running sum over the pages of the tensor, which the workgroups hand
// on to each other while they run (a chained scan with look-back: every workgroup publishes the sum over its own
// pages at once, then adds up what the workgroups before it have published until it meets one that already knows its
// whole prefix, and publishes its own).
//
// A workgroup takes the next unclaimed work item (a counter in memory, so that items are claimed in the order in
// which workgroups start: whoever waits for item j knows that the workgroup of every item before j is running),
// codes the item's pages, joins the chain, writes the item's index entries and the exponent streams.  HOLD: the
// exponent streams wait in LDS for their place, `hold` words per page (an item is as many pages as fit), and the
// source is read once; should a stream not fit its words, the workgroup codes the item again through the rings once
// the places are known.  !HOLD (pages too large for that): an item is several passes, sized with the
// encoder's dry run and encoded in a second run that reads the pages from the caches (an item is tens of KiB).
// The first item of a tensor writes the container's prologue, the last one the end of both indices, the total size
// and the totals for the host.  A wait in the chain is bounded: a workgroup that gives up (it never should) marks the
// tensor's totals invalid, and the call reports a device error instead of hanging.
constexpr uint32_t kChainItemPages = 256;                    // most pages of one work item
constexpr uint64_t kChainAggregate = 1ull << 32, kChainPrefix = 2ull << 32;
constexpr uint32_t kChainSpinLimit = 1u << 17;               // rounds of 64 reads: some tenths of a second

__device__ __forceinline__ uint64_t chain_read(uint64_t *p)
{
    return __hip_atomic_fetch_add(p, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     // a read-modify-write is served where all XCDs meet
}
__device__ __forceinline__ void chain_publish(uint64_t *p, uint64_t v)
{
    __hip_atomic_exchange(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// By one whole wavefront: the units of all items before `item` back to the start of its tensor.  The 64 lanes read the
// 64 items before it at once and add up those down to the nearest one that knows its whole prefix, waiting only for
// items between that one and `item` that have published nothing yet; if none of the 64 knows its prefix the next 64
// follow.  The first item of a tensor publishes a prefix without looking back, so the walk ends there at the latest.
// 0xFFFFFFFF: gave up waiting, or an item before this one had.
__device__ __forceinline__ uint32_t chain_look_back(uint64_t *status, uint32_t item)
{
    const uint32_t lane = threadIdx.x & 63;
    uint32_t before = 0, hi = item, spins = 0;
    for (;;) {
        const bool real = lane < hi;
        const uint64_t st = real ? chain_read(status + (hi - 1 - lane)) : kChainPrefix;     // in front of item 0: nothing, and known
        const uint32_t flag = (uint32_t)(st >> 32);
        const uint64_t knows = __ballot(flag == 2), silent = __ballot(flag == 0);
        const uint32_t stop = knows ? (uint32_t)__builtin_ctzll(knows) : 64u;
        const uint64_t needed = stop < 63 ? (2ull << stop) - 1 : ~0ull;
        if (silent & needed) {
            if (++spins > kChainSpinLimit) return 0xFFFFFFFFu;
            __builtin_amdgcn_s_sleep(8);
            continue;
        }
        const bool in = lane <= stop;
        if (__any(in && real && (uint32_t)st == 0xFFFFFFFFu)) return 0xFFFFFFFFu;
        uint32_t v = in ? (uint32_t)st : 0u;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += (uint32_t)__shfl_xor((int)v, o, 64);
        before += v;
        if (stop < 64) return before;
        hi -= 64;                                               // no lane knew: all 64 were real items, so hi >= 64
    }
}

template <int S, int BF, bool HOLD>
__global__ __launch_bounds__(256) void k_compress_pages_chained(const TensorDev *descs, const WorkItem *work, uint32_t n_work, uint32_t slots_per_item,
                                                                const uint32_t *enc_tables, const uint8_t *blobs, uint32_t blob_bytes, uint64_t *status,
                                                                uint64_t *counter, ScanOut *out, uint32_t hold)
{
    constexpr uint32_t kGroups = 64 / S, kRing = 32 * S;
    static_assert(kWavesPerGroup * kGroups * kRing == kHeldWords, "the rings and the kept streams share their memory");
    __shared__ uint32_t pair[256];
    __shared__ __attribute__((aligned(16))) uint32_t stage[kHeldWords];
    __shared__ __attribute__((aligned(16))) uint32_t pairs_of_rows[kWavesPerGroup * 256];
    __shared__ uint32_t sizes[kChainItemPages + 1];               // exponent units of the item's pages, then (idx1) the index of the other field
    __shared__ uint32_t idx0[kChainItemPages + 1];
    __shared__ uint32_t claimed, before_s;
    uint32_t *const idx1 = sizes;
    const uint32_t tid = threadIdx.x;
    // an item is whole passes of the workgroup (the launcher checks it too), so that no page of the next item is touched
    if (slots_per_item == 0 || slots_per_item > kChainItemPages || slots_per_item % (kWavesPerGroup * kGroups)) return;
    if (HOLD && (hold == 0 || hold % 4 || (uint64_t)slots_per_item * hold > kHeldWords)) return;
    if (tid == 0) claimed = (uint32_t)__hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t item = uni32(claimed);
    if (item >= n_work) return;                                 // whole workgroup
    const WorkItem it = work[item];
    const TensorDev *dp = descs + it.tensor;
    const uint32_t nc = uni32(dp->n_chunks), first = uni32(it.first), cb = uni32(dp->chunk_bytes);
    uint8_t *comp = reinterpret_cast<uint8_t *>(uni64((uint64_t)dp->comp));
    const uint32_t count = first < nc ? (nc - first < slots_per_item ? nc - first : slots_per_item) : 0;
    const uint32_t per_page = cb / 32;                          // units of a sign+mantissa stream
    // what the host checked before it chose this kernel; a tensor that is not as promised is left alone, but its
    // place in the chain is filled so that nobody waits for it
    const uint32_t period = uni32(dp->period[0]);
    const bool mine = dp->route == (BF ? 2 : 1) && (!BF || (BF == kAnyBf16 ? (period == 2 || period == 4 || period == 8) : period == (uint32_t)BF)) && comp && count > 0 &&
                      uni64(dp->n_elems) * (BF ? 2 : 1) == (uint64_t)nc * cb && (uint64_t)nc * per_page < 0x80000000ull;
    if (!mine) {
        if (tid == 0) chain_publish(status + item, kChainPrefix);
        return;
    }
    pair[tid] = enc_tables[(uint64_t)it.tensor * 768 + (BF ? 0 : 512) + tid];
    sizes[tid] = 0;                                             // kChainItemPages == 256: a slot without a page counts nothing
    const uint32_t i0 = uni32(dp->index_off[0]), i1 = uni32(dp->index_off[1]);
    if (first == 0) {
        // the prologue (header and code-length tables) as prepared in the blob, and zeros behind both indices
        const uint32_t *src = reinterpret_cast<const uint32_t *>(blobs + (uint64_t)it.tensor * blob_bytes);
        uint32_t *dst = reinterpret_cast<uint32_t *>(comp);
        for (uint32_t i = tid; i < i0 / 4; i += 256) if (i != 12 && i != 13) dst[i] = src[i];       // words 12, 13: the total size, the last item's to write
        if (tid < 8) {
            const uint32_t w = nc + 1 + (tid & 3);
            if (w < ((nc + 1 + 3) & ~3u)) dst[(tid < 4 ? i0 : i1) / 4 + w] = 0;
        }
    }
    __syncthreads();
    const uint32_t slots = (count + kWavesPerGroup * kGroups - 1) / (kWavesPerGroup * kGroups) * (kWavesPerGroup * kGroups);
    // HOLD: the sign+mantissa streams are written here, the exponent streams stay in `stage`
    const uint32_t did_not_fit = encode_pages_of<S, HOLD ? kPagesHold : kPagesSize, BF>(period, dp, first, slots, pair, stage, pairs_of_rows, nullptr, nullptr, sizes,
                                                                                        0, first, hold);
    const bool again = __syncthreads_or((int)did_not_fit) != 0;
    if (tid < 64) {
        // exclusive scan of up to 256 sizes by one wavefront, four consecutive pages per lane
        uint32_t v[4], t = 0;
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) { v[j] = tid * 4 + j < count ? sizes[tid * 4 + j] : 0u; t += v[j]; }
        uint32_t x = t;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t y = __shfl_up(x, o, 64);
            if (tid >= (uint32_t)o) x += y;
        }
        const uint32_t sum = __shfl(x, 63, 64);                 // units of the item's exponent streams
        uint32_t before = 0;
        if (first == 0) {
            if (tid == 0) chain_publish(status + item, kChainPrefix | sum);
        } else {
            if (tid == 0) chain_publish(status + item, kChainAggregate | sum);
            before = chain_look_back(status, item);             // 0xFFFFFFFF: lost; the last item passes it on to the host
            if (tid == 0) chain_publish(status + item, kChainPrefix | (before == 0xFFFFFFFFu ? 0xFFFFFFFFull : (uint64_t)(before + sum)));
        }
        if (tid == 0) before_s = before;
        const uint32_t base0 = nc * per_page + (before == 0xFFFFFFFFu ? 0u : before);
        uint32_t at = base0 + x - t;
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) { if (tid * 4 + j < count) idx0[tid * 4 + j] = at; at += v[j]; }
        if (tid == 63) idx0[count] = base0 + sum;
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) if (tid * 4 + j <= count) idx1[tid * 4 + j] = (first + tid * 4 + j) * per_page;
        if (tid == 63) idx1[count] = (first + count) * per_page;
    }
    __syncthreads();
    {
        uint32_t *g0 = reinterpret_cast<uint32_t *>(comp + i0), *g1 = reinterpret_cast<uint32_t *>(comp + i1);
        const bool last = first + count == nc;
        for (uint32_t c = tid; c < count + (last ? 1u : 0u); c += 256) { g0[first + c] = idx0[c]; g1[first + c] = idx1[c]; }
        if (last && tid == 0) {
            const bool lost = before_s == 0xFFFFFFFFu;
            const uint32_t total = idx0[count];
            ScanOut o = {{total - nc * per_page, nc * per_page, 0}, lost ? 0xFFFFFFFFu : total};
            out[it.tensor] = o;
            *reinterpret_cast<uint64_t *>(comp + 48) = uni64(dp->payload_off) + 16ull * total;
        }
    }
    if (HOLD && !again) {
        // every page's stream from LDS to its place, 16 bytes per lane
        const uint32_t lane = tid & 63, s = lane & (S - 1);
        const uint64_t payload = uni64(dp->payload_off), cap = uni64(dp->dst_bytes);
        const uint64_t pay_cap = cap > payload ? (cap - payload > 0xFFFFFFF0ull ? 0xFFFFFFF0ull : cap - payload) : 0;
        const __amdgpu_buffer_rsrc_t ps = rsrc_of(comp + payload, (uint32_t)pay_cap);
        for (uint32_t pass = 0; pass * kWavesPerGroup * kGroups < count; pass++) {
            const uint32_t local = (pass * kWavesPerGroup + (tid >> 6)) * kGroups + lane / S;
            const bool alive = local < count;
            const uint32_t *held = stage + (alive ? local : 0) * hold;
            const uint32_t end = alive ? 4 * (idx0[local + 1] - idx0[local]) : 0u;       // words; at most `hold`, or `again` were set
            const uint64_t e_off = alive ? 16ull * idx0[local] : 0;
            const bool fits = alive && e_off + 4ull * end <= pay_cap;
#pragma unroll 1
            for (uint32_t at = 4 * s; __any(at < end); at += 4 * S) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(held + (at < end ? at : 0u));
                __builtin_amdgcn_raw_buffer_store_b128(w, ps, (int)(fits && at < end ? (uint32_t)e_off + at * 4 : 0xFFFFFFF0u), 0, 0);
            }
        }
        return;
    }
    encode_pages_of<S, kPagesWrite, BF>(period, dp, first, slots, pair, stage, pairs_of_rows, idx0, idx1, nullptr, 0, first, 0);
}

__global__ void k_chain_reset(uint64_t *status, uint32_t n_work, uint64_t *counter)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_work) status[i] = 0;
    if (i == 0) *counter = 0;
}

template <int S, bool HOLD>
static void launch_chained_s(uint32_t hold, uint32_t bf16_period, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint32_t slots_per_item, const uint32_t *d_enc,
                             const uint8_t *d_blobs, uint32_t blob_bytes, uint64_t *d_status, uint64_t *d_counter, ScanOut *d_out, hipStream_t st)
{
#define ZC_CHAINED(BF) hipLaunchKernelGGL((k_compress_pages_chained<S, BF, HOLD>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, n_work, slots_per_item, d_enc, \
                                          d_blobs, blob_bytes, d_status, d_counter, d_out, hold)
    switch (bf16_period) {
    case 0: ZC_CHAINED(0); break;
    case 2: ZC_CHAINED(2); break;
    case 4: ZC_CHAINED(4); break;
    case 8: ZC_CHAINED(8); break;
    default: ZC_CHAINED(kAnyBf16); break;
    }
#undef ZC_CHAINED
}

// streams: 4, 8, 16 or 32.  bf16_period: 0 for FP8 tensors (route 1), else the one refill period of the exponent field that
// every BF16 tensor of the call has (route 2), or 16 where the tensors may differ in it (codes built on the device).  Work items in natural order (tensor by tensor, pages ascending), each
// slots_per_item pages (a multiple of the pages a workgroup takes per pass, at most compress_pages_chained_limit()).
// hold: 0, or the words of LDS per page (a multiple of 4) of the build that keeps the exponent streams there and reads
// the source once; slots_per_item * hold is then at most compress_pages_held_words().  d_status: n_work words,
// d_counter: one word; both are reset here.
int launch_compress_pages_chained(uint32_t streams, uint32_t bf16_period, uint32_t hold, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                                  uint32_t slots_per_item, const uint32_t *d_enc, const uint8_t *d_blobs, uint32_t blob_bytes, uint64_t *d_status,
                                  uint64_t *d_counter, ScanOut *d_out, void *stream)
{
    if (n_work == 0) return 0;
    if (slots_per_item == 0 || slots_per_item > kChainItemPages) return 1;
    if (bf16_period != 0 && bf16_period != 2 && bf16_period != 4 && bf16_period != 8 && bf16_period != (uint32_t)kAnyBf16) return 1;
    if (streams < 4 || streams > 32 || slots_per_item % (kWavesPerGroup * (64 / streams))) return 1;
    if (hold % 4 || (uint64_t)slots_per_item * hold > kHeldWords) return 1;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_chain_reset, dim3((n_work + 255) / 256), dim3(256), 0, st, d_status, n_work, d_counter);
#define ZC_CHAINED_S(S, HOLD) launch_chained_s<S, HOLD>(hold, bf16_period, d_descs, d_work, n_work, slots_per_item, d_enc, d_blobs, blob_bytes, d_status, d_counter, d_out, st)
    switch (streams) {
    case 4: if (hold) ZC_CHAINED_S(4, true); else ZC_CHAINED_S(4, false); break;
    case 8: if (hold) ZC_CHAINED_S(8, true); else ZC_CHAINED_S(8, false); break;
    case 16: if (hold) ZC_CHAINED_S(16, true); else ZC_CHAINED_S(16, false); break;
    case 32: if (hold) ZC_CHAINED_S(32, true); else ZC_CHAINED_S(32, false); break;
    default: return 1;
    }
#undef ZC_CHAINED_S
    return (int)hipGetLastError();
}

// words of LDS a workgroup of the `hold` build has for the exponent streams of a work item
uint32_t compress_pages_held_words() { return kHeldWords; }

uint32_t compress_pages_chained_limit() { return kChainItemPages; }

template <int S, bool WRITE>
static void launch_sub_t(bool bf16, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, uint32_t slots_per_group, hipStream_t st)
{
    if (!bf16) { hipLaunchKernelGGL((k_encode_fp8_sub<S, WRITE, 0>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, slots_per_group); return; }
    // one launch per refill period: a workgroup whose tensor has another one returns at once
    hipLaunchKernelGGL((k_encode_fp8_sub<S, WRITE, 2>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, slots_per_group);
    hipLaunchKernelGGL((k_encode_fp8_sub<S, WRITE, 4>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, slots_per_group);
    hipLaunchKernelGGL((k_encode_fp8_sub<S, WRITE, 8>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, slots_per_group);
}

// streams: 4, 8, 16 or 32.  write == 0: size pass (d_units), else encode.  bf16: the BF16 builds (tensors of route 2)
// instead of the FP8 one (route 1).
int launch_encode_fp8_sub(uint32_t streams, int write, bool bf16, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc,
                          uint32_t *d_units, uint32_t slots_per_group, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    switch (streams * 2 + (write ? 1 : 0)) {
    case 8: launch_sub_t<4, false>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 9: launch_sub_t<4, true>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 16: launch_sub_t<8, false>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 17: launch_sub_t<8, true>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 32: launch_sub_t<16, false>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 33: launch_sub_t<16, true>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 64: launch_sub_t<32, false>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    case 65: launch_sub_t<32, true>(bf16, d_descs, d_work, n_work, d_enc, d_units, slots_per_group, st); break;
    default: return 1;
    }
    return (int)hipGetLastError();
}

}  // namespace zc
