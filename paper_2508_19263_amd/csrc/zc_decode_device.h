// Device helpers shared by the specialised decoders (zc_decode_fast.hip, zc_decode_s64.hip, zc_decode_pages.hip): the
// canonical decode used to fill lookup tables, raw buffer resources, wave-uniform values, and the stream rings and
// table-driven symbol decoding of the 64-lane kernels.
#pragma once

#include <type_traits>

#include "zc_internal.h"
#include "zc_device.h"

namespace zc {


namespace {

__device__ __forceinline__ uint32_t prefix_count64(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// canonical tables of the 16-symbol exponent code, built by the first threads of the group
struct Canon16 { uint32_t first[17], cnt[17], start[17]; uint8_t sorted[16]; };

__device__ inline void build_canon16(Canon16 &Cn, const uint8_t *len_table)
{
    if (threadIdx.x == 0) {
        uint8_t len[16];
        for (int v = 0; v < 16; v++) len[v] = len_table[v];
        for (int l = 0; l <= 16; l++) Cn.cnt[l] = 0;
        for (int v = 0; v < 16; v++) if (len[v] && len[v] <= 16) Cn.cnt[len[v]]++;
        uint32_t code = 0, idx = 0;
        for (int l = 1; l <= 16; l++) {
            code <<= 1;
            Cn.first[l] = code; Cn.start[l] = idx;
            for (int v = 0; v < 16; v++) if (len[v] == l) Cn.sorted[idx++] = (uint8_t)v;
            code += Cn.cnt[l];
        }
    }
    __syncthreads();
}

// decode one symbol from stream bits `bits` (LSB first); returns length | symbol << 8, 0 if none within maxlen
__device__ __forceinline__ uint32_t canon_decode(const Canon16 &Cn, uint32_t bits, uint32_t maxlen)
{
    const uint32_t msb = __brev(bits);
    for (uint32_t l = 1; l <= maxlen; l++) {
        const uint32_t code = msb >> (32 - l);
        if (code >= Cn.first[l] && code - Cn.first[l] < Cn.cnt[l]) return l | ((uint32_t)Cn.sorted[Cn.start[l] + code - Cn.first[l]] << 8);
    }
    return 0;
}

}  // namespace

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kRingWords = 1024, kRingSegment = 256;

// raw buffer resource over [p, p + bytes): a load whose vector offset is past the end returns 0
// and such a store is dropped by the hardware (the scalar offset operand is NOT range checked:
// it is used only for offsets that are in range by construction), so a damaged stream cannot
// make a lane touch memory outside its chunk's streams
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// (x & 0xFF) << sh in one instruction (byte select on the shifted operand); sh lives in a VGPR
__device__ __forceinline__ uint32_t byte0_shl(uint32_t x, uint32_t sh)
{
    uint32_t r;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(sh), "v"(x));
    return r;
}

// readfirstlane returns a signed int: go through uint32_t so that nothing is sign-extended
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    return ((uint64_t)uniform32((uint32_t)(v >> 32)) << 32) | (uint64_t)uniform32((uint32_t)v);
}

// ---------------------------------------------------------------------------------------
// Full chunks of any format with 64 lanes per chunk: the same machinery (buffer accesses,
// LDS ring per Huffman-coded field, 16-byte stores) with table-driven decoding of any code
// (11-bit lookup + canonical search for longer codes) and a per-field switch between
// Huffman, flat code, raw and constant.

enum FieldKind : uint32_t { KIND_HUFF = 0, KIND_FLAT = 1, KIND_RAW = 2, KIND_CONST = 3 };

// Stream ring of these kernels: RW words per wavefront and table-decoded field, refilled a quarter (SEG = RW / 4
// words) at a time.  RW is 512 (8 bytes per lane and segment, serviced every two refill steps) when one field of a
// chunk is table decoded and 256 (4 bytes per lane, serviced at every step) when two are, so that a workgroup's
// rings take 8 KiB either way and eight workgroups fit the LDS of a compute unit.
// A segment that has been asked for is written into the ring only when the next one is asked for, i.e. after a whole
// segment has been consumed since: that is the time its load has to arrive.  Invariant when huff_ring_service is
// called: words [wbase, wbase + RW) are in the ring except the newest SEG, which may still be in flight or in
// registers; wpos - wbase < 2 * SEG, and at most SEG words are handed out before the next call, so every word asked
// for lies below wbase + 3 * SEG: present.
constexpr uint32_t kRing2Words = 512;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct HuffStream {
    uint64_t W;            // 64 stream bits, next unread bit = bit c
    uint32_t c;
    uint32_t wpos, wbase;  // words handed out so far; first word still in the ring
    uint32_t pslot;
    uint32_t rw;           // ring words: 512 or 256 (the same in all lanes)
    bool pending;
    u32x2 pv;
    char *ring;            // this wavefront's ring in LDS
    __amdgpu_buffer_rsrc_t rs;
    uint32_t lim[4];       // FieldTab::limit of lengths 12..15 (uniform): the code lengths beyond the lookup index
};

// first: does this lane own a symbol at step 0?  (always, in a chunk of whole rows; a chunk shorter than one row
// hands its first words to the lanes that do, in lane order)
__device__ __forceinline__ void huff_open(HuffStream &H, const FieldTab &T, __amdgpu_buffer_rsrc_t rs, char *ring, uint32_t lane, uint32_t rw = kRing2Words,
                                          bool first = true)
{
    H.rs = rs; H.ring = ring; H.rw = rw;
#pragma unroll
    for (int i = 0; i < 4; i++) H.lim[i] = uniform32(T.limit[kLutBits + 1 + i]);
    const uint32_t seg_bytes = rw;                       // SEG words of 4 bytes = RW bytes
#pragma unroll
    for (uint32_t q = 0; q < 4; q++) {
        if (rw == kRing2Words) *reinterpret_cast<u32x2 *>(ring + q * seg_bytes + lane * 8) = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(lane * 8 + q * seg_bytes), 0, 0);
        else *reinterpret_cast<uint32_t *>(ring + q * seg_bytes + lane * 4) = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(lane * 4 + q * seg_bytes), 0, 0);
    }
    const uint64_t takers = __ballot(first);
    H.W = (uint64_t)(*reinterpret_cast<const uint32_t *>(ring + prefix_count64(takers) * 4)) << 32;   // step 0: word `lane` when all take one
    H.c = 32; H.wpos = (uint32_t)__popcll(takers); H.wbase = 0; H.pslot = 0; H.pending = false;
    H.pv = u32x2{0, 0};
}

__device__ __forceinline__ void huff_ring_service(HuffStream &H, uint32_t lane)
{
    const uint32_t seg = H.rw / 4;
    if (H.wpos - H.wbase >= seg) {                       // the oldest segment is used up: its place takes the segment after the newest
        const bool wide = H.rw == kRing2Words;
        if (H.pending) {
            if (wide) *reinterpret_cast<u32x2 *>(H.ring + H.pslot * 4 + lane * 8) = H.pv;
            else *reinterpret_cast<uint32_t *>(H.ring + H.pslot * 4 + lane * 4) = H.pv.x;
        }
        if (wide) H.pv = __builtin_amdgcn_raw_buffer_load_b64(H.rs, (int)(lane * 8 + (H.wbase + H.rw) * 4), 0, 0);
        else H.pv.x = __builtin_amdgcn_raw_buffer_load_b32(H.rs, (int)(lane * 4 + (H.wbase + H.rw) * 4), 0, 0);
        H.pslot = H.wbase & (H.rw - 1);
        H.wbase += seg;
        H.pending = true;
    }
}

// is the ring serviced before refill step g of a run?  (every step with the small ring, every other one with the large)
__device__ __forceinline__ bool huff_service_due(const HuffStream &H, int g) { return (g & 1) == 0 || H.rw != kRing2Words; }

// owner: does this lane own a symbol at the step the words are for?  (always, inside whole rows)
__device__ __forceinline__ void huff_refill(HuffStream &H, bool owner = true)
{
    const bool need = owner && H.c >= 32;
    const uint64_t bm = __ballot(need);
    const uint32_t w = *reinterpret_cast<const uint32_t *>(H.ring + ((prefix_count64(bm) * 4 + H.wpos * 4) & (H.rw * 4 - 1)));
    H.W = need ? ((H.W >> 32) | ((uint64_t)w << 32)) : H.W;
    H.c = need ? H.c - 32 : H.c;
    H.wpos += (uint32_t)__popcll(bm);
}

// Code longer than the lookup index (12..16 bits), without a search: in a canonical code the left-aligned
// codes of length <= l all lie below limit[l], so the length is 12 plus the number of those limits that the
// next 16 stream bits reach, and the symbol's rank follows from the code value.  Inlined: a call here would
// cost the common path its registers.  A malformed table can only give a wrong symbol: the index is masked.
__device__ __forceinline__ uint32_t long_code(const FieldTab &T, const HuffStream &H, uint32_t x)
{
    static_assert(kLutBits == 11, "four limits cover the lengths 12..15; 16 is what is left");
    const uint32_t w = __brev(x) >> 16;                    // the next 16 stream bits in code order
    const uint32_t len = 12u + (w >= H.lim[0]) + (w >= H.lim[1]) + (w >= H.lim[2]) + (w >= H.lim[3]);
    const uint32_t idx = (T.rebase[len] + (w >> (16u - len))) & 255u;
    return len | ((uint32_t)T.sorted[idx] << 8);
}

// decode one run of G symbols (SB bits each) into P0 (symbols 0..64/SB-1) and P1 (the rest).
// LONG: the code has words longer than the lookup index.
// nsym: symbols of this run the lane owns, nsym_next: of its next run (both G inside whole rows).  The words of a
// refill step are taken at the end of the step before it, by the lanes that own a symbol at the step they are for;
// a lane decodes all G symbols whatever it owns, and what it does not own is never stored.
template <int SB, int G, int R, bool LONG>
__device__ __forceinline__ void huff_run_r(HuffStream &H, const FieldTab &T, uint64_t &P0, uint64_t &P1, uint32_t lane, uint32_t nsym = G, uint32_t nsym_next = G)
{
    static_assert(!LONG || R == 2, "codes beyond the lookup index come with a refill period of 2 only; the second look relies on it");
    constexpr int PER64 = 64 / SB;
    const uint32_t mask2 = T.mask << 1;                  // entries are two bytes
    const char *lut = reinterpret_cast<const char *>(T.lut);
    uint32_t q[4] = {(uint32_t)P0, (uint32_t)(P0 >> 32), (uint32_t)P1, (uint32_t)(P1 >> 32)};
#pragma unroll
    for (int g = 0; g < G / R; g++) {
        if (huff_service_due(H, g)) huff_ring_service(H, lane);
        const uint32_t x0 = (uint32_t)(H.W >> H.c);
        uint32_t e[R];
        if (R == 2) {
            // index from the window shifted left once: bits [1..] of (y >> n) are bits [0..] of (x >> n)
            uint32_t y = x0 << 1;
            e[0] = *reinterpret_cast<const uint16_t *>(lut + (y & mask2));
            y >>= (e[0] & 31u);
            e[1] = *reinterpret_cast<const uint16_t *>(lut + (y & mask2));
        } else {
            uint32_t x = x0;
#pragma unroll
            for (int j = 0; j < R; j++) {
                e[j] = *reinterpret_cast<const uint16_t *>(lut + ((x << 1) & mask2));
                x >>= (e[j] & 31u);
            }
        }
        if (LONG) {
            // An empty entry stands for a code longer than the index; it shifts by nothing, so the entry after it is
            // empty too and the last one tells.  Then the long code is searched for, and only what it spoiled is
            // done again: the lookup of the symbol after it.
            if (__any(e[R - 1] == 0)) {
                uint32_t x = x0;
#pragma unroll
                for (int j = 0; j < R; j++) {
                    if (e[j] == 0) {
                        e[j] = long_code(T, H, x);
                        if (j + 1 < R) e[j + 1] = *reinterpret_cast<const uint16_t *>(lut + (((x >> (e[j] & 31u)) << 1) & mask2));
                    }
                    x >>= (e[j] & 31u);
                }
            }
        }
        // lengths in bits 4..0 of the entries, symbols in byte 1: the low 7 bits of a sum are the sum of the lengths
        // (at most 32 per period, and c was at most 32)
        uint32_t c = H.c;
#pragma unroll
        for (int j = 0; j < R; j++) {
            const int jj = g * R + j;
            c += e[j];
            constexpr int kPer32 = 32 / SB;
            const int word = jj / kPer32, pos = jj % kPer32;
            if (SB == 8) {
                // byte 1 of the entry (the symbol) into byte `pos` of the word
                const uint32_t sel = pos == 0 ? 0x03020105u : pos == 1 ? 0x03020500u : pos == 2 ? 0x03050100u : 0x05020100u;
                q[word] = __builtin_amdgcn_perm(e[j], q[word], sel);
            } else q[word] |= (e[j] >> 8) << (pos * SB);
        }
        H.c = c & 0x7Fu;
        huff_refill(H, g + 1 < G / R ? (uint32_t)((g + 1) * R) < nsym : nsym_next > 0);
    }
    P0 = (uint64_t)q[0] | ((uint64_t)q[1] << 32);
    if (G > PER64) P1 = (uint64_t)q[2] | ((uint64_t)q[3] << 32);
}

template <int SB, int G, bool LONG>
__device__ __forceinline__ void huff_run_l(HuffStream &H, const FieldTab &T, uint32_t period, uint64_t &P0, uint64_t &P1, uint32_t lane,
                                           uint32_t nsym = G, uint32_t nsym_next = G)
{
    switch (period) {
    case 2: huff_run_r<SB, G, 2, LONG>(H, T, P0, P1, lane, nsym, nsym_next); break;
    case 4: huff_run_r<SB, G, 4, LONG>(H, T, P0, P1, lane, nsym, nsym_next); break;
    case 8: huff_run_r<SB, G, 8, LONG>(H, T, P0, P1, lane, nsym, nsym_next); break;
    case 16: if (G >= 16) huff_run_r<SB, G, (G >= 16 ? 16 : G), LONG>(H, T, P0, P1, lane, nsym, nsym_next); break;
    default: if (G >= 32) huff_run_r<SB, G, (G >= 32 ? 32 : G), LONG>(H, T, P0, P1, lane, nsym, nsym_next); break;
    }
}

template <int SB, int G>
__device__ __forceinline__ void huff_run(HuffStream &H, const FieldTab &T, uint32_t period, uint64_t &P0, uint64_t &P1, uint32_t lane,
                                         uint32_t nsym = G, uint32_t nsym_next = G)
{
    // only refill periods of 2 can come with codes longer than the 11-bit index (longest code > 11 bits)
    if (period == 2 && T.lmax > (uint32_t)kLutBits) huff_run_r<SB, G, 2, true>(H, T, P0, P1, lane, nsym, nsym_next);
    else huff_run_l<SB, G, false>(H, T, period, P0, P1, lane, nsym, nsym_next);
}

// One plainly stored field of the run a lane owns in the row after a chunk's last whole row (the row a short last
// chunk, or a chunk size that is not whole rows, ends with): nsym of its G symbols exist.  Flat code: every step of
// 32 / SB symbols hands one word to each lane that owns a symbol there, in lane order, after the words of the whole
// rows; raw: the run's words lie where they would in a whole row.  What the lane does not own is never stored.
template <int SB, int G>
__device__ __forceinline__ void plain_tail(uint32_t kind, __amdgpu_buffer_rsrc_t rs, uint32_t whole_rows, uint32_t lane, uint32_t nsym, uint64_t konst,
                                           uint64_t &P0, uint64_t &P1)
{
    constexpr int WPR = G * SB / 32;
    if (kind != KIND_FLAT && kind != KIND_RAW) { P0 = konst; P1 = konst; return; }
    uint32_t w[WPR];
    uint32_t at = whole_rows * WPR * 64;                  // words of the stream before this row
#pragma unroll
    for (int h = 0; h < WPR; h++) {
        if (kind == KIND_FLAT) {
            const bool owner = (uint32_t)(h * (32 / SB)) < nsym;
            const uint64_t bm = __ballot(owner);
            const uint32_t v = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(owner ? (at + prefix_count64(bm)) * 4 : 0xFFFFFFF0u), 0, 0);
            w[h] = reverse_in_groups<SB>(v);
            at += (uint32_t)__popcll(bm);
        } else w[h] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(((whole_rows * 64 + lane) * WPR + h) * 4), 0, 0);
    }
    P0 = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    if (WPR == 4) P1 = (uint64_t)w[2] | ((uint64_t)w[3] << 32);
}

// One field of one run when it is not table decoded, in two steps so that the loads of a row can be in flight while the
// row before it is decoded: plain_fetch asks for the run's words (G*SB/32 of them; all offsets are in the range-checked
// operand, so a row past the end reads zeros), plain_finish turns them into the packed symbols.
template <int SB, int G>
__device__ __forceinline__ void plain_fetch(uint32_t kind, __amdgpu_buffer_rsrc_t rs, uint32_t row, uint32_t lane, uint32_t w[G * SB / 32])
{
    constexpr int WPR = G * SB / 32;           // 2 for element fields, 4 for the scale field and for 16 symbols of 8 bits
    if (kind == KIND_FLAT) {
        // regular schedule: every lane takes one word per 32/SB symbols, rows of 64 words
#pragma unroll
        for (int h = 0; h < WPR; h++) w[h] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(((row * WPR + h) * 64 + lane) * 4), 0, 0);
    } else if (kind == KIND_RAW) {
#pragma unroll
        for (int h = 0; h < WPR; h++) w[h] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(((row * 64 + lane) * WPR + h) * 4), 0, 0);
    }
}

template <int SB, int G>
__device__ __forceinline__ void plain_finish(uint32_t kind, const uint32_t w_in[G * SB / 32], uint64_t konst, uint64_t &P0, uint64_t &P1)
{
    constexpr int WPR = G * SB / 32;
    if (kind != KIND_FLAT && kind != KIND_RAW) { P0 = konst; P1 = konst; return; }
    uint32_t w[WPR];
#pragma unroll
    for (int h = 0; h < WPR; h++) w[h] = kind == KIND_FLAT ? reverse_in_groups<SB>(w_in[h]) : w_in[h];
    P0 = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    if (WPR == 4) P1 = (uint64_t)w[2] | ((uint64_t)w[3] << 32);
}

template <int SB, int G>
__device__ __forceinline__ void plain_run(uint32_t kind, __amdgpu_buffer_rsrc_t rs, uint32_t row, uint32_t lane, uint64_t konst, uint64_t &P0, uint64_t &P1)
{
    uint32_t w[G * SB / 32] = {};
    plain_fetch<SB, G>(kind, rs, row, lane, w);
    plain_finish<SB, G>(kind, w, konst, P0, P1);
}

__device__ __forceinline__ bool stream_range(const TensorDev &d, const uint8_t *comp, int f, uint32_t chunk, uint64_t payload, uint64_t total,
                                             const uint8_t *&ptr, uint32_t &bytes)
{
    ptr = comp; bytes = 0;
    if (d.mode[f] != ZC_MODE_HUFF && d.mode[f] != ZC_MODE_RAW) return true;
    const uint32_t *index = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[f]));
    const uint64_t a = uniform32(index[chunk]), b = uniform32(index[chunk + 1]);
    if (a > b || payload + 16 * b > total || (b - a) * 16 > 0x7FFFFFFFull) return false;
    ptr = comp + payload + 16 * a;
    bytes = (uint32_t)((b - a) * 16);
    return true;
}

}  // namespace zc
