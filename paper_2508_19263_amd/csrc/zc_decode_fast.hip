// Specialised decode kernels for the common shapes of a container: FP8 E4M3, 64 lanes per
// chunk, full chunks, exponent field Huffman coded with a longest code of 5..8 bits (refill
// period 4), and a
// sign+mantissa field that is either stored raw or coded with the flat 4-bit code (which
// is what the Huffman construction returns for its near-uniform histogram).
// Everything else goes through the generic kernel in zc_kernels.hip.
//
// One wavefront decodes one chunk.  Per 16-byte run of output a lane
//   - decodes 16 exponent symbols from its window of the lane-interleaved stream, in
//     groups of 4 with one refill step per group (ballot + prefix count gives the word),
//     using a lookup table in LDS whose entries already hold the symbol at its place in
//     the output byte;
//   - takes the 16 sign+mantissa nibbles straight from the stream (two words per run for
//     the flat code, whose refill schedule is regular; 8 bytes for raw);
//   - merges both into the original bytes and stores 128 bits, contiguous across lanes.
#include <hip/hip_runtime.h>

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

__device__ void build_canon16(Canon16 &Cn, const uint8_t *len_table)
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

// EK: 0 = one symbol per lookup (codes <= 8 bits, 256 entries), 1 = two symbols per lookup
//     (codes <= 6 bits, 4096 entries).  MK: 0 = flat 4-bit code, 1 = raw.  XOR: delta container.
// IDS: a build that also takes tensors with a list of chunk ids (slot i of the output takes chunk ids[i]; whole chunks
// only: a short last chunk that a list names is left to the 64-lane kernel's build for such chunks).
template <int EK, int MK, bool XOR, bool IDS>
__global__ __launch_bounds__(256) void k_decode_fp8(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single)
{
    constexpr uint32_t kEntries = EK ? 4096u : 256u;
    // single lookups use 16-bit entries (length, exponent << 3): half as many distinct words
    // per LDS bank as 32-bit entries, so fewer bank conflicts at data-dependent addresses
    typedef typename std::conditional<EK == 0, uint16_t, uint32_t>::type entry_t;
    __shared__ entry_t lut[kEntries];
    // per wavefront: the next 1024 words of its exponent stream, refilled 256 words at a time
    // one output row ahead of use, so that a refill step never waits on global memory
    __shared__ __attribute__((aligned(16))) uint32_t ring[kWavesPerGroup][kRingWords];
    __shared__ Canon16 canon;
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = blockIdx.x * kWavesPerGroup; }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    build_canon16(canon, d.comp + d.table_off[0]);
    const uint32_t lmax = d.lmax[0] < (EK ? 6u : 8u) ? d.lmax[0] : (EK ? 6u : 8u);
    // table entries: bits 4..0 = bits consumed; byte 1 (and byte 2 for pairs) = exponent << 3
    for (uint32_t idx = threadIdx.x; idx < kEntries; idx += 256) {
        uint32_t e = canon_decode(canon, idx, lmax);
        uint32_t entry = (e & 31u) | (((e >> 8) << 3) << 8);
        if (EK) {
            const uint32_t e2 = canon_decode(canon, idx >> (e & 31u), lmax);
            entry = ((e & 31u) + (e2 & 31u)) | (((e >> 8) << 3) << 8) | (((e2 >> 8) << 3) << 16);
        }
        lut[idx] = (entry_t)entry;
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63;
    const uint32_t slot = uniform32(it.first + (threadIdx.x >> 6));
    uint32_t chunk = slot;
    if (IDS) {
        const uint32_t *ids = reinterpret_cast<const uint32_t *>(uniform64((uint64_t)d.ids));
        if (ids) {
            if (slot >= uniform32(d.n_ids)) return;
            chunk = uniform32(ids[slot]);
        }
    }
    const uint32_t E = uniform32(d.chunk_bytes);     // one element per byte
    const uint32_t n_full = (uint32_t)(uniform64(d.n_elems) / E);
    if (chunk >= n_full) return;                            // partial or absent chunk: not ours
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[0]));
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[1]));
    const uint64_t a0 = uniform32(index0[chunk]), b0 = uniform32(index0[chunk + 1]);
    const uint64_t a1 = uniform32(index1[chunk]), b1 = uniform32(index1[chunk + 1]);
    const uint32_t rows = E / (16 * 64);
    // a stream that does not lie inside the container, or a sign+mantissa stream shorter than
    // its fixed size, means a damaged index: leave the chunk alone rather than read outside
    if (a0 > b0 || a1 > b1 || payload + 16 * b1 > total || payload + 16 * b0 > total) return;
    if ((b1 - a1) * 16 < (uint64_t)E / 2 || (b0 - a0) * 16 > 0x7FFFFFFFull) return;
    const __amdgpu_buffer_rsrc_t es = make_rsrc(comp + payload + 16 * a0, (uint32_t)((b0 - a0) * 16));
    const __amdgpu_buffer_rsrc_t ms = make_rsrc(comp + payload + 16 * a1, E / 2);
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)) + (uint64_t)slot * E, E);       // slot == chunk without a list
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) + (uint64_t)chunk * E : comp, XOR ? E : 0);

    // Ring invariant at the top of every row: words [wbase, wbase + 1024) of the stream are in the
    // ring, except the newest 256 while their load is in flight; a row takes at most 4 * 64 words
    // and wpos - wbase < 512, so every word a row can ask for is already there.
    const uint32_t wave = threadIdx.x >> 6;
    char *const ring_bytes = reinterpret_cast<char *>(&ring[wave][0]);
#pragma unroll
    for (uint32_t q = 0; q < kRingWords / kRingSegment; q++) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(es, (int)(lane * 16 + q * kRingSegment * 4), 0, 0);
        *reinterpret_cast<u32x4 *>(ring_bytes + q * kRingSegment * 4 + lane * 16) = v;
    }
    // step 0 of the stream: every lane takes its first word
    uint64_t W = (uint64_t)(*reinterpret_cast<const uint32_t *>(ring_bytes + lane * 4)) << 32;
    uint32_t c = 32, wpos = 64, wbase = 0;
    bool pending = false;
    u32x4 pv = {0, 0, 0, 0};
    uint32_t pslot = 0;
    const uint32_t one = 1;
    const char *lut_bytes = reinterpret_cast<const char *>(lut);
    for (uint32_t row = 0; row < rows; row++) {
        if (pending) {                                   // the segment asked for one row ago has arrived
            *reinterpret_cast<u32x4 *>(ring_bytes + pslot * 4 + lane * 16) = pv;
            pending = false;
        }
        if (wpos - wbase >= kRingSegment) {              // oldest segment used up: fetch the one that replaces it
            pv = __builtin_amdgcn_raw_buffer_load_b128(es, (int)(lane * 16 + (wbase + kRingWords) * 4), 0, 0);
            pslot = wbase & (kRingWords - 1);
            wbase += kRingSegment;
            pending = true;
        }
        // ---- sign+mantissa: 16 nibbles -> bytes s0000mmm, four per word
        uint32_t m[4];
        if (MK == 0) {
            // flat code: one word per 8 symbols, rows of 64 words; code bits are MSB first in an
            // LSB-first string, so a bit reversal gives natural nibbles in reverse symbol order
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t w = __brev(__builtin_amdgcn_raw_buffer_load_b32(ms, (int)(lane * 4), (int)((row * 2 + h) * 256), 0));
                const uint32_t A = ((w << 4) & 0x80808080u) | (w & 0x07070707u);          // symbols 7,5,3,1 in bytes 0..3
                const uint32_t B = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);          // symbols 6,4,2,0
                m[2 * h] = perm(A, B, 0x06020703u);            // bytes: B3 A3 B2 A2 -> symbols 0,1,2,3
                m[2 * h + 1] = perm(A, B, 0x04000501u);        // bytes: B1 A1 B0 A0 -> symbols 4,5,6,7
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(ms, (int)(lane * 8 + h * 4), (int)(row * 512), 0);
                const uint32_t A = ((w << 4) & 0x80808080u) | (w & 0x07070707u);          // symbols 0,2,4,6
                const uint32_t B = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);          // symbols 1,3,5,7
                m[2 * h] = perm(A, B, 0x01050004u);            // bytes: A0 B0 A1 B1
                m[2 * h + 1] = perm(A, B, 0x03070206u);        // bytes: A2 B2 A3 B3
            }
        }
        // ---- exponent: 4 groups of 4 symbols, each followed by the refill step of the next group
        uint32_t o[4];
#pragma unroll
        for (int g = 0; g < 4; g++) {
            uint32_t x = (uint32_t)(W >> c);
            if (EK == 0) {
                const uint32_t t0 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t0 & 31u);
                const uint32_t t1 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t1 & 31u);
                const uint32_t t2 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t2 & 31u);
                const uint32_t t3 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one));
                c += (t0 + t1 + t2 + t3) & 0xFFu;
                // byte 1 of each entry -> bytes 0..3 of the output word
                o[g] = perm(t1, t0, 0x0C0C0501u) | perm(t3, t2, 0x05010C0Cu) | m[g];
            } else {
                x <<= 2;                                           // 30 bits left: two lookups need 24
                const uint32_t t0 = *reinterpret_cast<const uint32_t *>(lut_bytes + (x & 0x3FFCu)); x >>= (t0 & 31u);
                const uint32_t t1 = *reinterpret_cast<const uint32_t *>(lut_bytes + (x & 0x3FFCu));
                c += (t0 + t1) & 0xFFu;
                o[g] = perm(t1, t0, 0x06050201u) | m[g];          // [t0.b1, t0.b2, t1.b1, t1.b2]
            }
            // refill step: lanes whose low word is used up take the next word of the stream, in lane order
            const bool need = c >= 32;
            const uint64_t bm = __ballot(need);
            const uint32_t w = *reinterpret_cast<const uint32_t *>(ring_bytes + ((prefix_count64(bm) * 4 + wpos * 4) & (kRingWords * 4 - 1)));
            W = need ? ((W >> 32) | ((uint64_t)w << 32)) : W;
            c = need ? c - 32 : c;
            wpos += (uint32_t)__popcll(bm);
        }
        // ---- byte = s eeee mmm
        u32x4 v = {o[0], o[1], o[2], o[3]};
        if (XOR) v ^= __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(lane * 16), (int)(row * 1024), 0);
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 0);
    }
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
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 0);
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
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 0);
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
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 0);
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

// ---------------------------------------------------------------------------------------
// FP8 with fewer than 64 lanes per chunk (small chunks such as K/V-cache pages): a wavefront
// decodes 64/S chunks at once, one per S-lane group, optionally picked from an id list and
// written densely.  Same per-lane work as k_decode_fp8; what differs is that every stream
// position is per group (vector registers, prefix counts masked to the group) and that one
// buffer resource spans the whole payload, with the group's stream offset in the vector
// offset.  Each group owns 16*S words of the wavefront's 1024-word ring, refilled 4*S words
// (one 16-byte load per lane) at a time.
// LINES: the sign+mantissa words are fetched a cache line at a time and handed out through LDS.  That pays
// when neighbouring chunks are decoded together (whole tensors: 0.98 against 1.02 ms on the K/V set) and
// costs when pages are picked at random (0.31 against 0.28 ms), so id lists run without it.
template <int S, bool XOR, bool LINES>
__global__ __launch_bounds__(256) void k_decode_fp8_sub(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single,
                                                        uint32_t slots_per_group)
{
    constexpr uint32_t kGroups = 64 / S;
    constexpr uint32_t kSeg = 4 * S, kRing = 16 * S;             // words per group
    __shared__ uint16_t lut[256];
    __shared__ __attribute__((aligned(16))) uint32_t ring[kWavesPerGroup][kRingWords];
    __shared__ __attribute__((aligned(16))) uint32_t two_rows[kWavesPerGroup][LINES ? 256 : 4];      // 4*S words per group
    __shared__ Canon16 canon;
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = blockIdx.x * slots_per_group; }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    build_canon16(canon, d.comp + d.table_off[0]);
    {
        const uint32_t lmax = d.lmax[0] < 8u ? d.lmax[0] : 8u;
        const uint32_t e = canon_decode(canon, threadIdx.x, lmax);
        lut[threadIdx.x] = (uint16_t)((e & 31u) | (((e >> 8) << 3) << 8));
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t s = lane & (S - 1), grp = lane / S;
    const uint64_t gmask = ((1ull << S) - 1) << (lane - s);
    const uint32_t cb = uniform32(d.chunk_bytes);                // one element per byte
    const uint64_t n_elems = uniform64(d.n_elems);
    const uint32_t n_full = (uint32_t)(n_elems / cb);
    const uint32_t *ids = reinterpret_cast<const uint32_t *>(uniform64((uint64_t)d.ids));
    const uint64_t dst_bytes = uniform64(d.dst_bytes);
    const uint32_t n_slots = ids ? uniform32(d.n_ids) : uniform32(d.n_chunks);
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    if (total < payload || total - payload > 0xFFFFFFF0ull || dst_bytes > 0xFFFFFFF0ull) return;   // the host never launches this
    const uint32_t pay_bytes = (uint32_t)(total - payload);
    const __amdgpu_buffer_rsrc_t ps = make_rsrc(comp + payload, pay_bytes);
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)), (uint32_t)dst_bytes);
    const uint64_t base_bytes = XOR ? n_elems : 0;
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) : comp,
                                                base_bytes > 0xFFFFFFF0ull ? 0u : (uint32_t)base_bytes);
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[0]));
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[1]));
    const bool sm_raw = uniform32(d.kind[1]) == 2;
    const uint32_t rows = cb / (16 * S);
    const uint32_t one = 1;
    const char *lut_bytes = reinterpret_cast<const char *>(lut);
    char *const ring_bytes = reinterpret_cast<char *>(&ring[wave][0]) + grp * (kRing * 4);
    uint32_t *const sm_words = &two_rows[wave][LINES ? grp * 4 * S : 0];

    // the workgroup owns slots [first, first + slots_per_group): each pass takes 4 waves x kGroups of them
    for (uint32_t pass = 0; pass * kWavesPerGroup * kGroups < slots_per_group; pass++) {
        const uint32_t slot = it.first + (pass * kWavesPerGroup + wave) * kGroups + grp;
        uint32_t chunk = slot;
        bool alive = slot < n_slots && (pass * kWavesPerGroup + wave) * kGroups + grp < slots_per_group;
        if (ids && alive) chunk = ids[slot];
        alive = alive && chunk < n_full;                         // short last chunk: the host sends it to the generic kernel
        uint32_t e_off = pay_bytes, m_off = pay_bytes;           // out of range: loads return 0
        uint32_t e_len = 0;                                      // bytes of the exponent stream
        if (alive) {
            const uint64_t a0 = index0[chunk], b0 = index0[chunk + 1], a1 = index1[chunk], b1 = index1[chunk + 1];
            if (a0 <= b0 && a1 <= b1 && 16 * b1 <= pay_bytes && 16 * b0 <= pay_bytes && (b1 - a1) * 16 >= cb / 2) {
                e_off = (uint32_t)(16 * a0); m_off = (uint32_t)(16 * a1); e_len = (uint32_t)(16 * (b0 - a0));
            } else alive = false;
        }
        // the ring reads ahead of what is consumed: a piece past the end of this chunk's stream is not fetched
        // (it would be the next chunk's data, read a second time by whoever decodes that chunk)
        auto ring_piece = [&](uint32_t word) -> u32x4 {
            return __builtin_amdgcn_raw_buffer_load_b128(ps, (int)(word * 4 < e_len ? e_off + word * 4 : pay_bytes), 0, 0);
        };
        const uint32_t out_off = slot * cb, base_off = chunk * cb;

        // The sign+mantissa stream of two rows is 4*S contiguous words in both layouts: the group fetches them
        // with one 16-byte load per lane (whole cache lines instead of 4-byte pieces that are evicted between
        // rows), one pair of rows ahead, and hands every lane its own words through LDS.  The first pair is
        // asked for before the ring's prologue so that both waits overlap.
        u32x4 sm_next = {0, 0, 0, 0};
        if (LINES) sm_next = __builtin_amdgcn_raw_buffer_load_b128(ps, (int)(m_off + s * 16), 0, 0);
        // ring prologue: the group's first 16*S words (each lane 4 loads of 16 bytes)
#pragma unroll
        for (uint32_t q = 0; q < 4; q++) {
            const u32x4 v = ring_piece(q * kSeg + s * 4);
            *reinterpret_cast<u32x4 *>(ring_bytes + (q * kSeg + s * 4) * 4) = v;
        }
        uint64_t W = (uint64_t)(*reinterpret_cast<const uint32_t *>(ring_bytes + s * 4)) << 32;    // step 0: lane s takes word s
        uint32_t c = 32, wpos = S, wbase = 0, pslot = 0;
        bool pending = false;
        u32x4 pv = {0, 0, 0, 0};
        for (uint32_t row = 0; row < rows; row++) {
            if (LINES && (row & 1) == 0) {
                *reinterpret_cast<u32x4 *>(sm_words + 4 * s) = sm_next;
                const uint32_t next = ((row + 2) * 2 * S + 4 * s) * 4;                  // nothing past the chunk's cb/2 bytes
                sm_next = __builtin_amdgcn_raw_buffer_load_b128(ps, (int)(next < cb / 2 ? m_off + next : pay_bytes), 0, 0);
            }
            if (pending) { *reinterpret_cast<u32x4 *>(ring_bytes + (pslot + s * 4) * 4) = pv; pending = false; }
            if (wpos - wbase >= kSeg) {
                pv = ring_piece(wbase + kRing + s * 4);
                pslot = wbase & (kRing - 1);
                wbase += kSeg;
                pending = true;
            }
            uint32_t m[4];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                uint32_t A, B;
                if (sm_raw) {
                    const uint32_t w = LINES ? sm_words[((row & 1) * S + s) * 2 + h]
                                             : __builtin_amdgcn_raw_buffer_load_b32(ps, (int)(m_off + ((row * S + s) * 2 + h) * 4), 0, 0);
                    A = ((w << 4) & 0x80808080u) | (w & 0x07070707u);
                    B = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);
                    m[2 * h] = perm(A, B, 0x01050004u);
                    m[2 * h + 1] = perm(A, B, 0x03070206u);
                } else {
                    const uint32_t w = __brev(LINES ? sm_words[((row & 1) * 2 + h) * S + s]
                                                    : __builtin_amdgcn_raw_buffer_load_b32(ps, (int)(m_off + ((row * 2 + h) * S + s) * 4), 0, 0));
                    A = ((w << 4) & 0x80808080u) | (w & 0x07070707u);
                    B = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);
                    m[2 * h] = perm(A, B, 0x06020703u);
                    m[2 * h + 1] = perm(A, B, 0x04000501u);
                }
            }
            uint32_t o[4];
#pragma unroll
            for (int g = 0; g < 4; g++) {
                uint32_t x = (uint32_t)(W >> c);
                const uint32_t t0 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t0 & 31u);
                const uint32_t t1 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t1 & 31u);
                const uint32_t t2 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one)); x >>= (t2 & 31u);
                const uint32_t t3 = *reinterpret_cast<const uint16_t *>(lut_bytes + byte0_shl(x, one));
                c += (t0 + t1 + t2 + t3) & 0xFFu;
                o[g] = perm(t1, t0, 0x0C0C0501u) | perm(t3, t2, 0x05010C0Cu) | m[g];
                const bool need = c >= 32;
                const uint64_t bm = __ballot(need) & gmask;
                const uint32_t w = *reinterpret_cast<const uint32_t *>(ring_bytes + ((prefix_count64(bm) + wpos) & (kRing - 1)) * 4);
                W = need ? ((W >> 32) | ((uint64_t)w << 32)) : W;
                c = need ? c - 32 : c;
                wpos += (uint32_t)__popcll(bm);
            }
            u32x4 v = {o[0], o[1], o[2], o[3]};
            if (XOR) v ^= __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(base_off + (row * S + s) * 16), 0, 0);
            if (alive) __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(out_off + (row * S + s) * 16), 0, 0);
        }
    }
}

template <int S>
static int launch_fp8_sub_s(bool xor_delta, bool lines, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single,
                            uint32_t slots_per_group, hipStream_t st)
{
    if (xor_delta && lines) hipLaunchKernelGGL((k_decode_fp8_sub<S, true, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    else if (xor_delta) hipLaunchKernelGGL((k_decode_fp8_sub<S, true, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    else if (lines) hipLaunchKernelGGL((k_decode_fp8_sub<S, false, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    else hipLaunchKernelGGL((k_decode_fp8_sub<S, false, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    return (int)hipGetLastError();
}

// FP8, S in {4, 8, 16, 32}, full chunks, exponent refill period 4, sign+mantissa flat or raw.
// Each workgroup takes slots_per_group consecutive slots (chunk ids, or positions in d_ids).
// scattered: some tensor decodes an id list (pages picked at random rather than neighbours).
int launch_decode_fp8_sub(uint32_t streams, bool xor_delta, bool scattered, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                          const TensorDev *single, uint32_t slots_per_group, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    switch (streams) {
    case 4: return launch_fp8_sub_s<4>(xor_delta, !scattered, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 8: return launch_fp8_sub_s<8>(xor_delta, !scattered, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 16: return launch_fp8_sub_s<16>(xor_delta, !scattered, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 32: return launch_fp8_sub_s<32>(xor_delta, !scattered, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    }
    return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// BF16 with fewer than 64 lanes per chunk (K/V-cache pages in BF16, Sec. 3.3): the structure of
// k_decode_fp8_sub (64/S chunks per wavefront, one per S-lane group, per-group rings of 16*S words, id lists,
// one buffer resource over the payload) with the exponent field decoded through the general 11-bit table
// (codes up to 16 bits, refill period 2, 4 or 8) and a sign+mantissa field that is raw or flat coded.  A row is
// 8 values per lane: 8 exponent symbols and 8 sign+mantissa bytes (two words, as in the FP8 kernel).
template <int S, bool XOR>
__global__ __launch_bounds__(256) void k_decode_bf16_sub(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single,
                                                         uint32_t slots_per_group)
{
    constexpr uint32_t kGroups = 64 / S;
    constexpr uint32_t kSeg = 4 * S, kRing = 16 * S;             // words per group
    __shared__ FieldTab tab;
    __shared__ __attribute__((aligned(16))) uint32_t ring[kWavesPerGroup][kRingWords];
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = blockIdx.x * slots_per_group; }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    build_field_tab(tab, d.comp + d.table_off[0], 256, d.lmax[0]);

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t s = lane & (S - 1), grp = lane / S;
    const uint64_t gmask = ((1ull << S) - 1) << (lane - s);
    const uint32_t cb = uniform32(d.chunk_bytes);                // two bytes per element
    const uint64_t n_elems = uniform64(d.n_elems);
    const uint32_t n_full = (uint32_t)(n_elems / (cb / 2));
    const uint32_t *ids = reinterpret_cast<const uint32_t *>(uniform64((uint64_t)d.ids));
    const uint64_t dst_bytes = uniform64(d.dst_bytes);
    const uint32_t n_slots = ids ? uniform32(d.n_ids) : uniform32(d.n_chunks);
    const uint8_t *comp = reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.comp));
    const uint64_t payload = uniform64(d.payload_off), total = uniform64(d.total_bytes);
    if (total < payload || total - payload > 0xFFFFFFF0ull || dst_bytes > 0xFFFFFFF0ull) return;   // the host never launches this
    const uint32_t pay_bytes = (uint32_t)(total - payload);
    const __amdgpu_buffer_rsrc_t ps = make_rsrc(comp + payload, pay_bytes);
    const __amdgpu_buffer_rsrc_t ds = make_rsrc(reinterpret_cast<uint8_t *>(uniform64((uint64_t)d.dst)), (uint32_t)dst_bytes);
    const uint64_t base_bytes = XOR ? n_elems * 2 : 0;
    const __amdgpu_buffer_rsrc_t bs = make_rsrc(XOR ? reinterpret_cast<const uint8_t *>(uniform64((uint64_t)d.base)) : comp,
                                                base_bytes > 0xFFFFFFF0ull ? 0u : (uint32_t)base_bytes);
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[0]));
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(comp + uniform32(d.index_off[1]));
    const bool sm_raw = uniform32(d.kind[1]) == 2;
    const uint32_t period = uniform32(d.period[0]);
    const bool has_long = uniform32(tab.lmax) > (uint32_t)kLutBits;
    const uint32_t rows = cb / (16 * S);
    const uint32_t mask = uniform32(tab.mask);
    const char *lut = reinterpret_cast<const char *>(tab.lut);
    char *const ring_bytes = reinterpret_cast<char *>(&ring[wave][0]) + grp * (kRing * 4);
    HuffStream Hl;                                               // only its limits are used (long_code)
#pragma unroll
    for (int i = 0; i < 4; i++) Hl.lim[i] = uniform32(tab.limit[kLutBits + 1 + i]);

    // the workgroup owns slots [first, first + slots_per_group): each pass takes 4 waves x kGroups of them
    for (uint32_t pass = 0; pass * kWavesPerGroup * kGroups < slots_per_group; pass++) {
        const uint32_t slot = it.first + (pass * kWavesPerGroup + wave) * kGroups + grp;
        uint32_t chunk = slot;
        bool alive = slot < n_slots && (pass * kWavesPerGroup + wave) * kGroups + grp < slots_per_group;
        if (ids && alive) chunk = ids[slot];
        alive = alive && chunk < n_full;                         // short last chunk: the host sends it to the generic kernel
        uint32_t e_off = pay_bytes, m_off = pay_bytes;           // out of range: loads return 0
        uint32_t e_len = 0;                                      // bytes of the exponent stream
        if (alive) {
            const uint64_t a0 = index0[chunk], b0 = index0[chunk + 1], a1 = index1[chunk], b1 = index1[chunk + 1];
            if (a0 <= b0 && a1 <= b1 && 16 * b1 <= pay_bytes && 16 * b0 <= pay_bytes && (b1 - a1) * 16 >= cb / 2) {
                e_off = (uint32_t)(16 * a0); m_off = (uint32_t)(16 * a1); e_len = (uint32_t)(16 * (b0 - a0));
            } else alive = false;
        }
        // the ring reads ahead of what is consumed: a piece past the end of this chunk's stream is not fetched
        auto ring_piece = [&](uint32_t word) -> u32x4 {
            return __builtin_amdgcn_raw_buffer_load_b128(ps, (int)(word * 4 < e_len ? e_off + word * 4 : pay_bytes), 0, 0);
        };
        const uint32_t out_off = slot * cb, base_off = chunk * cb;
        // ring prologue: the group's first 16*S words (each lane 4 loads of 16 bytes)
#pragma unroll
        for (uint32_t q = 0; q < 4; q++) {
            const u32x4 v = ring_piece(q * kSeg + s * 4);
            *reinterpret_cast<u32x4 *>(ring_bytes + (q * kSeg + s * 4) * 4) = v;
        }
        uint64_t W = (uint64_t)(*reinterpret_cast<const uint32_t *>(ring_bytes + s * 4)) << 32;    // step 0: lane s takes word s
        uint32_t c = 32, wpos = S, wbase = 0, pslot = 0;
        bool pending = false;
        u32x4 pv = {0, 0, 0, 0};
        // one refill period of R exponent symbols into bytes first .. first+R-1 of ex[]
        auto decode_period = [&](auto r_tag, int first, uint32_t ex[2]) {
            constexpr int R = decltype(r_tag)::value;
            const uint32_t x0 = (uint32_t)(W >> c);
            uint32_t x = x0, e[R];
#pragma unroll
            for (int j = 0; j < R; j++) {
                e[j] = *reinterpret_cast<const uint16_t *>(lut + ((x & mask) << 1));
                x >>= (e[j] & 31u);
            }
            if (R == 2 && has_long) {
                // an empty entry stands for a code longer than the index; it shifts by nothing, so the last one tells
                if (__any(e[R - 1] == 0)) {
                    x = x0;
#pragma unroll
                    for (int j = 0; j < R; j++) {
                        e[j] = *reinterpret_cast<const uint16_t *>(lut + ((x & mask) << 1));
                        if (e[j] == 0) e[j] = long_code(tab, Hl, x);
                        x >>= (e[j] & 31u);
                    }
                }
            }
            uint32_t used = 0;
#pragma unroll
            for (int j = 0; j < R; j++) {
                const int jj = first + j, pos = jj % 4;
                used += e[j];
                const uint32_t sel = pos == 0 ? 0x03020105u : pos == 1 ? 0x03020500u : pos == 2 ? 0x03050100u : 0x05020100u;
                ex[jj / 4] = __builtin_amdgcn_perm(e[j], ex[jj / 4], sel);      // byte 1 of the entry (the symbol) into byte pos
            }
            c += used & 0xFFu;
            const bool need = c >= 32;
            const uint64_t bm = __ballot(need) & gmask;
            const uint32_t w = *reinterpret_cast<const uint32_t *>(ring_bytes + ((prefix_count64(bm) + wpos) & (kRing - 1)) * 4);
            W = need ? ((W >> 32) | ((uint64_t)w << 32)) : W;
            c = need ? c - 32 : c;
            wpos += (uint32_t)__popcll(bm);
        };
        for (uint32_t row = 0; row < rows; row++) {
            if (pending) { *reinterpret_cast<u32x4 *>(ring_bytes + (pslot + s * 4) * 4) = pv; pending = false; }
            if (wpos - wbase >= kSeg) {
                pv = ring_piece(wbase + kRing + s * 4);
                pslot = wbase & (kRing - 1);
                wbase += kSeg;
                pending = true;
            }
            // ---- sign+mantissa: 8 bytes per lane and row
            uint32_t m[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                if (sm_raw) m[h] = __builtin_amdgcn_raw_buffer_load_b32(ps, (int)(m_off + ((row * S + s) * 2 + h) * 4), 0, 0);
                else m[h] = reverse_in_groups<8>(__builtin_amdgcn_raw_buffer_load_b32(ps, (int)(m_off + ((row * 2 + h) * S + s) * 4), 0, 0));
            }
            // ---- exponents
            uint32_t ex[2] = {0, 0};
            if (period == 2) {
#pragma unroll
                for (int g = 0; g < 4; g++) decode_period(std::integral_constant<int, 2>{}, g * 2, ex);
            } else if (period == 4) {
#pragma unroll
                for (int g = 0; g < 2; g++) decode_period(std::integral_constant<int, 4>{}, g * 4, ex);
            } else decode_period(std::integral_constant<int, 8>{}, 0, ex);
            const uint4 j = join_run4<ZC_FMT_BF16>((uint64_t)ex[0] | ((uint64_t)ex[1] << 32), 0, (uint64_t)m[0] | ((uint64_t)m[1] << 32), 0);
            u32x4 v = {j.x, j.y, j.z, j.w};
            if (XOR) v ^= __builtin_amdgcn_raw_buffer_load_b128(bs, (int)(base_off + (row * S + s) * 16), 0, 0);
            if (alive) __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(out_off + (row * S + s) * 16), 0, 0);
        }
    }
}

template <int S>
static int launch_bf16_sub_s(bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single,
                             uint32_t slots_per_group, hipStream_t st)
{
    if (xor_delta) hipLaunchKernelGGL((k_decode_bf16_sub<S, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    else hipLaunchKernelGGL((k_decode_bf16_sub<S, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, slots_per_group);
    return (int)hipGetLastError();
}

// BF16, S in {4, 8, 16, 32}, full chunks, exponent field table decoded, sign+mantissa flat or raw
int launch_decode_bf16_sub(uint32_t streams, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, uint32_t slots_per_group, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    switch (streams) {
    case 4: return launch_bf16_sub_s<4>(xor_delta, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 8: return launch_bf16_sub_s<8>(xor_delta, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 16: return launch_bf16_sub_s<16>(xor_delta, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    case 32: return launch_bf16_sub_s<32>(xor_delta, d_descs, d_work, n_work, s, use_single, slots_per_group, st);
    }
    return (int)hipErrorInvalidValue;
}

template <int EK, int MK>
static int launch_fp8_x(bool xor_delta, bool with_ids, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single, hipStream_t st)
{
    if (with_ids) {
        if (xor_delta) hipLaunchKernelGGL((k_decode_fp8<EK, MK, true, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
        else hipLaunchKernelGGL((k_decode_fp8<EK, MK, false, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    } else {
        if (xor_delta) hipLaunchKernelGGL((k_decode_fp8<EK, MK, true, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
        else hipLaunchKernelGGL((k_decode_fp8<EK, MK, false, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    }
    return (int)hipGetLastError();
}

// exp_kind: 0 = single lookups, 1 = pair lookups; sm_kind: 0 = flat code, 1 = raw; with_ids: some tensor has a list of
// chunk ids (the build that looks for one)
int launch_decode_fp8_fast(int exp_kind, int sm_kind, bool xor_delta, bool with_ids, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    if (exp_kind == 0 && sm_kind == 0) return launch_fp8_x<0, 0>(xor_delta, with_ids, d_descs, d_work, n_work, s, use_single, st);
    if (exp_kind == 0 && sm_kind == 1) return launch_fp8_x<0, 1>(xor_delta, with_ids, d_descs, d_work, n_work, s, use_single, st);
    if (exp_kind == 1 && sm_kind == 0) return launch_fp8_x<1, 0>(xor_delta, with_ids, d_descs, d_work, n_work, s, use_single, st);
    return launch_fp8_x<1, 1>(xor_delta, with_ids, d_descs, d_work, n_work, s, use_single, st);
}

}  // namespace zc
