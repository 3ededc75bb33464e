// Device-side helpers shared by the kernels of the HIP library (zc_kernels.hip,
// zc_decode_fast.hip).  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>

#include "zc_internal.h"

namespace zc {

// ------------------------------------------------------------------ lane helpers

struct Lanes {
    uint32_t lane, s, grp;     // lane in wave, lane in its S-lane group, group in wave
    uint64_t gmask;            // wave mask of the lanes of this group
};

__device__ __forceinline__ Lanes make_lanes(uint32_t S)
{
    Lanes L;
    L.lane = threadIdx.x & 63;
    L.s = L.lane & (S - 1);
    L.grp = L.lane / S;
    L.gmask = (S == 64) ? ~0ull : (((1ull << S) - 1) << (L.lane - L.s));
    return L;
}

// number of set bits of m in lanes below this one
__device__ __forceinline__ uint32_t prefix_count(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// EB element bits, EPR elements per 16-byte run, GRP field values per coded symbol, G symbols per run,
// SB symbol bits, NF fields, BASE the element format (whose split and join the format uses)
template <int FMT> struct Fmt;
// SCALE elements share one scale byte (1 where the format has none: never used there)
template <> struct Fmt<ZC_FMT_BF16> { static constexpr int EB = 16, EPR = 8, GRP = 1, G = 8, SB = 8, NF = 2, BASE = ZC_FMT_BF16, SCALE = 1; };
template <> struct Fmt<ZC_FMT_FP8_E4M3> { static constexpr int EB = 8, EPR = 16, GRP = 1, G = 16, SB = 4, NF = 2, BASE = ZC_FMT_FP8_E4M3, SCALE = 1; };
template <> struct Fmt<ZC_FMT_FP4_E2M1_MX> { static constexpr int EB = 4, EPR = 32, GRP = 1, G = 32, SB = 2, NF = 3, BASE = ZC_FMT_FP4_E2M1_MX, SCALE = 32; };
template <> struct Fmt<ZC_FMT_FP4_E2M1_NV> { static constexpr int EB = 4, EPR = 32, GRP = 1, G = 32, SB = 2, NF = 3, BASE = ZC_FMT_FP4_E2M1_MX, SCALE = 16; };
// byte-grouped symbols: the packed field words are those of the element format, read 8 bits at a time
// E5M2: 16 symbols of 8 bits per run and field, i.e. two 64-bit words per field (P, Q)
template <> struct Fmt<ZC_FMT_FP8_E5M2> { static constexpr int EB = 8, EPR = 16, GRP = 1, G = 16, SB = 8, NF = 2, BASE = ZC_FMT_FP8_E5M2, SCALE = 1; };
template <> struct Fmt<ZC_FMT_FP8_E4M3_BYTES> { static constexpr int EB = 8, EPR = 16, GRP = 2, G = 8, SB = 8, NF = 2, BASE = ZC_FMT_FP8_E4M3, SCALE = 1; };
template <> struct Fmt<ZC_FMT_FP4_E2M1_MX_BYTES> { static constexpr int EB = 4, EPR = 32, GRP = 4, G = 8, SB = 8, NF = 3, BASE = ZC_FMT_FP4_E2M1_MX, SCALE = 32; };

// ------------------------------------------------- field split / join of one 16-byte run
// P0 = the run's exponent symbols, P1 = its sign+mantissa symbols, SB bits each, symbol j at
// bits j*SB (always 64 bits per field per run).

__device__ __forceinline__ uint32_t pack_nibbles_of_bytes(uint32_t x)   // 4 bytes with a value < 16 each -> 16 bits
{
    x = (x | (x >> 4)) & 0x00FF00FFu;
    return (x | (x >> 8)) & 0xFFFFu;
}
__device__ __forceinline__ uint32_t pack_pairs_of_nibbles(uint32_t x)   // 8 nibbles with a value < 4 each -> 16 bits
{
    x = (x | (x >> 2)) & 0x0F0F0F0Fu;
    return pack_nibbles_of_bytes(x);
}
__device__ __forceinline__ uint32_t spread_nibbles_to_bytes(uint32_t x)  // inverse of pack_nibbles_of_bytes
{
    x = (x | (x << 8)) & 0x00FF00FFu;
    return (x | (x << 4)) & 0x0F0F0F0Fu;
}
__device__ __forceinline__ uint32_t spread_pairs_to_nibbles(uint32_t x)  // inverse of pack_pairs_of_nibbles
{
    x = spread_nibbles_to_bytes(x);
    return (x | (x << 2)) & 0x33333333u;
}

template <int FMT_>
__device__ __forceinline__ void split_run(const uint4 &v, uint64_t &P0, uint64_t &P1)
{
    constexpr int FMT = Fmt<FMT_>::BASE;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    P0 = 0; P1 = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t e, m;
        if (FMT == ZC_FMT_BF16) {                       // s eeeeeeee mmmmmmm, two per word
            uint32_t lo = w[i] & 0xFFFFu, hi = w[i] >> 16;
            e = ((lo >> 7) & 0xFFu) | (((hi >> 7) & 0xFFu) << 8);
            m = (((lo >> 8) & 0x80u) | (lo & 0x7Fu)) | ((((hi >> 8) & 0x80u) | (hi & 0x7Fu)) << 8);
        } else if (FMT == ZC_FMT_FP8_E4M3) {            // s eeee mmm, four per word
            e = pack_nibbles_of_bytes((w[i] >> 3) & 0x0F0F0F0Fu);
            m = pack_nibbles_of_bytes(((w[i] >> 4) & 0x08080808u) | (w[i] & 0x07070707u));
        } else {                                        // s ee m, eight per word
            e = pack_pairs_of_nibbles((w[i] >> 1) & 0x33333333u);
            m = pack_pairs_of_nibbles(((w[i] >> 2) & 0x22222222u) | (w[i] & 0x11111111u));
        }
        P0 |= (uint64_t)e << (16 * i);
        P1 |= (uint64_t)m << (16 * i);
    }
}

template <int FMT_>
__device__ __forceinline__ uint4 join_run(uint64_t P0, uint64_t P1)
{
    constexpr int FMT = Fmt<FMT_>::BASE;
    uint32_t w[4];
    if (FMT == ZC_FMT_BF16) {
        // two values per word: a byte permute pairs every exponent byte (high) with its sign+mantissa byte (low);
        // then, in both halves at once, the exponent moves down one bit, the low 7 bits stay and the sign moves up 8
        const uint32_t e[2] = {(uint32_t)P0, (uint32_t)(P0 >> 32)}, m[2] = {(uint32_t)P1, (uint32_t)(P1 >> 32)};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint32_t a = __builtin_amdgcn_perm(e[i / 2], m[i / 2], (i & 1) ? 0x07030602u : 0x05010400u);
            const uint32_t u = ((a >> 1) & 0x7F807F80u) | (a & ~0x7F807F80u);      // bit 15 of each half is still the exponent's top bit
            w[i] = (u & 0x7FFF7FFFu) | ((a << 8) & ~0x7FFF7FFFu);
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t e = (uint32_t)(P0 >> (16 * i)) & 0xFFFFu, m = (uint32_t)(P1 >> (16 * i)) & 0xFFFFu;
        if (FMT == ZC_FMT_FP8_E4M3) {
            uint32_t eb = spread_nibbles_to_bytes(e), mb = spread_nibbles_to_bytes(m);
            w[i] = ((mb & 0x08080808u) << 4) | (eb << 3) | (mb & 0x07070707u);
        } else {
            uint32_t en = spread_pairs_to_nibbles(e), mn = spread_pairs_to_nibbles(m);
            w[i] = ((mn & 0x22222222u) << 2) | (en << 1) | (mn & 0x11111111u);
        }
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The same for any format: a field's symbols of one run in (P, Q); Q is used only by formats whose run is
// 16 symbols of 8 bits (E5M2), where P holds symbols 0..7 and Q symbols 8..15.
template <int FMT>
__device__ __forceinline__ void split_run4(const uint4 &v, uint64_t &P0, uint64_t &Q0, uint64_t &P1, uint64_t &Q1)
{
    if (FMT == ZC_FMT_FP8_E5M2) {                       // s eeeee mm, four per word, one byte per symbol
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t e[4], m[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            e[i] = (w[i] >> 2) & 0x1F1F1F1Fu;
            m[i] = ((w[i] >> 5) & 0x04040404u) | (w[i] & 0x03030303u);
        }
        P0 = (uint64_t)e[0] | ((uint64_t)e[1] << 32); Q0 = (uint64_t)e[2] | ((uint64_t)e[3] << 32);
        P1 = (uint64_t)m[0] | ((uint64_t)m[1] << 32); Q1 = (uint64_t)m[2] | ((uint64_t)m[3] << 32);
    } else {
        constexpr int F = FMT == ZC_FMT_FP8_E5M2 ? ZC_FMT_FP8_E4M3 : FMT;
        split_run<F>(v, P0, P1);
        Q0 = 0; Q1 = 0;
    }
}

template <int FMT>
__device__ __forceinline__ uint4 join_run4(uint64_t P0, uint64_t Q0, uint64_t P1, uint64_t Q1)
{
    if (FMT == ZC_FMT_FP8_E5M2) {
        const uint32_t e[4] = {(uint32_t)P0, (uint32_t)(P0 >> 32), (uint32_t)Q0, (uint32_t)(Q0 >> 32)};
        const uint32_t m[4] = {(uint32_t)P1, (uint32_t)(P1 >> 32), (uint32_t)Q1, (uint32_t)(Q1 >> 32)};
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = ((m[i] & 0x04040404u) << 5) | ((e[i] & 0x1F1F1F1Fu) << 2) | (m[i] & 0x03030303u);
        return make_uint4(w[0], w[1], w[2], w[3]);
    } else {
        constexpr int F = FMT == ZC_FMT_FP8_E5M2 ? ZC_FMT_FP8_E4M3 : FMT;
        return join_run<F>(P0, P1);
    }
}

// 16 bytes from p, of which only the first `valid` may be read
__device__ __forceinline__ uint4 load_run(const uint8_t *p, uint32_t valid)
{
    if (valid >= 16) return *reinterpret_cast<const uint4 *>(p);
    uint32_t w[4] = {0, 0, 0, 0};
    for (uint32_t i = 0; i < valid; i++) w[i >> 2] |= (uint32_t)p[i] << (8 * (i & 3));
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ void store_run(uint8_t *p, const uint4 &v, uint32_t valid)
{
    if (valid >= 16) { *reinterpret_cast<uint4 *>(p) = v; return; }
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    for (uint32_t i = 0; i < valid; i++) p[i] = (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
}

__device__ __forceinline__ uint4 xor4(const uint4 &a, const uint4 &b) { return make_uint4(a.x ^ b.x, a.y ^ b.y, a.z ^ b.z, a.w ^ b.w); }

// Tables of one field in LDS: a direct lookup on the next kLutBits stream bits and the
// canonical first-code arrays for the rare codes longer than that.

constexpr int kLutBits = 11;

struct FieldTab {
    uint16_t lut[1 << kLutBits];   // (symbol << 8) | length, 0 = code longer than the index
    uint32_t first[17], cnt[17], start[17];
    // for the codes longer than the index, by length l: limit = (first + cnt) << (16 - l), the left-aligned
    // exclusive upper bound of all codes of length <= l (non-decreasing in l); rebase = start - first
    uint32_t limit[17], rebase[17];
    uint8_t sorted[256];
    uint8_t len[256];
    uint32_t mask;                 // (1 << min(Lmax, kLutBits)) - 1
    uint32_t lmax;
};

// all threads of the workgroup; lengths come from the container's table
__attribute__((unused)) static __device__ void build_field_tab(FieldTab &T, const uint8_t *len_table, int alphabet, uint32_t lmax)
{
    const uint32_t tid = threadIdx.x, nt = blockDim.x;
    if (tid < 17) T.cnt[tid] = 0;
    for (uint32_t v = tid; v < 256; v += nt) T.len[v] = v < (uint32_t)alphabet ? len_table[v] : 0;
    if (lmax > 16) lmax = 16;
    __syncthreads();
    for (uint32_t v = tid; v < (uint32_t)alphabet; v += nt)
        if (T.len[v] && T.len[v] <= 16) atomicAdd(&T.cnt[T.len[v]], 1u);
    __syncthreads();
    if (tid == 0) {
        uint32_t code = 0, idx = 0;
        for (int l = 1; l <= 16; l++) {
            code <<= 1;
            T.first[l] = code; T.start[l] = idx;
            T.rebase[l] = idx - code;
            code += T.cnt[l]; idx += T.cnt[l];
            T.limit[l] = code << (16 - l);
        }
        T.limit[0] = 0; T.rebase[0] = 0;
        const uint32_t bits = lmax < (uint32_t)kLutBits ? lmax : (uint32_t)kLutBits;
        T.mask = (1u << bits) - 1;
        T.lmax = lmax;
    }
    __syncthreads();
    for (uint32_t v = tid; v < (uint32_t)alphabet; v += nt) {
        const uint32_t l = T.len[v];
        if (l && l <= 16) {
            uint32_t rank = 0;
            for (uint32_t u = 0; u < v; u++) rank += T.len[u] == l;
            T.sorted[T.start[l] + rank] = (uint8_t)v;
        }
    }
    __syncthreads();
    const uint32_t bits = lmax < (uint32_t)kLutBits ? lmax : (uint32_t)kLutBits;
    for (uint32_t idx = tid; idx < (1u << bits); idx += nt) {
        const uint32_t msb = __brev(idx);                  // stream bits in code order, left aligned
        uint32_t entry = 0;
        for (uint32_t l = 1; l <= bits; l++) {
            const uint32_t code = msb >> (32 - l);
            if (code - T.first[l] < T.cnt[l] && code >= T.first[l]) { entry = l | ((uint32_t)T.sorted[T.start[l] + code - T.first[l]] << 8); break; }
        }
        T.lut[idx] = (uint16_t)entry;
    }
    __syncthreads();
}

// Code longer than the lookup index (12..16 bits), without a search: in a canonical code the left-aligned
// codes of length <= l all lie below limit[l], so the length is 12 plus the number of those limits that the
// next 16 stream bits reach, and the symbol's rank follows from the code value.  A malformed table can only
// give a wrong symbol: the index is masked.
__attribute__((unused)) static __device__ __noinline__ uint32_t dec_long(const FieldTab &T, uint32_t x)
{
    static_assert(kLutBits == 11, "four limits cover the lengths 12..15; 16 is what is left");
    const uint32_t w = __brev(x) >> 16;                    // the next 16 stream bits in code order
    const uint32_t len = 12u + (w >= T.limit[12]) + (w >= T.limit[13]) + (w >= T.limit[14]) + (w >= T.limit[15]);
    return len | ((uint32_t)T.sorted[(T.rebase[len] + (w >> (16u - len))) & 255u] << 8);
}

// every symbol of a 64-bit packed run equal to v
__device__ __forceinline__ uint64_t splat(uint32_t v, int sb)
{
    uint64_t x = v;
    for (int w = sb; w < 64; w *= 2) x |= x << w;
    return x;
}


// Rows of a chunk that the four wavefronts of a workgroup share (fields stored plainly, so rows do not depend on each
// other).  The first wavefront also takes the chunk's block scales, scale_rows rows of 1024 of them, whose table-driven
// coding costs about kScaleRowCost element rows each: it gets fewer element rows, the others a third of the rest each.
constexpr uint32_t kScaleRowCost = 3;
__device__ __forceinline__ void shared_chunk_rows(uint32_t rows, uint32_t scale_rows, uint32_t wave, uint32_t &begin, uint32_t &end)
{
    const uint32_t extra = scale_rows * kScaleRowCost;
    const uint32_t first = rows > 3 * extra ? (rows - 3 * extra) / 4 : 0u;         // first + extra = (rows - first) / 3
    const uint32_t rest = rows - first;
    begin = wave == 0 ? 0u : first + (wave - 1) * rest / 3;
    end = wave == 0 ? first : first + wave * rest / 3;
}


// reverse the bit order inside every SB-bit group of a word (a flat code is the symbol value
// written most significant bit first into an LSB-first string)
template <int SB>
__device__ __forceinline__ uint32_t reverse_in_groups(uint32_t w)
{
    if (SB == 8) return __builtin_amdgcn_perm(0, __brev(w), 0x00010203u);          // all bits reversed, then bytes back in order
    if (SB == 4) { w = ((w >> 1) & 0x55555555u) | ((w & 0x55555555u) << 1); return ((w >> 2) & 0x33333333u) | ((w & 0x33333333u) << 2); }
    return ((w >> 1) & 0x55555555u) | ((w & 0x55555555u) << 1);
}


}  // namespace zc
