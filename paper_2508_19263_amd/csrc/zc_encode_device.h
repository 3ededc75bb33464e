// Device helpers shared by the specialised histogram, size and encode kernels (zc_encode_fast.hip, zc_hist_lanes.hip,
// zc_encode_pages.hip): wave-uniform values, buffer resources, and the table lookups that join the codes of two or more
// symbols.  Everything lives in an unnamed namespace, so every file has a copy of its own.
#pragma once

#include "zc_internal.h"
#include "zc_device.h"

namespace zc {

namespace {


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t uni32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uni64(uint64_t v) { return ((uint64_t)uni32((uint32_t)(v >> 32)) << 32) | (uint64_t)uni32((uint32_t)v); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// (x.byte[B]) << 2: LDS byte offset of a 32-bit table entry
template <int B>
__device__ __forceinline__ uint32_t byte_times4(uint32_t x, uint32_t two)
{
    static_assert(B >= 0 && B < 4, "byte of a word");
    uint32_t r;
    if (B == 0) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(two), "v"(x));
    else if (B == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(two), "v"(x));
    else if (B == 2) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(two), "v"(x));
    else asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(two), "v"(x));
    return r;
}
// the same with the byte's number as a value that is constant once the caller's loop is unrolled
__device__ __forceinline__ uint32_t byte_times4(uint32_t x, int b, uint32_t two)
{
    switch (b & 3) {
    case 0: return byte_times4<0>(x, two);
    case 1: return byte_times4<1>(x, two);
    case 2: return byte_times4<2>(x, two);
    default: return byte_times4<3>(x, two);
    }
}

// Two entries of an encode table (bits 15..0 the code, first bit lowest; bits 20..16 its length) joined into
// the code of both symbols and its length, with the halves of the entries as operands:
// code = a.lo | b.lo << a.hi (a.hi <= 16), len = a.hi + b.hi.
__device__ __forceinline__ void join_codes(uint32_t a, uint32_t b, uint32_t &code, uint32_t &len)
{
    uint32_t sh;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:WORD_0" : "=v"(sh) : "v"(a), "v"(b));
    asm("v_or_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(code) : "v"(sh), "v"(a));
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:WORD_1" : "=v"(len) : "v"(a), "v"(b));
}

// code and length of the four exponents of one source word: bits 15..0 of an entry are the
// two codes of a byte pair (first symbol in the low bits), bits 20..16 their total length
__device__ __forceinline__ void group_code(uint32_t w, const char *pair_lut, uint32_t two, uint32_t &code, uint32_t &len)
{
    const uint32_t t = (w >> 3) & 0x0F0F0F0Fu;          // exponent of every byte
    const uint32_t u = t | (t >> 4);                    // bytes 0 and 2: e0 | e1 << 4, e2 | e3 << 4
    const uint32_t a = *reinterpret_cast<const uint32_t *>(pair_lut + byte_times4<0>(u, two));
    const uint32_t b = *reinterpret_cast<const uint32_t *>(pair_lut + byte_times4<2>(u, two));
    join_codes(a, b, code, len);
}


// The R codes of one refill period of a BF16 field joined into one code (at most 32 bits) and its length: bytes
// first .. first+R-1 of the 8 symbol bytes in w, looked up in the field's 256-entry table, joined in pairs, then
// pairs of pairs.
template <int R>
__device__ __forceinline__ void codes_of_period(const uint32_t w[2], int first, const char *lut, uint32_t &code_out, uint32_t &len_out)
{
    static_assert(R == 2 || R == 4 || R == 8, "symbols are joined in pairs, then pairs of pairs");
    const uint32_t two = 2;
    uint32_t code[R / 2], len[R / 2];
#pragma unroll
    for (int j = 0; j < R / 2; j++) {
        const int jj = first + 2 * j;
        const uint32_t a = *reinterpret_cast<const uint32_t *>(lut + byte_times4(w[jj / 4], jj % 4, two));
        const uint32_t b = *reinterpret_cast<const uint32_t *>(lut + byte_times4(w[(jj + 1) / 4], (jj + 1) % 4, two));
        join_codes(a, b, code[j], len[j]);
    }
#pragma unroll
    for (int n = R / 2; n > 1; n /= 2)
#pragma unroll
        for (int j = 0; j < n / 2; j++) {
            code[j] = code[2 * j] | (code[2 * j + 1] << len[2 * j]);
            len[j] = len[2 * j] + len[2 * j + 1];
        }
    code_out = code[0]; len_out = len[0];
}

}  // namespace

}  // namespace zc
