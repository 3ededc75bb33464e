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

}  // namespace

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

// ---------------------------------------------------------------------------------------
// Histogram and stream sizes of FP8 chunks in two reads of the source instead of three.  With 64 lanes per chunk
// a lane owns every 64th 16-byte run, and the number of words its stream takes follows from its bit total alone
// (shown at k_sizes_fp8_counts).  So the histogram pass, which reads the chunk anyway, also counts the exponents
// per lane (16 counts of 16 bits per lane, 2 KiB per chunk of 256 KiB), and once the code is known the size pass
// reads those counts instead of the source.
//
// k_hist_fp8_lanes: one workgroup per whole chunk of kHistBlockBytes (= the chunk size; the host uses this kernel
// for no other).  Thread t takes the runs t, t+256, ...: all of chunk lane t % 64, which it shares with three
// threads of the other wavefronts.  Every chunk lane has a histogram of all 256 byte values in LDS (16-bit
// counters, lanes l and l + 32 in the two halves of word [value][l % 32]: one atomic addition of a constant per
// byte; each half of a wavefront falls into 32 different banks, so nothing collides, whatever the data; a lane
// holds 4096 bytes, so nothing overflows).  At the end the lanes' histograms are folded into exponent counts
// per lane, which go to lane_counts, and into the chunk's two field histograms, which are added to the tensor's
// second histogram slot (exponents at 0..15, sign+mantissa at 16..31; the first slot keeps the byte histogram
// of what k_hist counts, a short last chunk).
__global__ __launch_bounds__(256) void k_hist_fp8_lanes(const TensorDev *descs, const WorkItem *work, uint64_t *hist, uint16_t *lane_counts)
{
    static_assert(kHistBlockBytes / 64 < 65536, "a lane's count of one byte value fits 16 bits");
    __shared__ uint32_t cnt[256 * 32];                            // 32 KiB
    const WorkItem it = work[blockIdx.x];
    const TensorDev &d = descs[it.tensor];
    const uint32_t tid = threadIdx.x, lane = tid & 63, quarter = tid >> 6;
    const uint64_t start = (uint64_t)it.first * kHistBlockBytes;
    if (d.chunk_bytes != kHistBlockBytes || start + kHistBlockBytes > d.n_elems) return;      // whole workgroup; the host never asks for this
    for (uint32_t i = tid; i < 256 * 32; i += 256) cnt[i] = 0;
    __syncthreads();
    const uint8_t *p = d.src + start;
    const uint8_t *base = d.base ? d.base + start : nullptr;
    // byte value b of lane l: word b * 32 + l % 32, half l / 32 (the same for everything a thread counts)
    const uint32_t l4 = (lane & 31) * 4, inc = lane < 32 ? 1u : 0x10000u;
    char *const lds = reinterpret_cast<char *>(cnt);
    auto count = [&](const uint4 &v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            atomicAdd(reinterpret_cast<uint32_t *>(lds + (((w[i] << 7) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds + (((w[i] >> 1) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds + (((w[i] >> 9) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds + (((w[i] >> 17) & 0x7F80u) | l4)), inc);
        }
    };
    // eight 16-byte loads per thread in flight at a time
    constexpr uint32_t kStep = 256 * 16, kDepth = 8;
    static_assert(kHistBlockBytes % (kStep * kDepth) == 0, "whole rounds");
    for (uint32_t off = tid * 16; off < kHistBlockBytes; off += kDepth * kStep) {
        uint4 v[kDepth];
#pragma unroll
        for (uint32_t k = 0; k < kDepth; k++) v[k] = *reinterpret_cast<const uint4 *>(p + off + k * kStep);
        if (base) {
#pragma unroll
            for (uint32_t k = 0; k < kDepth; k++) v[k] = xor4(v[k], *reinterpret_cast<const uint4 *>(base + off + k * kStep));
        }
#pragma unroll
        for (uint32_t k = 0; k < kDepth; k++) count(v[k]);
    }
    __syncthreads();
    // Thread (lane, quarter) folds the byte values 64*quarter .. +63 of its lane: value = s eeee mmm, so a quarter
    // is one sign, eight exponents and all eight mantissas.
    uint32_t ce[8], cm[8];
#pragma unroll
    for (int i = 0; i < 8; i++) { ce[i] = 0; cm[i] = 0; }
    const uint32_t half_shift = lane < 32 ? 0u : 16u;
#pragma unroll
    for (int v = 0; v < 64; v++) {
        const uint32_t c = (cnt[(quarter * 64 + v) * 32 + (lane & 31)] >> half_shift) & 0xFFFFu;
        ce[v >> 3] += c;
        cm[v & 7] += c;
    }
    const uint32_t e0 = (quarter & 1) * 8, s = quarter >> 1;      // the quarter's first exponent and its sign
    __syncthreads();                                             // every thread has read its part of cnt: the array is free
    // the exponent counts of (lane, quarter), in rows of 9 words against bank conflicts
    uint32_t *const part = cnt;
#pragma unroll
    for (int i = 0; i < 8; i++) part[(quarter * 64 + lane) * 9 + i] = ce[i];
    // the chunk's field histograms: every lane of this wavefront holds partial counts of the same 16 symbols.  They are
    // summed over the lanes in a butterfly that halves what a lane carries at every step (8, 4, 2 and 1 exchanges, then
    // two more of the one value left), so that lane j < 16 ends with the total of symbol j.
    {
        uint32_t c[16];
#pragma unroll
        for (int i = 0; i < 8; i++) { c[i] = ce[i]; c[8 + i] = cm[i]; }
#pragma unroll
        for (int step = 0; step < 4; step++) {
            const int n = 8 >> step;                             // values kept per lane after this step
            const bool upper = (lane >> step) & 1;
#pragma unroll
            for (int i = 0; i < n; i++) {
                const uint32_t give = upper ? c[i] : c[n + i], keep = upper ? c[n + i] : c[i];
                c[i] = keep + (uint32_t)__shfl_xor((int)give, 1 << step, 64);
            }
        }
        c[0] += (uint32_t)__shfl_xor((int)c[0], 16, 64);
        c[0] += (uint32_t)__shfl_xor((int)c[0], 32, 64);
        // bit `step` of the lane chose the half it kept at that step, i.e. bit 3 - step of the symbol
        const uint32_t sym = ((lane & 1) << 3) | ((lane & 2) << 1) | ((lane & 4) >> 1) | ((lane & 8) >> 3);
        if (lane < 16 && c[0]) {
            unsigned long long *slot = reinterpret_cast<unsigned long long *>(&hist[((uint64_t)it.tensor * 3 + 1) * 256]);
            atomicAdd(slot + (sym < 8 ? e0 + sym : 16 + s * 8 + (sym - 8)), (unsigned long long)c[0]);
        }
    }
    __syncthreads();
    // thread t writes the counts of exponents 4*(t/64) .. +3 of lane t%64: those came from the quarters with the
    // same exponent half (quarter & 1 == t/128), one per sign
    {
        const uint32_t s0 = quarter * 4, half = quarter >> 1, i0 = s0 & 7;
        const uint32_t *pa = part + ((half + 0) * 64 + lane) * 9 + i0, *pb = part + ((half + 2) * 64 + lane) * 9 + i0;
        const uint32_t c0 = pa[0] + pb[0], c1 = pa[1] + pb[1], c2 = pa[2] + pb[2], c3 = pa[3] + pb[3];
        const uint64_t chunk_global = (uint64_t)(d.units_off / 2) + it.first;      // two fields: units_off counts two entries per chunk
        const uint2 packed = make_uint2(c0 | (c1 << 16), c2 | (c3 << 16));
        *reinterpret_cast<uint2 *>(lane_counts + (chunk_global * 64 + lane) * 16 + s0) = packed;
    }
}

// Stream sizes of full chunks from the per-lane exponent counts.  The decoder of a lane asks for a word at a
// refill step (every 4 symbols) when it holds k <= 32 unread bits, one word per step at most.  With B(g) the bits
// of the lane's symbols before step g, the words asked for up to and including step g are min(g + 1,
// floor(B(g) / 32) + 2): by induction, since B grows by at most 32 per step (four codes of at most 8 bits).  The
// lane's total is that expression at its last step, where B is its bit total minus its last four codes.
__global__ __launch_bounds__(256) void k_sizes_fp8_counts(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables,
                                                          const uint16_t *lane_counts, uint32_t *units)
{
    __shared__ uint32_t len16[16];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (!dp->route) return;                                      // whole workgroup: the code does not suit this kernel
    if (threadIdx.x < 16) len16[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + threadIdx.x] >> 16;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = uni32(it.first + (threadIdx.x >> 6));
    const uint32_t E = uni32(dp->chunk_bytes);
    const uint64_t n_elems = uni64(dp->n_elems);
    if (E != kHistBlockBytes || chunk >= (uint32_t)(n_elems / E)) return;
    const uint64_t chunk_global = (uint64_t)(uni32(dp->units_off) / 2) + chunk;
    const uint4 *mine = reinterpret_cast<const uint4 *>(lane_counts + (chunk_global * 64 + lane) * 16);
    const uint4 c0 = mine[0], c1 = mine[1];
    const uint32_t c[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 8; j++) bits += (c[j] & 0xFFFFu) * len16[2 * j] + (c[j] >> 16) * len16[2 * j + 1];
    // the lane's last four symbols: the last word of its run in the chunk's last row
    const uint64_t at = (uint64_t)chunk * E + (E - 1024) + lane * 16 + 12;
    uint32_t w = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + at);
    if (uni64((uint64_t)dp->base) != 0) w ^= *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + at);
    const uint32_t last = len16[(w >> 3) & 15] + len16[(w >> 11) & 15] + len16[(w >> 19) & 15] + len16[(w >> 27) & 15];
    const uint32_t steps = E / 256;                              // 4 per row of 1 KiB
    uint32_t q = ((bits - last) >> 5) + 2;
    q = q < steps ? q : steps;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
    if (lane == 0) {
        uint32_t *my = units + uni32(dp->units_off);
        const uint32_t nc = uni32(dp->n_chunks);
        my[chunk] = (q + 3) / 4;
        my[nc + chunk] = E / 32;                            // 4 bits per element, 16-byte units (flat code and raw alike)
    }
}

// ---------------------------------------------------------------------------------------
// The same two reads instead of three for the formats whose fields are 8-bit symbols, 8 per 16-byte run (BF16;
// FP8 in byte symbols) or 16 (FP8 E5M2), with 64 lanes and chunks of kHistBlockBytes: weights, checkpoints and
// checkpoint deltas (Sec. 3.1, 3.2, 4.1).  A lane's field has 256 possible symbols, so its counts are 512 bytes per field and lane, 64 KiB
// per chunk: a quarter of the chunk, written once here and read once by k_sizes_rows8_counts, against a whole
// second read of the source (and of the base of a delta) by the generic size pass.
//
// k_hist_rows8_lanes: one workgroup of eight wavefronts per whole chunk.  Thread t takes the runs t, t + 512, ...:
// all of chunk lane t % 64.  LDS holds, per field, a histogram of the 256 symbols per lane in the layout of
// k_hist_fp8_lanes (16-bit counters, lanes l and l + 32 in the halves of word [symbol][l % 32]: conflict-free
// whatever the data; a lane holds 2,048 symbols of a field).  At the end the arrays go to lane_counts as they are
// (field, symbol, word: 64 KiB at lane_counts + chunk * 16384 words), and their sums over the lanes are added to the
// tensor's histograms, beside what k_hist counts.
template <int FMT>
__global__ __launch_bounds__(512) void k_hist_rows8_lanes(const TensorDev *descs, const WorkItem *work, uint64_t *hist, uint32_t *lane_counts)
{
    static_assert((Fmt<FMT>::G == 8 || Fmt<FMT>::G == 16) && Fmt<FMT>::SB == 8 && Fmt<FMT>::NF == 2, "two fields of 8 or 16 symbols of 8 bits per run");
    static_assert(kHistBlockBytes / 16 / 64 * Fmt<FMT>::G < 65536, "a lane's count of one symbol fits 16 bits");
    constexpr int kWords = Fmt<FMT>::G / 4;                      // words of four symbols per run and field
    __shared__ __attribute__((aligned(16))) uint32_t cnt[2 * 256 * 32];      // 64 KiB
    const WorkItem it = work[blockIdx.x];
    const TensorDev &d = descs[it.tensor];
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint64_t start = (uint64_t)it.first * kHistBlockBytes, nbytes = d.n_elems * (uint64_t)Fmt<FMT>::EB / 8;
    if (d.chunk_bytes != kHistBlockBytes || start + kHistBlockBytes > nbytes) return;          // whole workgroup; the host never asks for this
    uint4 *const cnt4 = reinterpret_cast<uint4 *>(cnt);
    for (uint32_t i = tid; i < 2 * 256 * 32 / 4; i += 512) cnt4[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    const uint8_t *p = d.src + start;
    const uint8_t *base = d.base ? d.base + start : nullptr;
    const uint32_t l4 = (lane & 31) * 4, inc = lane < 32 ? 1u : 0x10000u;
    char *const lds0 = reinterpret_cast<char *>(cnt), *const lds1 = lds0 + 256 * 32 * 4;
    auto count = [&](const uint4 &v) {
        uint64_t P0, Q0, P1, Q1;
        split_run4<FMT>(v, P0, Q0, P1, Q1);
        const uint32_t w0[4] = {(uint32_t)P0, (uint32_t)(P0 >> 32), (uint32_t)Q0, (uint32_t)(Q0 >> 32)};
        const uint32_t w1[4] = {(uint32_t)P1, (uint32_t)(P1 >> 32), (uint32_t)Q1, (uint32_t)(Q1 >> 32)};
#pragma unroll
        for (int i = 0; i < kWords; i++) {
            atomicAdd(reinterpret_cast<uint32_t *>(lds0 + (((w0[i] << 7) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds0 + (((w0[i] >> 1) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds0 + (((w0[i] >> 9) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds0 + (((w0[i] >> 17) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds1 + (((w1[i] << 7) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds1 + (((w1[i] >> 1) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds1 + (((w1[i] >> 9) & 0x7F80u) | l4)), inc);
            atomicAdd(reinterpret_cast<uint32_t *>(lds1 + (((w1[i] >> 17) & 0x7F80u) | l4)), inc);
        }
    };
    // eight 16-byte loads per thread in flight at a time
    constexpr uint32_t kStep = 512 * 16, kDepth = 8;
    static_assert(kHistBlockBytes % (kStep * kDepth) == 0, "whole rounds");
    for (uint32_t off = tid * 16; off < kHistBlockBytes; off += kDepth * kStep) {
        uint4 v[kDepth];
#pragma unroll
        for (uint32_t k = 0; k < kDepth; k++) v[k] = *reinterpret_cast<const uint4 *>(p + off + k * kStep);
        if (base) {
#pragma unroll
            for (uint32_t k = 0; k < kDepth; k++) v[k] = xor4(v[k], *reinterpret_cast<const uint4 *>(base + off + k * kStep));
        }
#pragma unroll
        for (uint32_t k = 0; k < kDepth; k++) count(v[k]);
    }
    __syncthreads();
    // the counts per lane, as they lie
    const uint64_t chunk_global = (uint64_t)(d.units_off / 2) + it.first;          // two fields: units_off counts two entries per chunk
    uint4 *const out = reinterpret_cast<uint4 *>(lane_counts + chunk_global * (2 * 256 * 32));
    for (uint32_t i = tid; i < 2 * 256 * 32 / 4; i += 512) out[i] = cnt4[i];
    // thread (field, symbol) sums the symbol's 64 lanes, starting at a different word per thread (different banks)
    const uint32_t f = tid >> 8, bin = tid & 255;
    uint32_t sum = 0;
#pragma unroll 8
    for (uint32_t r = 0; r < 32; r++) {
        const uint32_t c = cnt[(f * 256 + bin) * 32 + ((r + bin) & 31)];
        sum += (c & 0xFFFFu) + (c >> 16);
    }
    // BF16 and byte symbols: field f's histogram is the tensor's slot f.  E5M2: slot 0 is the histogram of the bytes that
    // k_hist counts, and the field histograms of what this kernel counts go to slot 1, exponents at 0..31 and sign+mantissa
    // symbols at 32..39 (k_codes adds them up)
    const uint64_t at = FMT == ZC_FMT_FP8_E5M2 ? 256 + (f ? 32 : 0) + bin : f * 256 + bin;
    if (sum && (FMT != ZC_FMT_FP8_E5M2 || bin < (f ? 8u : 32u)))
        atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(uint64_t)it.tensor * 768 + at]), (unsigned long long)sum);
}

// Stream sizes of whole chunks from those counts, for the tensors the 64-lane encoder of these formats takes (route 2:
// exponent field table coded, sign+mantissa field flat, raw or table coded) and for every E5M2 tensor (whichever
// encoder writes it).  A table-coded field: as in
// k_sizes_fp8_counts, with R symbols per refill step (R codes are at most 32 bits, which is all the argument there
// needs): a lane's words are min(steps, floor((bits - bits of its last R codes) / 32) + 2), its bits the counts times
// the code lengths.  A flat or raw field takes its plain size.  One wavefront per chunk, work items as for the
// generic whole-chunk size pass.  A wavefront reads a field's counts 16 bytes per lane (eight symbols' rows of 32
// words per load), so a lane gathers parts of eight chunk lanes' bit totals; LDS additions bring them together.
template <int FMT>
__global__ __launch_bounds__(256) void k_sizes_rows8_counts(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables,
                                                            const uint32_t *lane_counts, uint32_t *units)
{
    __shared__ uint32_t lens[2][256];
    __shared__ uint32_t total[kWavesPerGroup][2][64];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (dp->route != 2 && (FMT != ZC_FMT_FP8_E5M2 || dp->route != 0)) return;      // whole workgroup: the generic size pass takes this tensor
    constexpr uint32_t G = Fmt<FMT>::G;                           // symbols per run and field
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    lens[0][tid] = enc_tables[(uint64_t)it.tensor * 768 + tid] >> 16;
    lens[1][tid] = enc_tables[(uint64_t)it.tensor * 768 + 256 + tid] >> 16;
    total[wave][0][lane] = 0;
    total[wave][1][lane] = 0;
    __syncthreads();
    const uint32_t chunk = uni32(it.first + wave);
    const uint32_t cb = uni32(dp->chunk_bytes);
    const uint64_t nbytes = uni64(dp->n_elems) * (uint64_t)Fmt<FMT>::EB / 8;
    const bool mine = cb == kHistBlockBytes && chunk < (uint32_t)(nbytes / cb);
    const uint64_t chunk_global = (uint64_t)(uni32(dp->units_off) / 2) + (mine ? chunk : 0u);
    const uint32_t kind[2] = {uni32(dp->kind[0]), uni32(dp->kind[1])};       // 0 table coded, 1 flat code, 2 raw, 3 constant
    const bool coded[2] = {kind[0] == 0, kind[1] == 0};
    if (mine) {
#pragma unroll
        for (int f = 0; f < 2; f++) {
            if (!coded[f]) continue;
            const uint4 *rows = reinterpret_cast<const uint4 *>(lane_counts + chunk_global * (2 * 256 * 32) + f * (256 * 32)) + lane;
            uint32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
            for (uint32_t i = 0; i < 32; i++) {
                const uint4 c = rows[i * 64];                    // symbol 8 * i + lane / 8, chunk lanes 4 * (lane % 8) .. + 3 and those + 32
                const uint32_t len = lens[f][8 * i + (lane >> 3)];
                const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                for (int k = 0; k < 4; k++) { acc[k] += (w[k] & 0xFFFFu) * len; acc[4 + k] += (w[k] >> 16) * len; }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) {
                atomicAdd(&total[wave][f][4 * (lane & 7) + k], acc[k]);
                atomicAdd(&total[wave][f][32 + 4 * (lane & 7) + k], acc[4 + k]);
            }
        }
    }
    __syncthreads();
    if (!mine) return;
    // the lane's last run: its last R symbols of either field
    const uint64_t at = (uint64_t)chunk * cb + (cb - 1024) + lane * 16;
    uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + at);
    if (uni64((uint64_t)dp->base) != 0) v = xor4(v, *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + at));
    uint64_t P[2], Q[2];
    split_run4<FMT>(v, P[0], Q[0], P[1], Q[1]);
    uint32_t u[2];
#pragma unroll
    for (int f = 0; f < 2; f++) {
        if (!coded[f]) {
            u[f] = kind[f] == 3 ? 0u : cb / 256 * G;              // 8 bits per symbol, G symbols per 16 bytes of the chunk; a constant field: nothing
            continue;
        }
        const uint32_t R = uni32(dp->period[f]);                 // 2, 4, 8 or, with runs of 16 symbols, 16
        uint32_t last = 0;
        for (uint32_t j = G - R; j < G; j++) last += lens[f][(uint32_t)((G == 16 && j >= 8 ? Q[f] : P[f]) >> (8 * (j & 7))) & 0xFFu];
        const uint32_t steps = cb / 1024 * G / R;
        uint32_t q = ((total[wave][f][lane] - last) >> 5) + 2;
        q = q < steps ? q : steps;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
        u[f] = (q + 3) / 4;
    }
    if (lane == 0) {
        uint32_t *my = units + uni32(dp->units_off);
        const uint32_t nc = uni32(dp->n_chunks);
        my[chunk] = u[0];
        my[nc + chunk] = u[1];
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
    auto fetch = [&](uint32_t row, u32x4 &x, u32x4 &y) {
        row = row < rows ? row : rows - 1;
        x = __builtin_amdgcn_raw_buffer_load_b128(src, (int)(lane * 16), (int)(row * 1024), 0);
        if (has_base) y = __builtin_amdgcn_raw_buffer_load_b128(bas, (int)(lane * 16), (int)(row * 1024), 0);
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
    const bool mine = dp->route == (BF ? 2 : 1) && (!BF || dp->period[0] == BF) && comp && count > 0 &&
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
    const uint32_t did_not_fit = encode_pages<S, HOLD ? kPagesHold : kPagesSize, BF>(dp, first, slots, pair, stage, pairs_of_rows, nullptr, nullptr, sizes,
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
    encode_pages<S, kPagesWrite, BF>(dp, first, slots, pair, stage, pairs_of_rows, idx0, idx1, nullptr, 0, first);
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
    default: ZC_CHAINED(8); break;
    }
#undef ZC_CHAINED
}

// streams: 4, 8, 16 or 32.  bf16_period: 0 for FP8 tensors (route 1), else the one refill period of the exponent field that
// every BF16 tensor of the call has (route 2).  Work items in natural order (tensor by tensor, pages ascending), each
// slots_per_item pages (a multiple of the pages a workgroup takes per pass, at most compress_pages_chained_limit()).
// hold: 0, or the words of LDS per page (a multiple of 4) of the build that keeps the exponent streams there and reads
// the source once; slots_per_item * hold is then at most compress_pages_held_words().  d_status: n_work words,
// d_counter: one word; both are reset here.
int launch_compress_pages_chained(uint32_t streams, uint32_t bf16_period, uint32_t hold, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                                  uint32_t slots_per_item, const uint32_t *d_enc, const uint8_t *d_blobs, uint32_t blob_bytes, uint64_t *d_status,
                                  uint64_t *d_counter, ScanOut *d_out, void *stream)
{
    if (n_work == 0) return 0;
    if (slots_per_item == 0 || slots_per_item > kChainItemPages || (bf16_period != 0 && bf16_period != 2 && bf16_period != 4 && bf16_period != 8)) return 1;
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

int launch_sizes_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_sizes_fp8, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_units);
    return (int)hipGetLastError();
}

int launch_hist_fp8_lanes(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint16_t *d_lane_counts, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_hist_fp8_lanes, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    return (int)hipGetLastError();
}

int launch_sizes_fp8_counts(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, const uint16_t *d_lane_counts,
                            uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_sizes_fp8_counts, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    return (int)hipGetLastError();
}

// fmt: ZC_FMT_BF16, ZC_FMT_FP8_E4M3_BYTES or ZC_FMT_FP8_E5M2.  One work item per whole chunk of kHistBlockBytes.
int launch_hist_rows8_lanes(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint32_t *d_lane_counts, void *stream)
{
    if (n_work == 0) return 0;
    if (fmt == ZC_FMT_BF16) hipLaunchKernelGGL(k_hist_rows8_lanes<ZC_FMT_BF16>, dim3(n_work), dim3(512), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    else if (fmt == ZC_FMT_FP8_E4M3_BYTES)
        hipLaunchKernelGGL(k_hist_rows8_lanes<ZC_FMT_FP8_E4M3_BYTES>, dim3(n_work), dim3(512), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    else if (fmt == ZC_FMT_FP8_E5M2)
        hipLaunchKernelGGL(k_hist_rows8_lanes<ZC_FMT_FP8_E5M2>, dim3(n_work), dim3(512), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    else return 1;
    return (int)hipGetLastError();
}

// work items of kWavesPerGroup whole chunks, as for the generic whole-chunk size pass
int launch_sizes_rows8_counts(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc,
                              const uint32_t *d_lane_counts, uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    if (fmt == ZC_FMT_BF16)
        hipLaunchKernelGGL(k_sizes_rows8_counts<ZC_FMT_BF16>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    else if (fmt == ZC_FMT_FP8_E4M3_BYTES)
        hipLaunchKernelGGL(k_sizes_rows8_counts<ZC_FMT_FP8_E4M3_BYTES>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    else if (fmt == ZC_FMT_FP8_E5M2)
        hipLaunchKernelGGL(k_sizes_rows8_counts<ZC_FMT_FP8_E5M2>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    else return 1;
    return (int)hipGetLastError();
}

int launch_encode_fp8(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_encode_fp8, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc);
    return (int)hipGetLastError();
}

}  // namespace zc
