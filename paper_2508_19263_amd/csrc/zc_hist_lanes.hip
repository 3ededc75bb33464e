// Histogram passes that also count symbols per chunk lane, and the size passes that work from those counts instead
// of reading the source a second time (a3 and a5 for 64 lanes and chunks of one histogram block); and the size pass
// of a tensor's short last chunk, which rests on the same closed form (k_sizes_tail).
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_encode_device.h"

namespace zc {

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
// E5M2 (s eeeee mm) is counted the same way and folded differently: 32 exponent counts and 8 sign+mantissa counts per
// lane (80 bytes, 5 KiB per chunk), field histograms at 0..31 and 32..39 of the second slot.
template <bool E5M2>
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
    if (E5M2) {
        // Thread (lane, quarter) folds the byte values 64*quarter .. +63 of its lane: value = s eeeee mm, so a quarter is one
        // sign, the exponents 16 * (quarter & 1) .. + 15 and all four mantissas.
        uint32_t c[32];
#pragma unroll
        for (int i = 0; i < 32; i++) c[i] = 0;
        const uint32_t half_shift = lane < 32 ? 0u : 16u;
#pragma unroll
        for (int v = 0; v < 64; v++) {
            const uint32_t n = (cnt[(quarter * 64 + v) * 32 + (lane & 31)] >> half_shift) & 0xFFFFu;
            c[v >> 2] += n;                                      // exponent 16 * (quarter & 1) + v / 4
            c[16 + (v & 3)] += n;                                // sign+mantissa symbol 4 * (quarter >> 1) + v % 4
        }
        const uint32_t e_hi = quarter & 1, sgn = quarter >> 1;
        __syncthreads();                                         // every thread has read its part of cnt: the array is free
        uint32_t *const part = cnt;                              // rows of 21 words against bank conflicts
#pragma unroll
        for (int i = 0; i < 20; i++) part[(quarter * 64 + lane) * 21 + i] = c[i];
        // the chunk's field histograms: the wavefront's 20 counts summed over its lanes in a butterfly that halves what a
        // lane carries at every step; lane j < 32 ends with the total of count bitrev5(j)
#pragma unroll
        for (int step = 0; step < 5; step++) {
            const int n = 16 >> step;
            const uint32_t upper = 0u - ((lane >> step) & 1u);   // all ones in the lanes that keep the upper half
#pragma unroll
            for (int i = 0; i < n; i++) {
                // (bitwise, so that the counts stay in registers: a choice between two array elements becomes an
                // element at a computed index, which the compiler looks up with a chain of compares)
                const uint32_t a = c[i], b = c[n + i], d = (a ^ b) & upper;
                c[i] = (a ^ d) + (uint32_t)__shfl_xor((int)(b ^ d), 1 << step, 64);      // keeps b, gives a where upper
            }
        }
        c[0] += (uint32_t)__shfl_xor((int)c[0], 32, 64);
        const uint32_t k = ((lane & 1) << 4) | ((lane & 2) << 2) | (lane & 4) | ((lane & 8) >> 2) | ((lane & 16) >> 4);
        if (lane < 32 && k < 20 && c[0]) {
            unsigned long long *slot = reinterpret_cast<unsigned long long *>(&hist[((uint64_t)it.tensor * 3 + 1) * 256]);
            atomicAdd(slot + (k < 16 ? e_hi * 16 + k : 32 + sgn * 4 + (k - 16)), (unsigned long long)c[0]);
        }
        __syncthreads();
        // the lane's 40 counts: quarters 0 and 1 write the exponents 0..15 and 16..31 (both signs added), quarter 2 the eight
        // sign+mantissa symbols (both exponent halves added)
        const uint64_t chunk_global = (uint64_t)(d.units_off / 2) + it.first;
        uint16_t *mine = lane_counts + (chunk_global * 64 + lane) * 40;
        if (quarter < 2) {
            const uint32_t *pa = part + ((0 * 2 + quarter) * 64 + lane) * 21, *pb = part + ((1 * 2 + quarter) * 64 + lane) * 21;
            uint32_t w[8];
#pragma unroll
            for (int j = 0; j < 8; j++) w[j] = (pa[2 * j] + pb[2 * j]) | ((pa[2 * j + 1] + pb[2 * j + 1]) << 16);
            uint4 *out = reinterpret_cast<uint4 *>(mine + quarter * 16);
            out[0] = make_uint4(w[0], w[1], w[2], w[3]);
            out[1] = make_uint4(w[4], w[5], w[6], w[7]);
        } else if (quarter == 2) {
            uint32_t m[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint32_t sg = j >> 2;
                m[j] = part[((sg * 2 + 0) * 64 + lane) * 21 + 16 + (j & 3)] + part[((sg * 2 + 1) * 64 + lane) * 21 + 16 + (j & 3)];
            }
            *reinterpret_cast<uint4 *>(mine + 32) = make_uint4(m[0] | (m[1] << 16), m[2] | (m[3] << 16), m[4] | (m[5] << 16), m[6] | (m[7] << 16));
        }
        return;
    }
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
            const uint32_t upper = 0u - ((lane >> step) & 1u);   // all ones in the lanes that keep the upper half
#pragma unroll
            for (int i = 0; i < n; i++) {
                // (bitwise, so that the counts stay in registers: a choice between two array elements becomes an
                // element at a computed index, which the compiler looks up with a chain of compares)
                const uint32_t a = c[i], b = c[n + i], d = (a ^ b) & upper;
                c[i] = (a ^ d) + (uint32_t)__shfl_xor((int)(b ^ d), 1 << step, 64);      // keeps b, gives a where upper
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
// FP8 in byte symbols), with 64 lanes and chunks of kHistBlockBytes: weights, checkpoints and
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
    static_assert(Fmt<FMT>::G == 8 && Fmt<FMT>::SB == 8 && Fmt<FMT>::NF == 2, "two fields of 8 symbols of 8 bits per run");
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
    // field f's histogram is the tensor's slot f
    if (sum) atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(uint64_t)it.tensor * 768 + f * 256 + bin]), (unsigned long long)sum);
}

// Stream sizes of whole chunks from those counts, for the tensors the 64-lane encoder of these formats takes (route 2:
// exponent field table coded, sign+mantissa field flat, raw or table coded).  A table-coded field: as in
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
    if (dp->route != 2) return;                                  // whole workgroup: the generic size pass takes this tensor
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
        const uint32_t R = uni32(dp->period[f]);                 // 2, 4 or 8
        uint32_t last = 0;
        for (uint32_t j = G - R; j < G; j++) last += lens[f][(uint32_t)(P[f] >> (8 * j)) & 0xFFu];
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

// Stream sizes of the chunks the whole-chunk kernels leave over: with 64 lanes and chunks of whole rows that is a
// tensor's short last chunk.  The closed form of the count-based size passes holds for lanes of different lengths
// too: a lane of n symbols takes min(steps, floor((bits before its last step) / 32) + 2) words, steps = ceil(n / R).
// So the chunk need not be walked step by step by one wavefront, which takes a few hundred microseconds whatever
// else the GPU does: the sixteen wavefronts of the workgroup add up code lengths over a sixteenth of the rows each.
// Work items as for the generic size pass (up to kWavesPerGroup chunks from `first` on, one after the other).
constexpr uint32_t kTailWaves = 16;
template <int FMT>
__global__ __launch_bounds__(64 * kTailWaves) void k_sizes_tail(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables, uint32_t *units)
{
    using F_ = Fmt<FMT>;
    static_assert(F_::NF == 2 && (F_::SB == 4 || F_::SB == 8) && F_::G * F_::SB <= 128, "two fields of 4- or 8-bit symbols, at most two 64-bit words per run");
    __shared__ uint32_t lens[2][256];
    __shared__ uint32_t part[kTailWaves][2][64];
    __shared__ uint32_t last_step[2][64];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 512) lens[tid >> 8][tid & 255] = enc_tables[(uint64_t)it.tensor * 768 + tid] >> 16;
    const uint32_t nc = uni32(dp->n_chunks);
    if (uni32(dp->streams) != 64) return;                        // whole workgroup; the host never asks for this
    const uint64_t E = (uint64_t)uni32(dp->chunk_bytes) * 8 / F_::EB;     // elements of a whole chunk
    const uint64_t n_elems = uni64(dp->n_elems);
    const uint32_t mode[2] = {uni32(dp->mode[0]), uni32(dp->mode[1])};
    const uint32_t R[2] = {uni32(dp->period[0]), uni32(dp->period[1])};
    auto symbol = [](uint64_t P, uint64_t Q, uint32_t j) { return (uint32_t)((j * F_::SB < 64 ? P >> (j * F_::SB) : Q >> (j * F_::SB - 64)) & ((1u << F_::SB) - 1)); };
    for (uint32_t chunk = it.first; chunk < it.first + kWavesPerGroup && chunk < nc; chunk++) {
        const uint64_t first = (uint64_t)chunk * E;
        const uint32_t n = (uint32_t)(n_elems - first < E ? n_elems - first : E);
        const uint32_t nbytes = (uint32_t)(((uint64_t)n * F_::EB + 7) / 8);
        const uint32_t runs = (nbytes + 15) / 16, rows = (runs + 63) / 64;
        const uint8_t *src = reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + (uint64_t)chunk * uni32(dp->chunk_bytes);
        const uint8_t *base = uni64((uint64_t)dp->base) ? reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + (uint64_t)chunk * uni32(dp->chunk_bytes) : nullptr;
        __syncthreads();                                         // the tables are there; the last chunk's sums have been read
        uint32_t bits[2] = {0, 0};
        for (uint32_t row = wave; row < rows; row += kTailWaves) {
            const uint32_t run = row * 64 + lane;
            if (run >= runs) continue;
            const uint32_t done = run * F_::EPR;
            const uint32_t nel = n - done < (uint32_t)F_::EPR ? n - done : (uint32_t)F_::EPR;
            const uint32_t nsym = (nel + F_::GRP - 1) / F_::GRP;  // a last partial group is filled with zeros
            uint4 v = load_run(src + (uint64_t)run * 16, nbytes - run * 16);
            if (base) v = xor4(v, load_run(base + (uint64_t)run * 16, nbytes - run * 16));
            uint64_t P[2], Q[2];
            split_run4<FMT>(v, P[0], Q[0], P[1], Q[1]);
            const bool lanes_last = run + 64 >= runs;            // no later row has a run of this lane
#pragma unroll
            for (int f = 0; f < 2; f++) {
                if (mode[f] != ZC_MODE_HUFF) continue;
                const uint32_t j0 = (nsym - 1) / R[f] * R[f];    // first symbol of the run's last refill step
                uint32_t all = 0, tail = 0;
                for (uint32_t j = 0; j < nsym; j++) {
                    const uint32_t l = lens[f][symbol(P[f], Q[f], j)];
                    all += l;
                    tail += j >= j0 ? l : 0u;
                }
                bits[f] += all;
                // the lane's symbols: G per run before this one, nsym here
                if (lanes_last) last_step[f][lane] = tail | ((row * (uint32_t)F_::G + nsym + R[f] - 1) / R[f]) << 8;
            }
        }
        part[wave][0][lane] = bits[0];
        part[wave][1][lane] = bits[1];
        __syncthreads();
        if (wave == 0) {
            uint32_t u[2];
#pragma unroll
            for (int f = 0; f < 2; f++) {
                uint32_t q = 0;
                if (mode[f] == ZC_MODE_HUFF && lane < runs) {
                    uint32_t B = 0;
#pragma unroll
                    for (uint32_t w = 0; w < kTailWaves; w++) B += part[w][f][lane];
                    const uint32_t ls = last_step[f][lane], steps = ls >> 8;
                    q = ((B - (ls & 0xFFu)) >> 5) + 2;
                    q = q < steps ? q : steps;
                }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
                const uint32_t nsyms = (n + F_::GRP - 1) / F_::GRP;
                u[f] = mode[f] == ZC_MODE_HUFF ? (q + 3) / 4 : mode[f] == ZC_MODE_RAW ? (uint32_t)((((uint64_t)nsyms * F_::SB + 7) / 8 + 15) / 16) : 0u;
            }
            if (lane == 0) {
                uint32_t *my = units + uni32(dp->units_off);
                my[chunk] = u[0];
                my[nc + chunk] = u[1];
            }
        }
    }
}

// fmt: a format of two fields.  The tensors must have 64 lanes per chunk.
int launch_sizes_tail(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    const dim3 grid(n_work), block(64 * kTailWaves);
    hipStream_t st = (hipStream_t)stream;
    switch (fmt) {
    case ZC_FMT_BF16: hipLaunchKernelGGL(k_sizes_tail<ZC_FMT_BF16>, grid, block, 0, st, d_descs, d_work, d_enc, d_units); break;
    case ZC_FMT_FP8_E4M3: hipLaunchKernelGGL(k_sizes_tail<ZC_FMT_FP8_E4M3>, grid, block, 0, st, d_descs, d_work, d_enc, d_units); break;
    case ZC_FMT_FP8_E4M3_BYTES: hipLaunchKernelGGL(k_sizes_tail<ZC_FMT_FP8_E4M3_BYTES>, grid, block, 0, st, d_descs, d_work, d_enc, d_units); break;
    case ZC_FMT_FP8_E5M2: hipLaunchKernelGGL(k_sizes_tail<ZC_FMT_FP8_E5M2>, grid, block, 0, st, d_descs, d_work, d_enc, d_units); break;
    default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

int launch_hist_fp8_lanes(bool e5m2, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint16_t *d_lane_counts, void *stream)
{
    if (n_work == 0) return 0;
    if (e5m2) hipLaunchKernelGGL(k_hist_fp8_lanes<true>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    else hipLaunchKernelGGL(k_hist_fp8_lanes<false>, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    return (int)hipGetLastError();
}

int launch_sizes_fp8_counts(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, const uint16_t *d_lane_counts,
                            uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_sizes_fp8_counts, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    return (int)hipGetLastError();
}

// The same for FP8 E5M2 from the 40 counts per lane that k_hist_fp8_lanes<true> leaves (32 exponents, 8 sign+mantissa
// symbols): either field, when table coded, takes min(steps, floor((bits - bits of its last R codes) / 32) + 2) words
// per lane with R symbols per refill step (2, 4, 8 or 16 of the 16 symbols of a run).  One wavefront per chunk, work
// items of kWavesPerGroup whole chunks (the list of the generic whole-chunk size pass, which leaves these tensors alone).
__global__ __launch_bounds__(256) void k_sizes_e5m2_counts(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables,
                                                           const uint16_t *lane_counts, uint32_t *units)
{
    __shared__ uint32_t len_e[32], len_m[8];
    const WorkItem it = work[blockIdx.x];
    const TensorDev *dp = descs + it.tensor;
    if (threadIdx.x < 32) len_e[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + threadIdx.x] >> 16;
    if (threadIdx.x < 8) len_m[threadIdx.x] = enc_tables[(uint64_t)it.tensor * 768 + 256 + threadIdx.x] >> 16;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = uni32(it.first + (threadIdx.x >> 6));
    const uint32_t cb = uni32(dp->chunk_bytes);
    const uint64_t n_elems = uni64(dp->n_elems);
    if (cb != kHistBlockBytes || chunk >= (uint32_t)(n_elems / cb)) return;
    const uint64_t chunk_global = (uint64_t)(uni32(dp->units_off) / 2) + chunk;
    const uint4 *mine = reinterpret_cast<const uint4 *>(lane_counts + (chunk_global * 64 + lane) * 40);
    uint32_t bits[2] = {0, 0};
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const uint4 c = mine[q];
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int j = 0; j < 4; j++) bits[0] += (w[j] & 0xFFFFu) * len_e[8 * q + 2 * j] + (w[j] >> 16) * len_e[8 * q + 2 * j + 1];
    }
    {
        const uint4 c = mine[4];
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int j = 0; j < 4; j++) bits[1] += (w[j] & 0xFFFFu) * len_m[2 * j] + (w[j] >> 16) * len_m[2 * j + 1];
    }
    // the lane's last run: its last R symbols of either field
    const uint64_t at = (uint64_t)chunk * cb + (cb - 1024) + lane * 16;
    uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->src)) + at);
    if (uni64((uint64_t)dp->base) != 0) v = xor4(v, *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(uni64((uint64_t)dp->base)) + at));
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t u[2];
#pragma unroll
    for (int f = 0; f < 2; f++) {
        const uint32_t kind = uni32(dp->kind[f]);                // 0 table coded, 1 flat code, 2 raw, 3 constant
        if (kind != 0) { u[f] = kind == 3 ? 0u : cb / 16; continue; }     // (8 bits per symbol, one symbol per byte of the chunk)
        const uint32_t R = uni32(dp->period[f]);
        uint32_t last = 0;
        for (uint32_t j = 16 - R; j < 16; j++) {
            const uint32_t b = (w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
            last += f == 0 ? len_e[(b >> 2) & 31u] : len_m[((b >> 7) << 2) | (b & 3u)];
        }
        const uint32_t steps = cb / 64 / R;                      // cb / 64 symbols per lane
        uint32_t q = ((bits[f] - last) >> 5) + 2;
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

int launch_sizes_e5m2_counts(const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, const uint16_t *d_lane_counts,
                             uint32_t *d_units, void *stream)
{
    if (n_work == 0) return 0;
    hipLaunchKernelGGL(k_sizes_e5m2_counts, dim3(n_work), dim3(256), 0, (hipStream_t)stream, d_descs, d_work, d_enc, d_lane_counts, d_units);
    return (int)hipGetLastError();
}

// fmt: ZC_FMT_BF16 or ZC_FMT_FP8_E4M3_BYTES.  One work item per whole chunk of kHistBlockBytes.
int launch_hist_rows8_lanes(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint64_t *d_hist, uint32_t *d_lane_counts, void *stream)
{
    if (n_work == 0) return 0;
    if (fmt == ZC_FMT_BF16) hipLaunchKernelGGL(k_hist_rows8_lanes<ZC_FMT_BF16>, dim3(n_work), dim3(512), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
    else if (fmt == ZC_FMT_FP8_E4M3_BYTES)
        hipLaunchKernelGGL(k_hist_rows8_lanes<ZC_FMT_FP8_E4M3_BYTES>, dim3(n_work), dim3(512), 0, (hipStream_t)stream, d_descs, d_work, d_hist, d_lane_counts);
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
    else return 1;
    return (int)hipGetLastError();
}

}  // namespace zc
