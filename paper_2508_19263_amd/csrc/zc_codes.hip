// Code construction on the device: from the histograms that k_hist left in the workspace to everything the
// size pass and the encoder read (encode tables, field modes and refill periods in the descriptors, the
// code-length tables in the header blobs), without a round trip to the host.  One workgroup per (tensor,
// field).  The result is bit for bit what the host construction in zc_codebook.cpp gives: the same optimal
// length-limited code (package-merge) with the same tie rules
//   * leaves ordered by (frequency, symbol value), ascending;
//   * in a merged row a leaf goes before a package of equal weight;
//   * canonical codes handed out in (length, symbol value) order,
// the same choice between a coded, a raw and a constant field (Sec. 3.1: a field that does not compress is
// stored as is), and the same histogram marginals per format.
//
// Package-merge in the form used here keeps, per row, only the weights (two rows at a time) and one bit
// per item that says whether it is a leaf: the code length of the i-th cheapest leaf is the number of rows
// in which it lies inside the item budget that is walked down from the top row (2n-2 items there; every
// package inside the budget stands for two items of the row below).  A row is the merge of the sorted
// leaves with the sorted packages of the row below, so every item finds its place with one binary search.
#include <hip/hip_runtime.h>

#include "zc_internal.h"

namespace zc {

namespace {

constexpr int kCodeThreads = 256;          // >= the largest alphabet: one thread per symbol, leaf and package
constexpr int kMaxRow = 512;               // a row holds at most 2n-1 items

__device__ __forceinline__ uint32_t reverse_code(uint32_t code, uint32_t len) { return len ? __brev(code) >> (32 - len) : 0u; }

// sums and maxima over the workgroup: shuffles inside a wavefront, then one LDS atomic per wavefront (all lanes
// of a workgroup hitting one LDS address with atomics take their turns one by one)
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64); return v; }
__device__ __forceinline__ uint32_t wave_max(uint32_t v) { for (int o = 32; o > 0; o >>= 1) { const uint32_t w = __shfl_xor(v, o, 64); v = w > v ? w : v; } return v; }
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v)
{
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, o, 64), hi = __shfl_xor((uint32_t)(v >> 32), o, 64);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

// symbols of field f counted in byte b of the joint histogram: up to two (FP4 holds two elements per byte)
__device__ __forceinline__ int joint_symbols(uint32_t fmt, int f, uint32_t b, uint32_t sym[2])
{
    if (fmt == ZC_FMT_FP8_E4M3) { sym[0] = f == 0 ? (b >> 3) & 0xF : ((b >> 4) & 8) | (b & 7); return 1; }
    if (fmt == ZC_FMT_FP8_E5M2) { sym[0] = f == 0 ? (b >> 2) & 0x1F : ((b >> 5) & 4) | (b & 3); return 1; }
    for (int h = 0; h < 2; h++) {
        const uint32_t nib = (b >> (4 * h)) & 0xF;
        sym[h] = f == 0 ? (nib >> 1) & 3 : ((nib >> 2) & 2) | (nib & 1);
    }
    return 2;
}

// Rows limit-1 .. 1 of the package-merge (the row `limit` is the leaves themselves, lw[0..n) ascending): fills
// leaf_bits and row_size.  W: the weight type; 32 bits are enough when 16 times the sum of all weights fits (an
// item of any row holds a leaf at most once per row below it), and halve the LDS traffic of the searches.
// Called by the whole workgroup.
template <typename W>
__device__ void build_rows(const W *lw, W *pw, W *row0, W *row1, uint32_t n, int limit, uint32_t (*leaf_bits)[kMaxRow / 32], uint32_t *row_size)
{
    const uint32_t tid = threadIdx.x;
    if (tid == 0) row_size[limit] = n;
    uint32_t m = n;                                       // items of the row below
    const W *below = lw;
    W *out = row0, *other = row1;
    for (int d = limit - 1; d >= 1; d--) {
        const uint32_t n_pk = m / 2;
        if (tid < n_pk) pw[tid] = below[2 * tid] + below[2 * tid + 1];
        __syncthreads();
        // Both searches of a thread advance together, a fixed nine halving steps each (rows hold fewer than
        // 512 items): the packages strictly cheaper than leaf `tid` go before it, the leaves that cost no
        // more than package `tid` go before that.
        const W wl = tid < n ? lw[tid] : (W)0, wp = tid < n_pk ? pw[tid] : (W)0;
        uint32_t below_leaf = 0, below_pack = 0;
#pragma unroll
        for (uint32_t step = 256; step > 0; step >>= 1) {
            const uint32_t a = below_leaf + step, b = below_pack + step;
            const W pa = pw[(a <= n_pk ? a : 1u) - 1], lb = lw[(b <= n ? b : 1u) - 1];
            if (a <= n_pk && pa < wl) below_leaf = a;
            if (b <= n && lb <= wp) below_pack = b;
        }
        if (tid < n) {
            const uint32_t pos = tid + below_leaf;
            out[pos] = wl;
            atomicOr(&leaf_bits[d][pos / 32], 1u << (pos % 32));
        }
        if (tid < n_pk) out[tid + below_pack] = wp;
        m = n + n_pk;
        if (tid == 0) row_size[d] = m;
        __syncthreads();
        below = out;
        W *const swap = out; out = other; other = swap;
    }
}

}  // namespace

__global__ __launch_bounds__(kCodeThreads) void k_codes(TensorDev *descs, const uint64_t *hist, CodeParams cp, uint8_t *blobs, uint32_t *enc_tables)
{
    __shared__ unsigned long long h[256];              // the field's histogram by symbol
    __shared__ unsigned long long lw[256];             // leaf weights, cheapest first
    __shared__ unsigned long long row[2][kMaxRow];     // the row below and the row being merged
    __shared__ unsigned long long pw[256];             // package weights of the row below
    __shared__ uint32_t leaf_bits[17][kMaxRow / 32];   // per row: which items are leaves
    __shared__ uint32_t row_size[17], leaves_in[17];
    __shared__ uint32_t count[17], next[17];
    __shared__ uint8_t order[256], len[256];
    __shared__ unsigned long long pay_s, sum_s;
    __shared__ uint32_t n_s, konst_s, flat_s, lmax_s;

    const uint32_t t = blockIdx.x, f = blockIdx.y, tid = threadIdx.x;
    const uint32_t fmt = cp.fmt;
    const uint32_t grouped = (fmt == ZC_FMT_FP8_E4M3_BYTES || fmt == ZC_FMT_FP4_E2M1_MX_BYTES) ? 1u : 0u;
    const uint32_t sb = (f == 2 || grouped || fmt == ZC_FMT_FP8_E5M2 || fmt == ZC_FMT_BF16) ? 8u : fmt == ZC_FMT_FP8_E4M3 ? 4u : 2u;
    const uint32_t A = 1u << sb;
    const int limit = cp.limit[f];
    const uint64_t *hist3 = hist + (uint64_t)t * 768;

    // ---- the field's histogram
    h[tid] = 0; len[tid] = 0;
    if (tid < 17) { row_size[tid] = 0; leaves_in[tid] = 0; count[tid] = 0; next[tid] = 0; }
    for (uint32_t i = tid; i < 17 * (kMaxRow / 32); i += kCodeThreads) (&leaf_bits[0][0])[i] = 0;
    if (tid == 0) { pay_s = 0; sum_s = 0; n_s = 0; konst_s = 0; flat_s = 0; lmax_s = 0; }
    __syncthreads();
    if (f == 2) h[tid] = hist3[512 + tid];
    else if (fmt == ZC_FMT_BF16 || grouped) h[tid] = hist3[256 * f + tid];
    else {
        uint32_t sym[2];
        const int k = joint_symbols(fmt, (int)f, tid, sym);
        const unsigned long long c = hist3[tid];
        for (int i = 0; i < k; i++) atomicAdd(&h[sym[i]], c);
    }
    __syncthreads();
    // FP8: chunks counted by k_hist_fp8_lanes left their field histograms in the second slot (exponents at 0..15,
    // sign+mantissa at 16..31); the byte histogram above then covers only what that kernel did not take
    if (fmt == ZC_FMT_FP8_E4M3 && f < 2 && tid < 16) h[tid] += hist3[256 + 16 * f + tid];
    // FP8 E5M2: likewise for k_hist_fp8_lanes<true> (exponents at 0..31, sign+mantissa symbols at 32..39)
    if (fmt == ZC_FMT_FP8_E5M2 && f < 2 && tid < (f ? 8u : 32u)) h[tid] += hist3[256 + (f ? 32 : 0) + tid];
    __syncthreads();

    // ---- leaves in (frequency, symbol) order
    const unsigned long long hv = tid < A ? h[tid] : 0ull;
    const bool present = hv != 0;
    {
        const uint32_t wn = wave_sum(present ? 1u : 0u), wk = wave_max(present ? tid : 0u);
        const unsigned long long ws = wave_sum(hv);
        if ((tid & 63) == 0) { atomicAdd(&n_s, wn); atomicMax(&konst_s, wk); atomicAdd(&sum_s, ws); }
    }
    __syncthreads();
    const uint32_t n = n_s;
    const bool narrow = 16ull * sum_s < (1ull << 32);         // every weight of every row fits 32 bits
    uint32_t rank = 0;
    if (narrow) {
        // absent symbols get the largest key, so they rank behind every present one and need no test of their own
        uint32_t *h32 = reinterpret_cast<uint32_t *>(pw);
        h32[tid] = present ? (uint32_t)hv : 0xFFFFFFFFu;
        __syncthreads();
        const uint32_t mine = h32[tid];
#pragma unroll 8
        for (uint32_t u = 0; u < A; u++) {
            const uint32_t hu = h32[u];
            rank += (hu < mine || (hu == mine && u < tid)) ? 1u : 0u;
        }
    } else {
#pragma unroll 8
        for (uint32_t u = 0; u < A; u++) {
            const unsigned long long hu = h[u];
            rank += (hu != 0 && (hu < hv || (hu == hv && u < tid))) ? 1u : 0u;
        }
    }
    if (present) { lw[rank] = hv; order[rank] = (uint8_t)tid; }
    __syncthreads();

    uint32_t mode = ZC_MODE_EMPTY, konst = 0, lmax = 0;
    if (n == 1) { mode = ZC_MODE_CONST; konst = konst_s; }
    else if (n > 1) {
        mode = ZC_MODE_HUFF;
        // ---- rows limit-1 .. 1
        if (narrow) {
            uint32_t *lw32 = reinterpret_cast<uint32_t *>(h);      // the histogram by symbol is not needed any more
            const uint32_t mine = tid < n ? (uint32_t)lw[tid] : 0u;
            __syncthreads();
            if (tid < n) lw32[tid] = mine;
            __syncthreads();
            build_rows<uint32_t>(lw32, reinterpret_cast<uint32_t *>(pw), reinterpret_cast<uint32_t *>(row[0]), reinterpret_cast<uint32_t *>(row[1]),
                                 n, limit, leaf_bits, row_size);
        } else build_rows<unsigned long long>(lw, pw, row[0], row[1], n, limit, leaf_bits, row_size);
        // ---- walk the budget down from the top row (one wavefront: 16 mask words per row)
        if (tid < 64) {
            uint32_t budget = 2 * n - 2;
            for (int d = 1; d <= limit && budget > 0; d++) {
                const uint32_t b = budget < row_size[d] ? budget : row_size[d];
                uint32_t leaves;
                if (d == limit) leaves = b;
                else {
                    uint32_t c = 0;
                    if (tid < kMaxRow / 32) {
                        const uint32_t lo = tid * 32;
                        const uint32_t take = b > lo ? (b - lo >= 32 ? 0xFFFFFFFFu : (1u << (b - lo)) - 1) : 0u;
                        c = (uint32_t)__popc(leaf_bits[d][tid] & take);
                    }
                    for (int o = 8; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
                    leaves = __shfl(c, 0, 64);
                }
                if (tid == 0) leaves_in[d] = leaves;
                budget = 2 * (b - leaves);
            }
        }
        __syncthreads();
        {
            uint32_t l = 0;
            if (tid < n) {
                for (int d = 1; d <= limit; d++) l += leaves_in[d] > tid ? 1u : 0u;
                len[order[tid]] = (uint8_t)l;
            }
            const unsigned long long wp = wave_sum(tid < n ? lw[tid] * l : 0ull);
            const uint32_t wl = wave_max(l);
            if ((tid & 63) == 0) { atomicAdd(&pay_s, wp); atomicMax(&lmax_s, wl); }
        }
        __syncthreads();
        lmax = lmax_s;
        // Sec. 3.1: a field that does not compress is stored as is
        if (cp.policy == ZC_POLICY_AUTO && 16ull * pay_s > 15ull * sum_s * sb) { mode = ZC_MODE_RAW; lmax = 0; }
    }
    __syncthreads();
    if (mode != ZC_MODE_HUFF) len[tid] = 0;
    __syncthreads();

    // ---- canonical codes in (length, symbol) order
    const uint32_t my_len = tid < A ? len[tid] : 0u;
    for (uint32_t l = 1; l <= 16; l++) {
        const uint32_t c = (uint32_t)__popcll(__ballot(my_len == l));
        if ((tid & 63) == 0 && c) atomicAdd(&count[l], c);
    }
    {
        const uint32_t c = (uint32_t)__popcll(__ballot(tid < A && my_len == sb));
        if ((tid & 63) == 0 && c) atomicAdd(&flat_s, c);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t code = 0;
        for (int l = 1; l <= 16; l++) { code = (code + (l > 1 ? count[l - 1] : 0u)) << 1; next[l] = code; }
    }
    __syncthreads();
    uint32_t code = 0;
    if (my_len) {
        uint32_t before = 0;
#pragma unroll 8
        for (uint32_t u = 0; u < tid; u++) before += len[u] == my_len ? 1u : 0u;
        code = next[my_len] + before;
    }

    // ---- what the other kernels read
    enc_tables[(uint64_t)t * 768 + f * 256 + tid] = tid < A ? (my_len << 16) | reverse_code(code, my_len) : 0u;
    uint8_t *blob = blobs + (uint64_t)t * cp.blob_bytes;
    TensorDev &d = descs[t];
    if (tid < A) blob[d.table_off[f] + tid] = (uint8_t)my_len;
    if (tid == 0) {
        const uint32_t kind = mode == ZC_MODE_RAW ? 2u : mode != ZC_MODE_HUFF ? 3u : flat_s == A ? 1u : 0u;
        // symbols between two refill steps of the field's stream: the largest power of two r with r * lmax <= 32,
        // at most a run
        const uint32_t G = f == 2 ? 16u : cp.run_len;
        uint32_t r = 1;
        const uint32_t lm = lmax < 1 ? 1u : lmax;
        while (2 * r * lm <= 32) r *= 2;
        if (r > G) r = G;
        blob[32 + 4 * f] = (uint8_t)mode; blob[33 + 4 * f] = (uint8_t)sb; blob[34 + 4 * f] = (uint8_t)lmax; blob[35 + 4 * f] = (uint8_t)konst;
        d.mode[f] = (uint8_t)mode; d.lmax[f] = (uint8_t)lmax; d.konst[f] = (uint8_t)konst; d.period[f] = (uint8_t)r; d.kind[f] = (uint8_t)kind;
    }
}

// After k_codes: which kernels take the tensor's whole chunks, and the exponent-pair table of the FP8
// kernels (two codes concatenated, for a pair of exponents: the table slot of the third field, which FP8
// does not have).  The FP8 kernels are written for a refill period of 4 on the exponents (longest code 5..8
// bits) and a sign+mantissa field that is flat coded or raw.
__global__ __launch_bounds__(256) void k_codes_finish(TensorDev *descs, CodeParams cp, uint32_t *enc_tables)
{
    TensorDev &d = descs[blockIdx.x];
    const bool fast = cp.fmt == ZC_FMT_FP8_E4M3 && d.fast_shape && d.mode[0] == ZC_MODE_HUFF && d.period[0] == 4 && (d.kind[1] == 1 || d.kind[1] == 2);
    uint32_t *enc = enc_tables + (uint64_t)blockIdx.x * 768;
    if (fast) {
        const uint32_t u = threadIdx.x, e0 = enc[u & 15], e1 = enc[u >> 4];
        const uint32_t l0 = e0 >> 16, l1 = e1 >> 16;
        enc[512 + u] = ((l0 + l1) << 16) | (e0 & 0xFFFFu) | ((e1 & 0xFFFFu) << l0);
    }
    // BF16, and FP8 in byte symbols: the 64-lane encoder takes a table-coded exponent field next to a sign+mantissa field
    // that is flat, raw, or table coded with a refill period of 2 or 4; the BF16 page kernels (fewer lanes) want the latter flat or raw and, with
    // two exponents per refill step, no 1-bit code (the bound on their staging ring needs 4 bits per step)
    __shared__ uint32_t lmin_s;
    if (threadIdx.x == 0) lmin_s = 16;
    __syncthreads();
    const uint32_t my_len = enc[threadIdx.x] >> 16;
    if (my_len) atomicMin(&lmin_s, my_len);
    __syncthreads();
    const bool plain_sm = d.kind[1] == 1 || d.kind[1] == 2;
    // (FP8 E5M2, 16 symbols per run: both fields table coded, refill periods of at most 8)
    const bool e5m2 = cp.fmt == ZC_FMT_FP8_E5M2 && d.streams == 64 && d.kind[1] == 0 && d.period[0] <= 8 && d.period[1] >= 2 && d.period[1] <= 8;
    const bool bf16 = d.fast_shape && d.kind[0] == 0 &&
                      (d.streams == 64 ? (e5m2 || ((cp.fmt == ZC_FMT_BF16 || cp.fmt == ZC_FMT_FP8_E4M3_BYTES) &&
                                                   (plain_sm || (d.kind[1] == 0 && (d.period[1] == 2 || d.period[1] == 4)))))
                                       : (cp.fmt == ZC_FMT_BF16 && plain_sm && (d.period[0] != 2 || lmin_s >= 2)));
    if (threadIdx.x == 0) d.route = fast ? 1 : bf16 ? 2 : 0;
}

int launch_codes(TensorDev *d_descs, uint32_t n_tensors, const uint64_t *d_hist, const CodeParams &cp, uint8_t *d_blobs, uint32_t *d_enc, void *stream)
{
    if (n_tensors == 0) return 0;
    hipLaunchKernelGGL(k_codes, dim3(n_tensors, cp.nf), dim3(kCodeThreads), 0, (hipStream_t)stream, d_descs, d_hist, cp, d_blobs, d_enc);
    hipLaunchKernelGGL(k_codes_finish, dim3(n_tensors), dim3(256), 0, (hipStream_t)stream, d_descs, cp, d_enc);
    return (int)hipGetLastError();
}

}  // namespace zc
