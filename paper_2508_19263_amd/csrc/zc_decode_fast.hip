// Specialised decode kernels for the common shapes of a container: FP8 E4M3, 64 lanes per
// chunk, full chunks, exponent field Huffman coded with codes of at most 8 bits, and a
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

#include "zc_internal.h"

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

// EK: 0 = one symbol per lookup (codes <= 8 bits, 256 entries), 1 = two symbols per lookup
//     (codes <= 6 bits, 4096 entries).  MK: 0 = flat 4-bit code, 1 = raw.  XOR: delta container.
template <int EK, int MK, bool XOR>
__global__ __launch_bounds__(256) void k_decode_fp8(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single)
{
    constexpr uint32_t kEntries = EK ? 4096u : 256u;
    __shared__ uint32_t lut[kEntries];
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
        lut[idx] = entry;
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63;
    const uint32_t chunk = __builtin_amdgcn_readfirstlane(it.first + (threadIdx.x >> 6));
    const uint32_t E = d.chunk_bytes;                       // one element per byte
    const uint32_t n_full = (uint32_t)(d.n_elems / E);
    if (chunk >= n_full) return;                            // partial or absent chunk: not ours
    const uint32_t *index0 = reinterpret_cast<const uint32_t *>(d.comp + d.index_off[0]);
    const uint32_t *index1 = reinterpret_cast<const uint32_t *>(d.comp + d.index_off[1]);
    const uint64_t a0 = index0[chunk], b0 = index0[chunk + 1], a1 = index1[chunk], b1 = index1[chunk + 1];
    const uint32_t rows = E / (16 * 64);
    // a stream that does not lie inside the container, or a sign+mantissa stream shorter than
    // its fixed size, means a damaged index: leave the chunk alone rather than read outside
    if (a0 > b0 || a1 > b1 || d.payload_off + 16 * b1 > d.total_bytes || d.payload_off + 16 * b0 > d.total_bytes) return;
    if ((b1 - a1) * 16 < (uint64_t)E / 2) return;
    const uint32_t *es = reinterpret_cast<const uint32_t *>(d.comp + d.payload_off + 16 * a0);
    const uint32_t *ms = reinterpret_cast<const uint32_t *>(d.comp + d.payload_off + 16 * a1);
    const uint32_t e_words = (uint32_t)(b0 - a0) * 4;
    uint4 *dst = reinterpret_cast<uint4 *>(d.dst + (uint64_t)chunk * E);
    const uint4 *base = XOR ? reinterpret_cast<const uint4 *>(d.base + (uint64_t)chunk * E) : nullptr;

    uint32_t lo = 0, hi = 0, c = 64, wpos = 0;
    constexpr uint32_t kMask = kEntries - 1;
    for (uint32_t row = 0; row < rows; row++) {
        // ---- sign+mantissa: 16 nibbles -> bytes 0000smmm, four per word
        uint32_t m[4];
        if (MK == 0) {
            // flat code: one word per 8 symbols, rows of 64 words; code bits are MSB first in an
            // LSB-first string, so a bit reversal gives natural nibbles in reverse symbol order
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t w = __brev(ms[(row * 2 + h) * 64 + lane]);
                const uint32_t A = w & 0x0F0F0F0Fu;            // symbols 7,5,3,1 in bytes 0..3
                const uint32_t B = (w >> 4) & 0x0F0F0F0Fu;     // symbols 6,4,2,0
                m[2 * h] = perm(A, B, 0x06020703u);            // bytes: B3 A3 B2 A2 -> symbols 0,1,2,3
                m[2 * h + 1] = perm(A, B, 0x04000501u);        // bytes: B1 A1 B0 A0 -> symbols 4,5,6,7
            }
        } else {
            const uint2 w2 = reinterpret_cast<const uint2 *>(ms)[row * 64 + lane];
            const uint32_t w[2] = {w2.x, w2.y};
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t A = w[h] & 0x0F0F0F0Fu;         // symbols 0,2,4,6
                const uint32_t B = (w[h] >> 4) & 0x0F0F0F0Fu;  // symbols 1,3,5,7
                m[2 * h] = perm(A, B, 0x01050004u);            // bytes: A0 B0 A1 B1
                m[2 * h + 1] = perm(A, B, 0x03070206u);        // bytes: A2 B2 A3 B3
            }
        }
        // ---- exponent: 4 groups of 4 symbols
        uint32_t ex[4];
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const bool need = c >= 32;
            const uint64_t bm = __ballot(need);
            if (need) {
                const uint32_t pos = wpos + prefix_count64(bm);
                const uint32_t w = pos < e_words ? es[pos] : 0u;
                lo = hi; hi = w; c -= 32;
            }
            wpos += (uint32_t)__popcll(bm);
            uint32_t x = (uint32_t)((((uint64_t)hi << 32) | lo) >> c);
            if (EK == 0) {
                const uint32_t t0 = lut[x & kMask]; x >>= (t0 & 31u);
                const uint32_t t1 = lut[x & kMask]; x >>= (t1 & 31u);
                const uint32_t t2 = lut[x & kMask]; x >>= (t2 & 31u);
                const uint32_t t3 = lut[x & kMask];
                c += (t0 + t1 + t2 + t3) & 0xFFu;
                // byte 1 of each entry -> bytes 0..3 of the output word
                const uint32_t p01 = perm(t1, t0, 0x0C0C0501u);   // [t0.b1, t1.b1, 0, 0]
                const uint32_t p23 = perm(t3, t2, 0x05010C0Cu);   // [0, 0, t2.b1, t3.b1]
                ex[g] = p01 | p23;
            } else {
                const uint32_t t0 = lut[x & kMask]; x >>= (t0 & 31u);
                const uint32_t t1 = lut[x & kMask];
                c += (t0 + t1) & 0xFFu;
                ex[g] = perm(t1, t0, 0x06050201u);                // [t0.b1, t0.b2, t1.b1, t1.b2]
            }
        }
        // ---- merge: byte = s eeee mmm
        uint4 v;
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; q++) o[q] = ex[q] | (m[q] & 0x07070707u) | ((m[q] & 0x08080808u) << 4);
        v = make_uint4(o[0], o[1], o[2], o[3]);
        if (XOR) { const uint4 b = base[row * 64 + lane]; v.x ^= b.x; v.y ^= b.y; v.z ^= b.z; v.w ^= b.w; }
        dst[row * 64 + lane] = v;
    }
}

template <int EK, int MK>
static int launch_fp8_x(bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const TensorDev &s, int use_single, hipStream_t st)
{
    if (xor_delta) hipLaunchKernelGGL((k_decode_fp8<EK, MK, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    else hipLaunchKernelGGL((k_decode_fp8<EK, MK, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single);
    return (int)hipGetLastError();
}

// exp_kind: 0 = single lookups, 1 = pair lookups; sm_kind: 0 = flat code, 1 = raw
int launch_decode_fp8_fast(int exp_kind, int sm_kind, bool xor_delta, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work,
                           const TensorDev *single, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    if (exp_kind == 0 && sm_kind == 0) return launch_fp8_x<0, 0>(xor_delta, d_descs, d_work, n_work, s, use_single, st);
    if (exp_kind == 0 && sm_kind == 1) return launch_fp8_x<0, 1>(xor_delta, d_descs, d_work, n_work, s, use_single, st);
    if (exp_kind == 1 && sm_kind == 0) return launch_fp8_x<1, 0>(xor_delta, d_descs, d_work, n_work, s, use_single, st);
    return launch_fp8_x<1, 1>(xor_delta, d_descs, d_work, n_work, s, use_single, st);
}

}  // namespace zc
