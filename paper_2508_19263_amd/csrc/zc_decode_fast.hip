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

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_decode_device.h"

namespace zc {

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
        // (whole cache lines written once: the non-temporal hint keeps them from displacing the streams' lines in the L2; 1.3 % on the weight set)
        __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(lane * 16), (int)(row * 1024), 2);
    }
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
