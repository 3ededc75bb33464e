// Decoders of chunks with fewer than 64 lanes: K/V-cache pages, whole tensors or lists of page ids (Sec. 3.3, 4.3, 5.2).
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"
#include "zc_decode_device.h"

namespace zc {

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
    // A group's store of a row is 16 * S contiguous bytes: from a whole cache line on (8 lanes) it carries the non-temporal
    // hint, so that the decoded pages do not push the partly read lines of the streams out of the L2 (page lists 4 % faster)
    constexpr int kOutPolicy = S >= 8 ? 2 : 0;
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
            if (alive) __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(out_off + (row * S + s) * 16), 0, kOutPolicy);
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
    // A group's store of a row is 16 * S contiguous bytes: from a whole cache line on (8 lanes) it carries the non-temporal
    // hint, so that the decoded pages do not push the partly read lines of the streams out of the L2 (page lists 4 % faster)
    constexpr int kOutPolicy = S >= 8 ? 2 : 0;
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
            if (alive) __builtin_amdgcn_raw_buffer_store_b128(v, ds, (int)(out_off + (row * S + s) * 16), 0, kOutPolicy);
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

}  // namespace zc
