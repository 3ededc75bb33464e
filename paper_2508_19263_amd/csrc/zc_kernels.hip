// HIP kernels (gfx950, wave64) of the field-split Huffman codec.
//
//   k_hist     field split + histogram over a tensor            (paper Sec. 3.1 / 3.2 / 3.4)
//   k_encode   per-chunk stream sizes (dry run) and the chunked encoder
//   k_scan     exclusive scan of the stream sizes into the chunk index
//   k_decode   chunked table-driven decode fused with the re-interleave of the fields
//
// Stream layout of one (chunk, field): the chunk's symbols are dealt to S lanes in runs of
// G symbols (16 bytes of the plain array), lane = (j / G) mod S.  A lane's codes, most
// significant bit first, form a bit string stored LSB-first in 32-bit words.  The words of
// all lanes are interleaved in the order a lock-step decoder asks for them: at every r-th
// symbol step each lane holding <= 32 unread bits takes the next word of the stream, lanes
// in ascending order.  One wavefront (or an S-lane part of it) owns one chunk, so the
// "next word" is a ballot + prefix count and both stream reads and 16-byte result writes
// are contiguous across the lanes.
#include <hip/hip_runtime.h>

#include "zc_internal.h"
#include "zc_device.h"

namespace zc {

// ------------------------------------------------------------------------ histogram
// One workgroup counts kHistBlockBytes of one tensor into LDS (8 replicas per bin to spread
// same-address atomics of skewed data) and merges into the tensor's 64-bit global bins.
// BYTES: one 256-bin histogram of the bytes (FP8: the joint (exponent, sign+mantissa)
// histogram; FP4: joint over two elements; E8M0 scales: the field itself); the host takes
// the marginals.  BF16: two histograms, exponent and sign+mantissa symbol.

// One copy of the 256 bins per LDS bank: lane l counts in copy l % 32, at word bin * 32 + l % 32, so the
// 32 lanes of an LDS pass always hit 32 different banks whatever the data is.
// FMT == 0: histogram of the bytes themselves (FP8 and FP4 elements, whose field histograms are marginals
// of the byte histogram, and the FP4 scale bytes).  Otherwise a format whose two fields have 8-bit symbols
// (BF16, the byte-grouped formats): the run is split and both fields are counted in one word, field 0 in
// the low half and field 1 in the high half: a copy is fed by 8 threads with at most 512 symbols each per
// block, so neither half can overflow.
template <int FMT>
__global__ __launch_bounds__(256) void k_hist(const TensorDev *descs, const WorkItem *work, int elem_bits_, int scales_view, uint64_t *hist, uint32_t split)
{
    constexpr bool TWO = FMT != 0;
    static_assert(kHistBlockBytes / 16 * 8 / 32 < 65536, "a copy counts at most 8 symbols per 16-byte run of the block, over 32 copies");
    __shared__ uint32_t h[256 * 32];
    // split: workgroups per block of the work list (1, 2 or 4), each counting its part of the block: a list of few blocks is
    // spread over more workgroups than the compute units hold at once, so that no second round of a few stragglers forms
    const WorkItem it = work[blockIdx.x / split];
    const uint32_t part_bytes = kHistBlockBytes / split;
    const TensorDev &d = descs[it.tensor];
    const uint8_t *p = scales_view ? d.scales : d.src;
    const uint8_t *base = scales_view ? nullptr : d.base;
    // scales_view: 0, or the number of elements per scale byte when the scale bytes are the input
    const uint64_t nbytes = scales_view ? d.n_elems / (uint32_t)scales_view : (d.n_elems * (uint64_t)elem_bits_ + 7) / 8;
    const uint64_t start = (uint64_t)it.first * kHistBlockBytes + (uint64_t)(blockIdx.x % split) * part_bytes;
    if (start >= nbytes) return;                                 // whole workgroup: the block ends before this part
    for (uint32_t i = threadIdx.x; i < 256 * 32; i += 256) h[i] = 0;
    __syncthreads();
    const uint64_t end = start + part_bytes < nbytes ? start + part_bytes : nbytes;
    uint32_t *const mine = h + (threadIdx.x & 31);
    auto count = [&](const uint4 &v, uint32_t valid) {
        if (TWO) {
            constexpr int F = TWO ? FMT : ZC_FMT_BF16;
            uint64_t P0, P1;
            split_run<F>(v, P0, P1);                      // bytes past `valid` are zero: a last partial group is zero filled
            const uint32_t nsym = (valid * 8 / Fmt<F>::EB + Fmt<F>::GRP - 1) / Fmt<F>::GRP;
#pragma unroll
            for (int i = 0; i < 8; i++)
                if ((uint32_t)i < nsym) {
                    atomicAdd(mine + ((uint32_t)(P0 >> (8 * i)) & 0xFFu) * 32, 1u);
                    atomicAdd(mine + ((uint32_t)(P1 >> (8 * i)) & 0xFFu) * 32, 0x10000u);
                }
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 16; i++)
                if ((uint32_t)i < valid) atomicAdd(mine + ((w[i >> 2] >> (8 * (i & 3))) & 0xFFu) * 32, 1u);
        }
    };
    if (end - start == part_bytes) {
        // whole part: four 16-byte loads per thread in flight at a time
        constexpr uint32_t kStep = 256 * 16;
        for (uint64_t off = start + (uint64_t)threadIdx.x * 16; off < end; off += 4 * kStep) {
            uint4 v[4];
#pragma unroll
            for (int k = 0; k < 4; k++) v[k] = *reinterpret_cast<const uint4 *>(p + off + k * kStep);
            if (base) {
#pragma unroll
                for (int k = 0; k < 4; k++) v[k] = xor4(v[k], *reinterpret_cast<const uint4 *>(base + off + k * kStep));
            }
#pragma unroll
            for (int k = 0; k < 4; k++) count(v[k], 16);
        }
    } else {
        for (uint64_t off = start + (uint64_t)threadIdx.x * 16; off < end; off += 256 * 16) {
            const uint32_t valid = end - off >= 16 ? 16u : (uint32_t)(end - off);
            uint4 v = load_run(p + off, valid);
            if (base) v = xor4(v, load_run(base + off, valid));
            count(v, valid);
        }
    }
    __syncthreads();
    // thread b sums the 32 copies of bin b, starting at a different copy per thread (different banks)
    const uint32_t bin = threadIdx.x;
    uint32_t lo = 0, hi = 0;
#pragma unroll 8
    for (uint32_t r = 0; r < 32; r++) {
        const uint32_t c = h[bin * 32 + ((r + bin) & 31)];
        if (TWO) { lo += c & 0xFFFFu; hi += c >> 16; } else lo += c;
    }
    const int slot = TWO ? 0 : (scales_view ? 2 : 0);
    if (lo) atomicAdd(reinterpret_cast<unsigned long long *>(&hist[((uint64_t)it.tensor * 3 + slot) * 256 + bin]), (unsigned long long)lo);
    if (TWO && hi) atomicAdd(reinterpret_cast<unsigned long long *>(&hist[((uint64_t)it.tensor * 3 + 1) * 256 + bin]), (unsigned long long)hi);
}

int launch_hist(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, int scales_view, uint64_t *d_hist, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    static_assert(kHistBlockBytes % (4 * 4 * 256 * 16) == 0, "a quarter of a block is whole rounds of the kernel's loads");
    // A list of so few blocks that the compute units are not full: two or four workgroups per block.  (Longer lists lose by
    // it: every workgroup clears and folds its 32 KiB of counters and adds up to 256 totals to the tensor's bins, and C3's
    // 1,344 blocks took 115 instead of 92 us in quarters.)
    const uint32_t split = n_work <= 320 ? 4u : n_work <= 640 ? 2u : 1u;
    const dim3 grid(n_work * split);
    if (fmt == ZC_FMT_BF16 && !scales_view)
        hipLaunchKernelGGL(k_hist<ZC_FMT_BF16>, grid, dim3(256), 0, st, d_descs, d_work, 16, 0, d_hist, split);
    else if (fmt == ZC_FMT_FP8_E4M3_BYTES && !scales_view)
        hipLaunchKernelGGL(k_hist<ZC_FMT_FP8_E4M3_BYTES>, grid, dim3(256), 0, st, d_descs, d_work, 8, 0, d_hist, split);
    else if (fmt == ZC_FMT_FP4_E2M1_MX_BYTES && !scales_view)
        hipLaunchKernelGGL(k_hist<ZC_FMT_FP4_E2M1_MX_BYTES>, grid, dim3(256), 0, st, d_descs, d_work, 4, 0, d_hist, split);
    else
        hipLaunchKernelGGL(k_hist<0>, grid, dim3(256), 0, st, d_descs, d_work, elem_bits(fmt), scales_view, d_hist, split);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------- chunk geometry shared by
// the encoder and the decoder: which chunk a lane group works on and how many symbols it has

uint32_t chunks_per_work_item(uint32_t streams) { return kWavesPerGroup * (64 / streams); }

struct ChunkJob {
    bool valid;
    uint32_t chunk;        // chunk id inside the tensor
    uint64_t slot;         // output slot (== chunk unless decoding an id list)
    uint64_t n_elems;      // elements in this chunk
};

// ------------------------------------------------------------------------- encoder
// One S-lane group per chunk, all fields of a run handled from one 16-byte load.
// WRITE = false is the dry run that only counts the words of every (chunk, field) stream.

struct EncField {
    uint64_t acc;          // bits not yet written, next free bit = nacc
    uint32_t nacc;
    int32_t k;             // unread bits the decoder would hold at this point
    uint32_t pend, p0, p1; // requested but unwritten words and their positions in the stream
    uint32_t wpos;         // writing: words of the stream handed out so far (same in all lanes of the group);
                           // size pass: words this lane alone has asked for (summed over the group at the end)
};

template <bool WRITE>
__device__ __forceinline__ void enc_request(EncField &F, bool active, const Lanes &L)
{
    const bool req = active && F.k <= 32;
    if (!WRITE) {                                   // positions are not needed to count words
        F.wpos += req ? 1u : 0u;
        F.k += req ? 32 : 0;
        return;
    }
    const uint64_t bm = __ballot(req) & L.gmask;
    const uint32_t pos = F.wpos + prefix_count(bm);
    F.p0 = (req && F.pend == 0) ? pos : F.p0;
    F.p1 = (req && F.pend != 0) ? pos : F.p1;
    F.pend += req ? 1u : 0u;
    F.k += req ? 32 : 0;
    F.wpos += (uint32_t)__popcll(bm);
}

template <bool WRITE>
__device__ __forceinline__ void enc_flush_word(EncField &F, uint8_t *stream)
{
    if (WRITE) reinterpret_cast<uint32_t *>(stream)[F.p0] = (uint32_t)F.acc;
    F.acc >>= 32;
    F.p0 = F.p1;
    F.pend--;
}

// encode symbols [j0, j0+R) of a run; symbol j sits at bit (j % PER64)*SB of P0 (j < PER64) or P1
template <bool WRITE, int SB, int R, bool FULL>
__device__ __forceinline__ void enc_group(EncField &F, uint64_t P0, uint64_t P1, int j0, uint32_t nsym, const uint32_t *enc, uint8_t *stream, const Lanes &L)
{
    constexpr int PER64 = 64 / SB;
    enc_request<WRITE>(F, FULL || (uint32_t)j0 < nsym, L);
    // the R codes of a refill period take at most 32 bits together (that is what defines the period)
    uint32_t code = 0, len = 0;
#pragma unroll
    for (int j = 0; j < R; j++) {
        if (FULL || (uint32_t)(j0 + j) < nsym) {
            const int jj = j0 + j;
            const uint32_t half = (uint32_t)((jj < PER64 ? P0 : P1) >> (((jj % PER64) * SB) & 32));
            const uint32_t v = (half >> (((jj % PER64) * SB) & 31)) & ((1u << SB) - 1);
            const uint32_t e = enc[v];
            if (WRITE) code |= (e & 0xFFFFu) << len;
            len += e >> 16;
        }
    }
    F.k -= (int32_t)len;
    if (WRITE) {
        F.acc |= (uint64_t)code << F.nacc;
        F.nacc += len;
        if (F.nacc >= 32) { enc_flush_word<WRITE>(F, stream); F.nacc -= 32; }
    }
}

template <bool WRITE, int SB, int G, int R, bool FULL>
__device__ __forceinline__ void enc_run_r(EncField &F, uint64_t P0, uint64_t P1, uint32_t nsym, const uint32_t *enc, uint8_t *stream, const Lanes &L)
{
#pragma unroll
    for (int j0 = 0; j0 < G; j0 += R) enc_group<WRITE, SB, R, FULL>(F, P0, P1, j0, nsym, enc, stream, L);
}

template <bool WRITE, int SB, int G, bool FULL>
__device__ __forceinline__ void enc_run(EncField &F, uint32_t period, uint64_t P0, uint64_t P1, uint32_t nsym, const uint32_t *enc, uint8_t *stream, const Lanes &L)
{
    switch (period) {
    case 2: enc_run_r<WRITE, SB, G, 2, FULL>(F, P0, P1, nsym, enc, stream, L); break;
    case 4: enc_run_r<WRITE, SB, G, 4, FULL>(F, P0, P1, nsym, enc, stream, L); break;
    case 8: enc_run_r<WRITE, SB, G, 8, FULL>(F, P0, P1, nsym, enc, stream, L); break;
    case 16: if (G >= 16) enc_run_r<WRITE, SB, G, (G >= 16 ? 16 : G), FULL>(F, P0, P1, nsym, enc, stream, L); break;
    default: if (G >= 32) enc_run_r<WRITE, SB, G, (G >= 32 ? 32 : G), FULL>(F, P0, P1, nsym, enc, stream, L); break;
    }
}

// One 64-bit run of a field whose code is flat (the canonical code of a symbol is the symbol),
// when every lane of the wavefront has a whole run: each refill step hands every lane exactly
// one word, so the run's two words sit at wpos + h*S + lane and all other encoder state
// (accumulator, look-ahead, owed words) is back at zero after the run, exactly as enc_run
// would leave it.
template <bool WRITE, int SB>
__device__ __forceinline__ void enc_flat_run(EncField &F, uint64_t P, uint8_t *stream, const Lanes &L, uint32_t S)
{
    if (WRITE) {
        uint32_t *w = reinterpret_cast<uint32_t *>(stream) + F.wpos + L.s;
        w[0] = reverse_in_groups<SB>((uint32_t)P);
        w[S] = reverse_in_groups<SB>((uint32_t)(P >> 32));
        F.wpos += 2 * S;
    } else F.wpos += 2;
}

// write the words still owed to the decoder, then zero the tail of the last 16-byte unit
template <bool WRITE>
__device__ __forceinline__ uint32_t enc_finish(EncField &F, uint8_t *stream, const Lanes &L)
{
    if (WRITE && F.pend > 0) enc_flush_word<WRITE>(F, stream);
    if (WRITE && F.pend > 0) enc_flush_word<WRITE>(F, stream);
    uint32_t words = F.wpos;
    if (!WRITE)                                     // per-lane counts: sum over the lanes of the group
        for (uint32_t o = 1; o < 64; o <<= 1) { const uint32_t y = __shfl_xor(words, o, 64); words += o < (uint32_t)__popcll(L.gmask) ? y : 0u; }
    if (WRITE && L.s == 0)
        for (uint32_t w = words; w & 3; w++) reinterpret_cast<uint32_t *>(stream)[w] = 0;
    return (words + 3) / 4;
}

// Encoder body for the symbols of one field kind.  ELEM = true: fields 0 and 1 of the
// element array; false: the FP4 scale field.
// WHOLE: the launch covers only whole chunks of tensors with 64 lanes per chunk (one wavefront per chunk, every
// run complete), which lets the compiler drop the lane-group masks and every partial-run path.
// shared (WHOLE only): a work item is ONE chunk for the four wavefronts of the workgroup.  When both element
// fields are stored plainly (flat code, raw, constant) its rows do not depend on each other: the encoder gives
// every wavefront a quarter of them, and the size pass needs no element data at all.  Otherwise the first
// wavefront takes the chunk alone.  The host asks for this where plain element fields are the rule (FP4): four
// times the wavefronts hide four times the memory latency, which is what bounds a set of few chunks.
template <int FMT, bool WRITE, bool WHOLE>
__global__ __launch_bounds__(256) void k_encode(const TensorDev *descs, const WorkItem *work, const uint32_t *enc_tables, uint32_t *units, int skip_routes,
                                                int shared_chunk)
{
    using F_ = Fmt<FMT>;
    __shared__ uint32_t enc[3][256];
    __shared__ TensorDev dsh;                       // a copy the compiler knows no store of this kernel can change
    const WorkItem it = work[blockIdx.x];
    // whole workgroup: these chunks belong to a specialised kernel (bit r of skip_routes: leave tensors of route r alone)
    if ((skip_routes >> descs[it.tensor].route) & 1) return;
    if (threadIdx.x == 0) dsh = descs[it.tensor];
    for (uint32_t i = threadIdx.x; i < 3 * 256; i += 256) (&enc[0][0])[i] = enc_tables[(uint64_t)it.tensor * 768 + i];
    __syncthreads();
    const TensorDev &d = dsh;
    const uint32_t S = WHOLE ? 64u : d.streams;
    const Lanes L = make_lanes(S);
    const uint32_t wave = threadIdx.x >> 6;
    const bool shared = WHOLE && shared_chunk;
    const uint32_t chunk = shared ? it.first : it.first + wave * (64 / S) + L.grp;
    const uint64_t E = (uint64_t)d.chunk_bytes * 8 / F_::EB;
    const uint64_t first = (uint64_t)chunk * E;
    // WHOLE: the host lists only whole chunks, up to four per work item; a wavefront beyond the last one idles
    const bool valid = WHOLE ? first + E <= d.n_elems : chunk < d.n_chunks;
    const uint32_t n = valid ? (uint32_t)(d.n_elems - first < E ? d.n_elems - first : E) : 0;
    const uint32_t *index[3];
    uint8_t *stream[3] = {nullptr, nullptr, nullptr};
    for (int f = 0; f < F_::NF; f++) {
        index[f] = reinterpret_cast<const uint32_t *>(d.comp + d.index_off[f]);
        if (WRITE && valid) stream[f] = d.comp + d.payload_off + 16ull * index[f][chunk];
    }
    uint32_t *my_units = units + d.units_off;

    // ---- element fields ----
    constexpr bool kWide = F_::G * F_::SB > 64;
    EncField F0 = {0, 0, 0, 0, 0, 0, 0}, F1 = F0;
    const uint32_t chunk_runs = (uint32_t)((E + F_::EPR - 1) / F_::EPR);
    const uint32_t rows = (chunk_runs + S - 1) / S;
    const uint8_t *src = d.src + (uint64_t)chunk * d.chunk_bytes;
    const uint8_t *base = d.base ? d.base + (uint64_t)chunk * d.chunk_bytes : nullptr;
    const uint32_t nbytes = (uint32_t)(((uint64_t)n * F_::EB + 7) / 8);
    const uint32_t m0 = d.mode[0], m1 = d.mode[1], kind0 = d.kind[0], kind1 = d.kind[1], per0 = d.period[0], per1 = d.period[1];
    if (WHOLE && !valid) return;                    // nothing below synchronises the workgroup
    // a field whose rows can be placed without knowing the rows before them
    const bool plain0 = !(m0 == ZC_MODE_HUFF && (kWide || kind0 != 1)), plain1 = !(m1 == ZC_MODE_HUFF && (kWide || kind1 != 1));
    const bool plain = plain0 && plain1;
    if (shared && !plain && wave != 0) return;
    uint32_t row_begin = 0, row_end = rows;
    if (shared && plain) shared_chunk_rows(rows, F_::NF == 3 ? (uint32_t)((E / F_::SCALE + 1023) / 1024) : 0u, wave, row_begin, row_end);
    if (WHOLE && !WRITE && plain) {
        // size pass: a flat code takes two words per run whatever the data, raw and constant fields are sized below
        if (m0 == ZC_MODE_HUFF) F0.wpos = 2 * rows;
        if (m1 == ZC_MODE_HUFF) F1.wpos = 2 * rows;
        row_end = row_begin;
        if (shared && wave != 0) return;
    } else if (shared && plain) {
        // a flat field's words lie row by row: start where this wavefront's rows start
        F0.wpos = 2 * S * row_begin; F1.wpos = 2 * S * row_begin;
    }
    for (uint32_t i = row_begin; i < row_end; i++) {
        const uint32_t run = i * S + L.s;
        const uint32_t done = run * F_::EPR;                                                       // elements before this run
        const uint32_t nel = WHOLE ? (uint32_t)F_::EPR : (n > done ? (n - done < (uint32_t)F_::EPR ? n - done : (uint32_t)F_::EPR) : 0);
        const uint32_t nsym = (nel + F_::GRP - 1) / F_::GRP;                                       // a last partial group is filled with zeros
        // a field's symbols of this run: P (and Q where a run is 16 symbols of 8 bits)
        uint64_t P0 = 0, P1 = 0, Q0 = 0, Q1 = 0;
        if (nsym) {
            const uint32_t vb = nbytes - run * 16;
            uint4 v = load_run(src + (uint64_t)run * 16, vb);
            if (base) v = xor4(v, load_run(base + (uint64_t)run * 16, vb));
            split_run4<FMT>(v, P0, Q0, P1, Q1);
        }
        const bool full = WHOLE || __all(nsym == (uint32_t)F_::G);
        // the direct path of a flat code is written for one 64-bit word per run; a wide field cannot be flat
        // anyway (its alphabet of 256 is never used in full)
        if (!kWide && m0 == ZC_MODE_HUFF && kind0 == 1 && full) enc_flat_run<WRITE, F_::SB>(F0, P0, stream[0], L, S);
        else if (m0 == ZC_MODE_HUFF) {
            if (full) enc_run<WRITE, F_::SB, F_::G, true>(F0, per0, P0, Q0, nsym, enc[0], stream[0], L);
            else if (!WHOLE) enc_run<WRITE, F_::SB, F_::G, false>(F0, per0, P0, Q0, nsym, enc[0], stream[0], L);
        } else if (m0 == ZC_MODE_RAW && WRITE && nsym) {
            if (kWide) { reinterpret_cast<uint64_t *>(stream[0])[2 * run] = P0; reinterpret_cast<uint64_t *>(stream[0])[2 * run + 1] = Q0; }
            else {
                reinterpret_cast<uint64_t *>(stream[0])[run] = P0;
                if ((run & 1) == 0 && done + F_::EPR >= n) reinterpret_cast<uint64_t *>(stream[0])[run + 1] = 0;
            }
        }
        if (!kWide && m1 == ZC_MODE_HUFF && kind1 == 1 && full) enc_flat_run<WRITE, F_::SB>(F1, P1, stream[1], L, S);
        else if (m1 == ZC_MODE_HUFF) {
            if (full) enc_run<WRITE, F_::SB, F_::G, true>(F1, per1, P1, Q1, nsym, enc[1], stream[1], L);
            else if (!WHOLE) enc_run<WRITE, F_::SB, F_::G, false>(F1, per1, P1, Q1, nsym, enc[1], stream[1], L);
        } else if (m1 == ZC_MODE_RAW && WRITE && nsym) {
            if (kWide) { reinterpret_cast<uint64_t *>(stream[1])[2 * run] = P1; reinterpret_cast<uint64_t *>(stream[1])[2 * run + 1] = Q1; }
            else {
                reinterpret_cast<uint64_t *>(stream[1])[run] = P1;
                if ((run & 1) == 0 && done + F_::EPR >= n) reinterpret_cast<uint64_t *>(stream[1])[run + 1] = 0;
            }
        }
        }
    {
        uint32_t u0 = 0, u1 = 0;
        const uint32_t nsyms = (n + F_::GRP - 1) / F_::GRP;
        if (m0 == ZC_MODE_HUFF) u0 = enc_finish<WRITE>(F0, stream[0], L);
        else if (m0 == ZC_MODE_RAW) u0 = (uint32_t)((((uint64_t)nsyms * F_::SB + 7) / 8 + 15) / 16);
        if (m1 == ZC_MODE_HUFF) u1 = enc_finish<WRITE>(F1, stream[1], L);
        else if (m1 == ZC_MODE_RAW) u1 = (uint32_t)((((uint64_t)nsyms * F_::SB + 7) / 8 + 15) / 16);
        if (!WRITE && valid && L.s == 0) { my_units[chunk] = u0; my_units[d.n_chunks + chunk] = u1; }
    }

    // ---- FP4 block scales: one byte per 32 elements, runs of 16 bytes ----
    if (F_::NF == 3 && !(shared && wave != 0)) {
        EncField F2 = {0, 0, 0, 0, 0, 0, 0};
        const uint32_t ns = n / F_::SCALE;
        const uint32_t srows = (uint32_t)((E / F_::SCALE + 15) / 16 + S - 1) / S;
        const uint8_t *sc = d.scales + (uint64_t)chunk * (E / F_::SCALE);
        const uint32_t m2 = d.mode[2];
        for (uint32_t i = 0; i < srows; i++) {
            const uint32_t run = i * S + L.s;
            const uint32_t done = run * 16;
            const uint32_t nsym = ns > done ? (ns - done < 16u ? ns - done : 16u) : 0;
            uint64_t P0 = 0, P1 = 0;
            if (nsym) {
                const uint4 v = load_run(sc + (uint64_t)run * 16, nsym);
                P0 = (uint64_t)v.x | ((uint64_t)v.y << 32);
                P1 = (uint64_t)v.z | ((uint64_t)v.w << 32);
            }
            const bool full = __all(nsym == 16u);
            if (m2 == ZC_MODE_HUFF) {
                if (full) enc_run<WRITE, 8, 16, true>(F2, d.period[2], P0, P1, nsym, enc[2], stream[2], L);
                else enc_run<WRITE, 8, 16, false>(F2, d.period[2], P0, P1, nsym, enc[2], stream[2], L);
            } else if (m2 == ZC_MODE_RAW && WRITE && nsym) {
                reinterpret_cast<uint64_t *>(stream[2])[2 * run] = P0;
                reinterpret_cast<uint64_t *>(stream[2])[2 * run + 1] = P1;
            }
        }
        uint32_t u2 = 0;
        if (m2 == ZC_MODE_HUFF) u2 = enc_finish<WRITE>(F2, stream[2], L);
        else if (m2 == ZC_MODE_RAW) u2 = (ns + 15) / 16;
        if (!WRITE && valid && L.s == 0) my_units[2 * d.n_chunks + chunk] = u2;
    }
}

template <int FMT, bool WRITE>
static void launch_encode_f(int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, hipStream_t st)
{
    if (whole) hipLaunchKernelGGL((k_encode<FMT, WRITE, true>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, skip_routes, whole == 2 ? 1 : 0);
    else hipLaunchKernelGGL((k_encode<FMT, WRITE, false>), dim3(n_work), dim3(256), 0, st, d_descs, d_work, d_enc, d_units, skip_routes, 0);
}

template <bool WRITE>
static int launch_encode_t(uint32_t fmt, int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, hipStream_t st)
{
    if (n_work == 0) return 0;
    switch (fmt) {
    case ZC_FMT_BF16: launch_encode_f<ZC_FMT_BF16, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP8_E4M3: launch_encode_f<ZC_FMT_FP8_E4M3, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP4_E2M1_MX: launch_encode_f<ZC_FMT_FP4_E2M1_MX, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP8_E4M3_BYTES: launch_encode_f<ZC_FMT_FP8_E4M3_BYTES, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP4_E2M1_MX_BYTES: launch_encode_f<ZC_FMT_FP4_E2M1_MX_BYTES, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP4_E2M1_NV: launch_encode_f<ZC_FMT_FP4_E2M1_NV, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    case ZC_FMT_FP8_E5M2: launch_encode_f<ZC_FMT_FP8_E5M2, WRITE>(whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, st); break;
    default: return 1;
    }
    return (int)hipGetLastError();
}

// whole: 1 = every work item is up to four whole chunks of a tensor with 64 lanes per chunk and chunks of whole
// 1 KiB rows; 2 = every work item is one such chunk, shared by the workgroup's four wavefronts; 0 = any chunks
int launch_sizes(uint32_t fmt, int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, uint32_t *d_units, void *stream)
{
    return launch_encode_t<false>(fmt, whole, skip_routes, d_descs, d_work, n_work, d_enc, d_units, (hipStream_t)stream);
}

int launch_encode(uint32_t fmt, int whole, int skip_routes, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, const uint32_t *d_enc, void *stream)
{
    return launch_encode_t<true>(fmt, whole, skip_routes, d_descs, d_work, n_work, d_enc, nullptr, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------- scan
// One workgroup per tensor: exclusive scan of the stream sizes (16-byte units) in
// field-major order, the fields in the payload's order (reversed: the last field first).  Writes the container's prologue (header and code-length tables as prepared in the
// tensor's blob, when blobs is given), the chunk index with the zero padding behind it and the total size into
// the container (when there is one), and the per-field totals for the host.

__global__ __launch_bounds__(1024) void k_scan(const TensorDev *descs, int n_fields, int reversed, int skip_routes, const uint32_t *units, ScanOut *out,
                                               const uint8_t *blobs, uint32_t blob_bytes)
{
    __shared__ uint32_t wave_sum[16];
    __shared__ uint32_t carry_s;
    // whole workgroup: a tensor of such a route has been placed and written by another kernel (bit r: route r)
    if ((skip_routes >> descs[blockIdx.x].route) & 1) return;
    // copies of what is needed from the descriptor: the stores below could alias it as far as the compiler knows
    const TensorDev &dg = descs[blockIdx.x];
    struct { uint8_t *comp; uint32_t n_chunks, index_off[kMaxFields]; uint64_t payload_off; } d;
    d.comp = dg.comp; d.n_chunks = dg.n_chunks; d.payload_off = dg.payload_off;
    for (int f = 0; f < kMaxFields; f++) d.index_off[f] = dg.index_off[f];
    const uint32_t *u = units + dg.units_off;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    if (d.comp && blobs) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(blobs + (uint64_t)blockIdx.x * blob_bytes);
        uint32_t *dst = reinterpret_cast<uint32_t *>(d.comp);
        for (uint32_t i = threadIdx.x; i < d.index_off[0] / 4; i += 1024) dst[i] = src[i];
        if (threadIdx.x < 4 * (uint32_t)n_fields) {
            const uint32_t f = threadIdx.x / 4, w = d.n_chunks + 1 + (threadIdx.x & 3);
            if (w < ((d.n_chunks + 1 + 3) & ~3u)) dst[d.index_off[f] / 4 + w] = 0;
        }
    }
    __syncthreads();                                             // the total size below overwrites a word of the prologue
    uint32_t field_units[kMaxFields] = {0, 0, 0};
    for (int k = 0; k < n_fields; k++) {
        const int f = reversed ? n_fields - 1 - k : k;
        uint32_t *index = d.comp ? reinterpret_cast<uint32_t *>(d.comp + d.index_off[f]) : nullptr;
        const uint32_t field_start = carry_s;
        // eight consecutive chunks per thread and pass: a tensor of pages has tens of thousands of chunks, and every
        // pass costs three workgroup barriers
        constexpr uint32_t K = 8;
        for (uint32_t c0 = 0; c0 < d.n_chunks; c0 += 1024 * K) {
            const uint32_t c = c0 + threadIdx.x * K;
            uint32_t v[K], t = 0;
#pragma unroll
            for (uint32_t j = 0; j < K; j++) { v[j] = c + j < d.n_chunks ? u[(uint64_t)f * d.n_chunks + c + j] : 0; t += v[j]; }
            uint32_t x = t;                                   // inclusive scan of the threads' sums inside the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t y = __shfl_up(x, o, 64);
                if (lane >= (uint32_t)o) x += y;
            }
            if (lane == 63) wave_sum[wave] = x;
            __syncthreads();
            uint32_t before = carry_s;
            for (uint32_t w = 0; w < wave; w++) before += wave_sum[w];
            uint32_t at = before + x - t;                     // units before this thread's first chunk
            if (index) {
#pragma unroll
                for (uint32_t j = 0; j < K; j++) { if (c + j < d.n_chunks) index[c + j] = at; at += v[j]; }
            }
            __syncthreads();
            if (threadIdx.x == 1023) carry_s = before + x;
            __syncthreads();
        }
        if (index && threadIdx.x == 0) index[d.n_chunks] = carry_s;
        field_units[f] = carry_s - field_start;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        ScanOut o = {{0, 0, 0}, 0};
        for (int f = 0; f < n_fields; f++) o.field_units[f] = field_units[f];
        o.total_units = carry_s;
        out[blockIdx.x] = o;
        if (d.comp) *reinterpret_cast<uint64_t *>(d.comp + 48) = d.payload_off + 16ull * carry_s;
    }
}

int launch_scan(const TensorDev *d_descs, uint32_t n_tensors, int n_fields, bool reversed, int skip_routes, const uint32_t *d_units, ScanOut *d_out,
                const uint8_t *d_blobs, uint32_t blob_bytes, void *stream)
{
    if (n_tensors == 0) return 0;
    hipLaunchKernelGGL(k_scan, dim3(n_tensors), dim3(1024), 0, (hipStream_t)stream, d_descs, n_fields, reversed ? 1 : 0, skip_routes, d_units, d_out, d_blobs,
                       blob_bytes);
    return (int)hipGetLastError();
}

// Zero the histogram counters.  A kernel rather than a memset call: the compress sequence then consists of kernel
// launches only once its descriptors and work lists are in the workspace (memset nodes recorded into a HIP graph
// have given wrong results on replays, so none is ever queued by this library).
__global__ __launch_bounds__(256) void k_zero(uint64_t *p, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

int launch_zero(uint64_t *d_words, uint64_t n_words, void *stream)
{
    if (n_words == 0) return 0;
    hipLaunchKernelGGL(k_zero, dim3((uint32_t)((n_words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, d_words, n_words);
    return (int)hipGetLastError();
}

// Plain copy, linear through memory, 16 bytes per thread and a workgroup per 4 KiB: the launch shape that moves the
// most bytes per second on this machine (workgroups that loop over the buffer, and hipMemcpy, reach 75 - 85 % of
// it).  The yardstick next to which the codec's throughput is reported, and the kernel of known traffic that scales
// the hardware's byte counters.
__global__ __launch_bounds__(256) void k_copy(const uint4 *src, uint4 *dst, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// The same bytes moved the way the 64-lane decoders and encoders move them: one wavefront per chunk, walking through
// its own chunk 1 KiB (16 bytes per lane) at a time, four loads in flight, thousands of chunks at once.  What this
// reaches is the ceiling of every kernel here that streams one chunk per wavefront.
__global__ __launch_bounds__(256) void k_copy_chunked(const uint8_t *src, uint8_t *dst, uint64_t n_chunks, uint32_t chunk_bytes)
{
    const uint64_t chunk = (uint64_t)blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
    if (chunk >= n_chunks) return;
    const uint32_t lane = threadIdx.x & 63, rows = chunk_bytes / 1024;
    const uint4 *s = reinterpret_cast<const uint4 *>(src + chunk * chunk_bytes) + lane;
    uint4 *d = reinterpret_cast<uint4 *>(dst + chunk * chunk_bytes) + lane;
    uint32_t row = 0;
    for (; row + 4 <= rows; row += 4) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = s[(uint64_t)(row + k) * 64];
#pragma unroll
        for (int k = 0; k < 4; k++) d[(uint64_t)(row + k) * 64] = v[k];
    }
    for (; row < rows; row++) d[(uint64_t)row * 64] = s[(uint64_t)row * 64];
}

int launch_copy_chunked(const void *d_src, void *d_dst, uint64_t bytes, uint32_t chunk_bytes, void *stream)
{
    const uint64_t n_chunks = bytes / chunk_bytes;
    if (n_chunks == 0) return 0;
    hipLaunchKernelGGL(k_copy_chunked, dim3((uint32_t)((n_chunks + kWavesPerGroup - 1) / kWavesPerGroup)), dim3(256), 0, (hipStream_t)stream,
                       (const uint8_t *)d_src, (uint8_t *)d_dst, n_chunks, chunk_bytes);
    return (int)hipGetLastError();
}

int launch_copy(const void *d_src, void *d_dst, uint64_t bytes, void *stream)
{
    const uint64_t n16 = bytes / 16;
    if (n16 == 0) return 0;
    const uint64_t blocks = (n16 + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(k_copy, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4 *)d_src, (uint4 *)d_dst, n16);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------- decoder
struct DecField {
    uint32_t lo, hi;       // 64 stream bits, next unread bit = bit c of {hi, lo}
    uint32_t c;
    uint32_t wpos;         // words of the stream taken so far by the group
    const uint8_t *ptr;    // stream start
    uint32_t words;        // stream length in words (reads beyond it return 0)
    // The next words of the stream, fetched ahead of use: lane s of the group holds word base + s in `cur` and
    // word base + S + s in `nxt` (base <= wpos < base + S).  A refill step hands out at most S words, all inside
    // these two windows, so a lane gets its word from the lane that holds it instead of waiting for memory.
    uint32_t base, cur, nxt;
};

__device__ __forceinline__ uint32_t stream_word(const DecField &D, uint32_t pos)
{
    return pos < D.words ? reinterpret_cast<const uint32_t *>(D.ptr)[pos] : 0u;
}

__device__ __forceinline__ void dec_refill(DecField &D, bool active, const Lanes &L)
{
    const uint32_t S = (uint32_t)__popcll(L.gmask);
    const bool need = active && D.c >= 32;
    const uint64_t bm = __ballot(need) & L.gmask;
    const uint32_t at = D.wpos + prefix_count(bm) - D.base;                 // 0 .. 2S-1 in the lanes that ask
    const int holder = (int)((threadIdx.x & 63u) - L.s + (at & (S - 1)));
    const uint32_t a = (uint32_t)__shfl((int)D.cur, holder, 64), b = (uint32_t)__shfl((int)D.nxt, holder, 64);
    if (need) { D.lo = D.hi; D.hi = at < S ? a : b; D.c -= 32; }
    D.wpos += (uint32_t)__popcll(bm);
    if (D.wpos - D.base >= S) {                                             // the first window is used up
        D.cur = D.nxt;
        D.base += S;
        D.nxt = stream_word(D, D.base + S + L.s);
    }
}

// decode symbols [j0, j0+R) of a run; symbol j goes to bit (j % PER64)*SB of P0 (j < PER64) or P1
template <int SB, int R, bool FULL>
__device__ __forceinline__ void dec_group(DecField &D, const FieldTab &T, uint64_t &P0, uint64_t &P1, int j0, uint32_t nsym, const Lanes &L)
{
    constexpr int PER64 = 64 / SB;
    dec_refill(D, FULL || (uint32_t)j0 < nsym, L);
    uint32_t x = (uint32_t)((((uint64_t)D.hi << 32) | D.lo) >> D.c);
    const uint32_t mask = T.mask;
#pragma unroll
    for (int j = 0; j < R; j++) {
        if (FULL || (uint32_t)(j0 + j) < nsym) {
            const int jj = j0 + j;
            uint32_t e = T.lut[x & mask];
            if (e == 0) e = dec_long(T, x);
            x >>= (e & 31u);
            D.c += (e & 31u);
            if (jj < PER64) P0 |= (uint64_t)(e >> 8) << ((jj % PER64) * SB);
            else P1 |= (uint64_t)(e >> 8) << ((jj % PER64) * SB);
        }
    }
}

template <int SB, int G, int R, bool FULL>
__device__ __forceinline__ void dec_run_r(DecField &D, const FieldTab &T, uint64_t &P0, uint64_t &P1, uint32_t nsym, const Lanes &L)
{
#pragma unroll
    for (int j0 = 0; j0 < G; j0 += R) dec_group<SB, R, FULL>(D, T, P0, P1, j0, nsym, L);
}

template <int SB, int G, bool FULL>
__device__ __forceinline__ void dec_run(DecField &D, const FieldTab &T, uint32_t period, uint64_t &P0, uint64_t &P1, uint32_t nsym, const Lanes &L)
{
    switch (period) {
    case 2: dec_run_r<SB, G, 2, FULL>(D, T, P0, P1, nsym, L); break;
    case 4: dec_run_r<SB, G, 4, FULL>(D, T, P0, P1, nsym, L); break;
    case 8: dec_run_r<SB, G, 8, FULL>(D, T, P0, P1, nsym, L); break;
    case 16: if (G >= 16) dec_run_r<SB, G, (G >= 16 ? 16 : G), FULL>(D, T, P0, P1, nsym, L); break;
    default: if (G >= 32) dec_run_r<SB, G, (G >= 32 ? 32 : G), FULL>(D, T, P0, P1, nsym, L); break;
    }
}

__device__ __forceinline__ DecField open_stream(const TensorDev &d, int f, uint32_t chunk, bool valid, const Lanes &L)
{
    DecField D = {0, 0, 64, 0, d.comp, 0, 0, 0, 0};
    if (valid && (d.mode[f] == ZC_MODE_HUFF || d.mode[f] == ZC_MODE_RAW)) {
        const uint32_t *index = reinterpret_cast<const uint32_t *>(d.comp + d.index_off[f]);
        const uint64_t a = index[chunk], b = index[chunk + 1];
        const uint64_t lo = d.payload_off + 16 * a, hi = d.payload_off + 16 * b;
        if (a <= b && hi <= d.total_bytes) { D.ptr = d.comp + lo; D.words = (uint32_t)((hi - lo) / 4); }
    }
    if (d.mode[f] == ZC_MODE_HUFF) {
        const uint32_t S = (uint32_t)__popcll(L.gmask);
        D.cur = stream_word(D, L.s);
        D.nxt = stream_word(D, S + L.s);
    }
    return D;
}

// A field with a flat code (every symbol coded by its own bits, most significant first) on rows where every lane of the
// wavefront holds a whole run: each lane takes one word per 32 / SB symbols and no look-ahead, so the words of row i
// are (i * WPR + h) * S + lane of the group, h < WPR, and need no table.  The first row that is not whole (the last
// of a short chunk) goes through the table again: flat_leave puts the stream state where that row starts.
template <int SB, int G>
__device__ __forceinline__ void flat_row(const DecField &D, uint32_t row, uint32_t S, uint32_t s, uint64_t &P, uint64_t &Q)
{
    constexpr int WPR = G * SB / 32;
    uint32_t w[WPR];
#pragma unroll
    for (int h = 0; h < WPR; h++) w[h] = reverse_in_groups<SB>(stream_word(D, (row * WPR + h) * S + s));
    P = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    if (WPR == 4) Q = (uint64_t)w[2] | ((uint64_t)w[3] << 32);
}

template <int SB, int G>
__device__ __forceinline__ void flat_leave(DecField &D, uint32_t row, uint32_t S, uint32_t s)
{
    constexpr int WPR = G * SB / 32;
    D.c = 64; D.lo = 0; D.hi = 0;                    // nothing unread: the row's first step takes a word
    D.wpos = row * WPR * S;
    D.base = D.wpos;
    D.cur = stream_word(D, D.base + s);
    D.nxt = stream_word(D, D.base + S + s);
}

template <int FMT>
__global__ __launch_bounds__(256) void k_decode(const TensorDev *descs, const WorkItem *work, TensorDev single, int use_single,
                                                uint32_t first_slot)
{
    using F_ = Fmt<FMT>;
    __shared__ FieldTab tab[F_::NF];
    __shared__ TensorDev dsh;
    WorkItem it;
    if (use_single) { it.tensor = 0; it.first = first_slot + blockIdx.x * kWavesPerGroup * (64 / single.streams); }
    else it = work[blockIdx.x];
    if (threadIdx.x == 0) dsh = use_single ? single : descs[it.tensor];
    __syncthreads();
    const TensorDev &d = dsh;
    for (int f = 0; f < F_::NF; f++)
        if (d.mode[f] == ZC_MODE_HUFF) build_field_tab(tab[f], d.comp + d.table_off[f], 1 << (f == 2 ? 8 : F_::SB), d.lmax[f]);
    const uint32_t S = d.streams;
    const Lanes L = make_lanes(S);
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t slot = it.first + wave * (64 / S) + L.grp;
    uint32_t chunk = slot;
    bool valid = slot < d.n_chunks;
    const uint32_t *ids = d.ids;
    if (ids) { valid = slot < d.n_ids; chunk = valid ? ids[slot] : 0; valid = valid && chunk < d.n_chunks; }
    const uint64_t E = (uint64_t)d.chunk_bytes * 8 / F_::EB;
    const uint64_t first = (uint64_t)chunk * E;
    const uint32_t n = valid ? (uint32_t)(d.n_elems - first < E ? d.n_elems - first : E) : 0;
    const uint32_t nbytes = (uint32_t)(((uint64_t)n * F_::EB + 7) / 8);
    uint8_t *dst = d.dst + (uint64_t)slot * d.chunk_bytes;
    const uint8_t *base = d.base ? d.base + (uint64_t)chunk * d.chunk_bytes : nullptr;

    DecField D0 = open_stream(d, 0, chunk, valid, L), D1 = open_stream(d, 1, chunk, valid, L);
    const uint32_t m0 = d.mode[0], m1 = d.mode[1];
    const uint64_t K0 = splat(d.konst[0], F_::SB), K1 = splat(d.konst[1], F_::SB);
    const uint32_t chunk_runs = (uint32_t)((E + F_::EPR - 1) / F_::EPR);
    const uint32_t rows = (chunk_runs + S - 1) / S;
    // flat-coded fields are read directly while the rows are whole (the same in all lanes: `full` is a wavefront vote)
    bool direct0 = m0 == ZC_MODE_HUFF && d.kind[0] == 1, direct1 = m1 == ZC_MODE_HUFF && d.kind[1] == 1;
    for (uint32_t i = 0; i < rows; i++) {
        const uint32_t run = i * S + L.s;
        const uint32_t done = run * F_::EPR;                                                       // elements before this run
        const uint32_t nel = n > done ? (n - done < (uint32_t)F_::EPR ? n - done : (uint32_t)F_::EPR) : 0;
        const uint32_t nsym = (nel + F_::GRP - 1) / F_::GRP;                                       // a last partial group is filled with zeros
        const bool full = __all(nsym == (uint32_t)F_::G);
        constexpr bool kWide = F_::G * F_::SB > 64;
        uint64_t P0 = 0, P1 = 0, Q0 = 0, Q1 = 0;       // Q: symbols 8..15 of a run of 16 symbols of 8 bits
        if (!full) {
            if (direct0) { flat_leave<F_::SB, F_::G>(D0, i, S, L.s); direct0 = false; }
            if (direct1) { flat_leave<F_::SB, F_::G>(D1, i, S, L.s); direct1 = false; }
        }
        if (direct0) flat_row<F_::SB, F_::G>(D0, i, S, L.s, P0, Q0);
        else if (m0 == ZC_MODE_HUFF) {
            if (full) dec_run<F_::SB, F_::G, true>(D0, tab[0], d.period[0], P0, Q0, nsym, L);
            else dec_run<F_::SB, F_::G, false>(D0, tab[0], d.period[0], P0, Q0, nsym, L);
        } else if (m0 == ZC_MODE_RAW) {
            if (kWide) { if (nsym && 4 * run + 3 < D0.words) { P0 = reinterpret_cast<const uint64_t *>(D0.ptr)[2 * run]; Q0 = reinterpret_cast<const uint64_t *>(D0.ptr)[2 * run + 1]; } }
            else if (nsym && 2 * run + 1 < D0.words) P0 = reinterpret_cast<const uint64_t *>(D0.ptr)[run];
        } else { P0 = K0; Q0 = K0; }
        if (direct1) flat_row<F_::SB, F_::G>(D1, i, S, L.s, P1, Q1);
        else if (m1 == ZC_MODE_HUFF) {
            if (full) dec_run<F_::SB, F_::G, true>(D1, tab[1], d.period[1], P1, Q1, nsym, L);
            else dec_run<F_::SB, F_::G, false>(D1, tab[1], d.period[1], P1, Q1, nsym, L);
        } else if (m1 == ZC_MODE_RAW) {
            if (kWide) { if (nsym && 4 * run + 3 < D1.words) { P1 = reinterpret_cast<const uint64_t *>(D1.ptr)[2 * run]; Q1 = reinterpret_cast<const uint64_t *>(D1.ptr)[2 * run + 1]; } }
            else if (nsym && 2 * run + 1 < D1.words) P1 = reinterpret_cast<const uint64_t *>(D1.ptr)[run];
        } else { P1 = K1; Q1 = K1; }
        if (nsym) {
            const uint32_t vb = nbytes - run * 16;
            uint4 v = join_run4<FMT>(P0, Q0, P1, Q1);
            if (base) v = xor4(v, load_run(base + (uint64_t)run * 16, vb));
            store_run(dst + (uint64_t)run * 16, v, vb);
        }
    }

    if (F_::NF == 3) {
        DecField D2 = open_stream(d, F_::NF - 1, chunk, valid, L);
        const uint32_t m2 = d.mode[F_::NF - 1];
        const uint32_t ns = n / F_::SCALE;
        const uint32_t srows = (uint32_t)((E / F_::SCALE + 15) / 16 + S - 1) / S;
        uint8_t *sc = d.scales_out + (uint64_t)slot * (E / F_::SCALE);
        const uint64_t K2 = splat(d.konst[F_::NF - 1], 8);
        for (uint32_t i = 0; i < srows; i++) {
            const uint32_t run = i * S + L.s;
            const uint32_t done = run * 16;
            const uint32_t nsym = ns > done ? (ns - done < 16u ? ns - done : 16u) : 0;
            const bool full = __all(nsym == 16u);
            uint64_t P0 = 0, P1 = 0;
            if (m2 == ZC_MODE_HUFF) {
                if (full) dec_run<8, 16, true>(D2, tab[F_::NF - 1], d.period[F_::NF - 1], P0, P1, nsym, L);
                else dec_run<8, 16, false>(D2, tab[F_::NF - 1], d.period[F_::NF - 1], P0, P1, nsym, L);
            } else if (m2 == ZC_MODE_RAW) {
                if (nsym && 4 * run + 3 < D2.words) { P0 = reinterpret_cast<const uint64_t *>(D2.ptr)[2 * run]; P1 = reinterpret_cast<const uint64_t *>(D2.ptr)[2 * run + 1]; }
            } else { P0 = K2; P1 = K2; }
            if (nsym) store_run(sc + (uint64_t)run * 16, make_uint4((uint32_t)P0, (uint32_t)(P0 >> 32), (uint32_t)P1, (uint32_t)(P1 >> 32)), nsym);
        }
    }
}

int launch_decode(uint32_t fmt, const TensorDev *d_descs, const WorkItem *d_work, uint32_t n_work, uint32_t,
                  const TensorDev *single, uint32_t first_slot, void *stream)
{
    if (n_work == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    TensorDev s = single ? *single : TensorDev{};
    const int use_single = single ? 1 : 0;
    switch (fmt) {
    case ZC_FMT_BF16: hipLaunchKernelGGL(k_decode<ZC_FMT_BF16>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP8_E4M3: hipLaunchKernelGGL(k_decode<ZC_FMT_FP8_E4M3>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP4_E2M1_MX: hipLaunchKernelGGL(k_decode<ZC_FMT_FP4_E2M1_MX>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP8_E4M3_BYTES: hipLaunchKernelGGL(k_decode<ZC_FMT_FP8_E4M3_BYTES>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP4_E2M1_MX_BYTES: hipLaunchKernelGGL(k_decode<ZC_FMT_FP4_E2M1_MX_BYTES>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP4_E2M1_NV: hipLaunchKernelGGL(k_decode<ZC_FMT_FP4_E2M1_NV>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    case ZC_FMT_FP8_E5M2: hipLaunchKernelGGL(k_decode<ZC_FMT_FP8_E5M2>, dim3(n_work), dim3(256), 0, st, d_descs, d_work, s, use_single, first_slot); break;
    default: return 1;
    }
    return (int)hipGetLastError();
}

}  // namespace zc
