// zc_compress_noalloc: compression of one tensor for callers that cannot allocate (code under HIP graph
// capture, tight serving loops, harnesses that forbid allocation).  The workspace that the other compress calls
// take from the caller is a file-scope device array here, and what they upload from page-locked host memory
// (descriptor, blank header, work lists) is written into it by a small kernel from its arguments.  The call makes
// kernel launches and nothing else: no hipMalloc / hipHostMalloc / hipFree, no copy, no wait, no heap memory.
#include <hip/hip_runtime.h>

#include <mutex>

#include "zc_host.h"

namespace zc {

namespace {

// Everything plan_workspace() lays out for one tensor must fit here: descriptor, work lists (8 bytes per histogram
// block and per work item), encode tables, histograms, 4 bytes per (chunk, field), and for FP8 with 64 lanes and
// 256 KiB chunks 2 KiB of lane counts per chunk.  4 MiB takes an FP8 tensor of 504 MiB in 256 KiB chunks, 901 MiB
// of FP8 K/V pages of 2 KiB, 1.7 GiB of BF16 pages of 4 KiB, and far more of anything in large chunks.
constexpr uint64_t kScratchBytes = ZC_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// `scratch` above is a host-side stand-in, not an address: each device has its own copy of the array at its own
// address, asked for once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
uint8_t *g_scratch_of[kMaxDevices];

zc_status scratch_of_current_device(uint8_t **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ZC_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_lock);
    if (!g_scratch_of[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZC_ERR_DEVICE;
        g_scratch_of[dev] = (uint8_t *)p;
    }
    *out = g_scratch_of[dev];
    return ZC_OK;
}

// One tensor: its descriptor, the blank header of its container and its work lists as ranges, all passed as
// kernel arguments and written into the workspace by k_setup_single, so that the host copies nothing.
struct SetupList { uint64_t off; uint32_t n, first, step, xcd_order; };
struct SetupArgs {
    TensorDev desc;
    uint8_t header[kHeaderBytes];
    uint64_t off_descs, off_blobs;
    SetupList list[7];
};

// Writes what a compress call's upload would have brought: the tensor's descriptor, its blob (the blank header,
// zeros behind it: k_codes fills in the code-dependent bytes) and the work lists, list l holding the items
// {0, first + step * i} in natural or XCD order.
__global__ __launch_bounds__(256) void k_setup_single(SetupArgs a, uint8_t *ws)
{
    const uint32_t gid = blockIdx.x * 256 + threadIdx.x, stride = gridDim.x * 256;
    if (gid == 0) *reinterpret_cast<TensorDev *>(ws + a.off_descs) = a.desc;
    uint32_t *blob = reinterpret_cast<uint32_t *>(ws + a.off_blobs);
    for (uint32_t i = gid; i < kBlobBytes / 4; i += stride) {
        uint32_t v = 0;
        if (i < kHeaderBytes / 4) v = (uint32_t)a.header[4 * i] | ((uint32_t)a.header[4 * i + 1] << 8) | ((uint32_t)a.header[4 * i + 2] << 16) | ((uint32_t)a.header[4 * i + 3] << 24);
        blob[i] = v;
    }
#pragma unroll 1
    for (int l = 0; l < 7; l++) {
        const SetupList L = a.list[l];
        WorkItem *items = reinterpret_cast<WorkItem *>(ws + L.off);
        for (uint32_t p = gid; p < L.n; p += stride) {
            const uint32_t i = L.xcd_order ? (uint32_t)xcd_order_source(p, L.n) : p;
            items[p] = WorkItem{0u, L.first + L.step * i};
        }
    }
}

int launch_setup_single(const SetupArgs &a, uint8_t *d_ws, void *stream)
{
    uint32_t most = (uint32_t)(kBlobBytes / 4);
    for (int l = 0; l < 7; l++) most = a.list[l].n > most ? a.list[l].n : most;
    uint32_t blocks = (most + 255) / 256;
    if (blocks > 1024) blocks = 1024;                // the kernel strides
    hipLaunchKernelGGL(k_setup_single, dim3(blocks), dim3(256), 0, (hipStream_t)stream, a, d_ws);
    return (int)hipGetLastError();
}

// zc_compress_batch_async for one tensor: codes built on the device, nothing waited for, and nothing copied from
// the host: descriptor, blank header and work lists travel as kernel arguments and k_setup_single writes them where
// an upload would have put them.
zc_status compress_single_device_setup(const zc_tensor &x, const zc_params *params, uint8_t *d_ws, uint64_t ws_bytes, void *stream)
{
    CompressQueue q;
    zc_status st = check_params(params, &q.g);
    if (st) return st;
    const Geometry &g = q.g;
    if (g.host_codes || !d_ws || !aligned16(d_ws)) return ZC_ERR_INVALID_ARG;
    st = check_compress_tensor(g, x, false);
    if (st) return st;
    uint64_t nc;
    st = check_count(g, x.n_elems, &nc);
    if (st) return st;
    st = plan_workspace(g, &x.n_elems, 1, &q.w);
    if (st) return st;
    if (ws_bytes < q.w.total) return ZC_ERR_BUFFER_TOO_SMALL;
    const uint64_t bound = zc_compress_bound(x.n_elems, params);
    if (x.comp_capacity < bound) return ZC_ERR_BUFFER_TOO_SMALL;          // the sizes are not read back before the encoder runs
    q.sh = compress_shape(g, true, nc);
    q.ws = d_ws; q.stream = stream; q.T = 1; q.stats_only = false;
    const bool fs = compress_fast_shape(g, x.n_elems, bound);
    const TensorLists L = device_code_lists(g, q.sh, x.n_elems, nc, fs);
    SetupArgs a;
    std::memset(&a, 0, sizeof(a));
    if (!compress_desc(g, x, nc, 0, false, &a.desc)) return ZC_ERR_BUFFER_TOO_SMALL;
    a.desc.fast_shape = (fs || q.sh.rows8) ? 1 : 0;
    {
        // the header without what depends on the code; k_codes fills that in
        const FieldCode no_code[3] = {};
        zc_info blank;
        uint8_t blob[kBlobBytes];
        fill_info(g, params->policy, x.d_xor_base != nullptr, x.n_elems, nc, no_code, 0, &blank);
        serialize_blob(blank, blob);
        std::memcpy(a.header, blob, kHeaderBytes);           // the rest of a blank blob is zero
    }
    a.off_descs = q.w.descs; a.off_blobs = q.w.blobs;
    q.n_hist = L.hist.count(); q.n_lane_hist = L.lane_hist.count(); q.n_scale = L.scale.count();
    q.n_fast = L.fast.count(); q.n_whole = L.whole.count(); q.n_other = L.other.count(); q.n_slow = L.slow.count();
    // the same places and the same order as CompressCall::run_with_device_codes gives them
    a.list[0] = {q.w.hist_work, q.n_hist, L.hist.first, L.hist.step, 0};
    a.list[1] = {q.w.hist_work + (uint64_t)q.n_hist * sizeof(WorkItem), q.n_lane_hist, L.lane_hist.first, L.lane_hist.step, 1};
    a.list[2] = {q.w.scale_work, q.n_scale, L.scale.first, L.scale.step, 0};
    a.list[3] = {q.w.chunk_work, q.n_slow, L.slow.first, L.slow.step, 1};
    a.list[4] = {q.w.fast_work, q.n_fast, L.fast.first, L.fast.step, 1};
    a.list[5] = {q.w.whole_work, q.n_whole, L.whole.first, L.whole.step, 1};
    a.list[6] = {q.w.other_work, q.n_other, L.other.first, L.other.step, 1};
    LAUNCH_TRY(launch_setup_single(a, d_ws, stream));
    st = q.queue_histogram();
    if (st) return st;
    st = q.queue_codes(params->policy);
    if (st) return st;
    st = q.queue_sizes_and_scan();
    if (st) return st;
    return q.queue_encoders();
}

}  // namespace

}  // namespace zc

extern "C" zc_status zc_compress_noalloc(const void *d_src, uint64_t n_elems, const zc_params *params, const void *d_xor_base,
                                         const void *d_scales, void *d_dst, uint64_t dst_capacity, void *stream)
{
    uint8_t *ws = nullptr;
    const zc_status st = zc::scratch_of_current_device(&ws);
    if (st) return st;
    zc_tensor t = {};
    t.d_src = d_src; t.d_xor_base = d_xor_base; t.d_scales = d_scales; t.n_elems = n_elems;
    t.d_comp = d_dst; t.comp_capacity = dst_capacity;
    return zc::compress_single_device_setup(t, params, ws, zc::kScratchBytes, stream);
}
