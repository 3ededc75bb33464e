// Page-locked host memory of the library: what the host sends to a workspace (descriptors, work lists, tables)
// and what it reads back between kernels (histograms, stream sizes, headers).  A copy to or from pageable
// memory is staged by the runtime in pieces and makes the caller wait; from page-locked memory it is one
// asynchronous transfer.  The buffers are allocated on first use and kept until zc_release_host_buffers() or
// the end of the process.
#include <hip/hip_runtime.h>

#include <mutex>
#include <utility>
#include <vector>

#include "zc_host.h"

namespace zc {

namespace {

// ---- uploads -----------------------------------------------------------------------------------
// A few buffers used in turn: the pieces of an upload are packed into one at their workspace offsets and leave in
// a single asynchronous copy.  A buffer's next user waits for the event of the copy that last left it, so calls
// queued back to back block only when more than kSlots uploads are still ahead of the device.  Every buffer has a
// lock of its own, held while its user waits for that event, fills the buffer and queues the copy: callers on
// other threads wait for each other only when they are dealt the same buffer.
class HostStage {
public:
    zc_status upload(uint8_t *d_ws, uint64_t lo, uint64_t hi, const Piece *pieces, int n, hipStream_t hs)
    {
        if (hi <= lo) return ZC_OK;
        int mine;
        {
            std::lock_guard<std::mutex> deal(m_);
            mine = next_;
            next_ = (next_ + 1) % kSlots;
        }
        Slot &k = slot_[mine];
        std::lock_guard<std::mutex> lock(k.m);
        if (k.pending && hipEventSynchronize(k.ev) != hipSuccess) return ZC_ERR_DEVICE;
        k.pending = false;
        const uint64_t need = hi - lo;
        if (need > k.cap) {
            if (k.buf) (void)hipHostFree(k.buf);
            k.buf = nullptr; k.cap = 0;
            const uint64_t want = need + need / 2 + 4096;
            if (hipHostMalloc((void **)&k.buf, want, hipHostMallocDefault) != hipSuccess) return ZC_ERR_DEVICE;
            k.cap = want;
        }
        if (!k.ev && hipEventCreateWithFlags(&k.ev, hipEventDisableTiming) != hipSuccess) return ZC_ERR_DEVICE;
        for (int i = 0; i < n; i++)
            if (pieces[i].bytes) std::memcpy(k.buf + (pieces[i].off - lo), pieces[i].src, pieces[i].bytes);
        HIP_TRY(hipMemcpyAsync(d_ws + lo, k.buf, need, hipMemcpyHostToDevice, hs));
        HIP_TRY(hipEventRecord(k.ev, hs));
        k.pending = true;
        return ZC_OK;
    }
    // waits for the copies still in flight, then frees every buffer
    zc_status release()
    {
        zc_status st = ZC_OK;
        for (Slot &k : slot_) {
            std::lock_guard<std::mutex> lock(k.m);
            if (k.pending && hipEventSynchronize(k.ev) != hipSuccess) st = ZC_ERR_DEVICE;
            k.pending = false;
            if (k.buf && hipHostFree(k.buf) != hipSuccess) st = ZC_ERR_DEVICE;
            k.buf = nullptr; k.cap = 0;
            if (k.ev) (void)hipEventDestroy(k.ev);
            k.ev = nullptr;
        }
        return st;
    }
private:
    static constexpr int kSlots = 4;
    struct Slot { std::mutex m; uint8_t *buf = nullptr; uint64_t cap = 0; hipEvent_t ev = nullptr; bool pending = false; };
    std::mutex m_;              // guards next_ only
    Slot slot_[kSlots];
    int next_ = 0;
};

HostStage &host_stage() { static HostStage s; return s; }

// ---- read-backs --------------------------------------------------------------------------------
// Buffers are handed out one per call in flight and come back when the call returns.
class HostLanding {
public:
    uint8_t *acquire(uint64_t bytes, uint64_t *cap)
    {
        std::lock_guard<std::mutex> lock(m_);
        for (size_t i = 0; i < free_.size(); i++)
            if (free_[i].second >= bytes) {
                uint8_t *b = free_[i].first; *cap = free_[i].second;
                free_.erase(free_.begin() + (long)i);
                return b;
            }
        if (!free_.empty()) { (void)hipHostFree(free_.back().first); free_.pop_back(); }     // too small: replace it
        uint8_t *b = nullptr;
        const uint64_t want = bytes + bytes / 2 + 4096;
        if (hipHostMalloc((void **)&b, want, hipHostMallocDefault) != hipSuccess) return nullptr;
        *cap = want;
        return b;
    }
    void give_back(uint8_t *b, uint64_t cap)
    {
        std::lock_guard<std::mutex> lock(m_);
        free_.push_back({b, cap});
    }
    // frees the buffers no call holds (a call in flight returns its buffer afterwards, to be freed by the next release)
    zc_status release()
    {
        std::lock_guard<std::mutex> lock(m_);
        zc_status st = ZC_OK;
        for (auto &f : free_) if (hipHostFree(f.first) != hipSuccess) st = ZC_ERR_DEVICE;
        free_.clear();
        return st;
    }
private:
    std::mutex m_;
    std::vector<std::pair<uint8_t *, uint64_t>> free_;
};

HostLanding &host_landing() { static HostLanding s; return s; }

}  // namespace

zc_status stage_upload(uint8_t *d_ws, uint64_t lo, uint64_t hi, const Piece *pieces, int n, void *stream)
{
    return host_stage().upload(d_ws, lo, hi, pieces, n, (hipStream_t)stream);
}

LandingLease::LandingLease(uint64_t bytes) { if (bytes) ptr = host_landing().acquire(bytes, &cap); }
LandingLease::~LandingLease() { if (ptr) host_landing().give_back(ptr, cap); }

}  // namespace zc

extern "C" zc_status zc_release_host_buffers(void)
{
    const zc_status a = zc::host_stage().release(), b = zc::host_landing().release();
    return a ? a : b;
}
