// Device and pinned-host scratch of the reduce library: blocks and buffers cached across calls,
// and the bump allocator a call or a session takes its staged programs, tables and scratch from -
// out of those caches, or out of one fixed stretch of device memory when nothing may be allocated.
// Included by hop_api.hip only (the caches are file-scope state of that translation unit).
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/hop.h"

namespace hop {

// ----------------------------------------------------------------------------
// workspace: pinned host staging + device memory, cached across calls
// ----------------------------------------------------------------------------

struct Block {
    int device = -1;
    char *host = nullptr;       // pinned
    char *host_dev = nullptr;   // the pinned memory as the device addresses it
    char *dev = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;    // last use on a stream
    bool pending = false;
};

static std::mutex g_mu;
static std::vector<Block *> g_free;
static constexpr size_t kMinBlock = 256 * 1024;

// Once this many staging blocks exist, a caller that finds a large enough block still in use
// by the GPU waits for the oldest such block instead of allocating another: a host that runs
// ahead of the GPU is slowed down rather than growing the cache without bound. (Blocks held
// by open sessions are not in the cache and are not waited for.)
static constexpr int kMaxBlocks = 8;
static int g_block_count = 0;

static Block *acquire_block(int device, size_t bytes)
{
    Block *wait_for = nullptr, *too_small = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        for (size_t i = 0; i < g_free.size(); ++i) {
            Block *b = g_free[i];
            if (b->device != device || b->cap < bytes) continue;
            if (b->pending) {
                if (hipEventQuery(b->ev) != hipSuccess) {
                    (void)hipGetLastError();
                    if (!wait_for) wait_for = b;          // g_free is in release order: the oldest one
                    continue;
                }
                b->pending = false;
            }
            g_free.erase(g_free.begin() + i);
            return b;
        }
        if (g_block_count >= kMaxBlocks) {
            // at the limit: an idle block that is too small makes room for one of the right size
            // (otherwise callers of the larger size would queue for the few blocks that fit them)
            for (size_t i = 0; i < g_free.size() && !too_small; ++i) {
                Block *b = g_free[i];
                if (b->device != device || b->cap >= bytes) continue;
                if (b->pending && hipEventQuery(b->ev) != hipSuccess) { (void)hipGetLastError(); continue; }
                too_small = b;
                g_free.erase(g_free.begin() + i);
            }
        }
        if (too_small) {
            wait_for = nullptr;                           // its place in the count goes to the new block
        } else if (wait_for && g_block_count >= kMaxBlocks) {
            g_free.erase(std::find(g_free.begin(), g_free.end(), wait_for));
        } else {
            wait_for = nullptr;
            g_block_count++;
        }
    }
    if (too_small) {
        (void)hipEventDestroy(too_small->ev);
        (void)hipFree(too_small->dev);
        (void)hipHostFree(too_small->host);
        delete too_small;
    }
    if (wait_for) {
        if (hipEventSynchronize(wait_for->ev) != hipSuccess) (void)hipGetLastError();
        wait_for->pending = false;
        return wait_for;
    }
    Block *b = new (std::nothrow) Block;
    bool ok = b != nullptr;
    if (ok) {
        b->device = device;
        b->cap = bytes < kMinBlock ? kMinBlock : ((bytes + kMinBlock - 1) / kMinBlock) * kMinBlock;
        ok = hipHostMalloc((void **)&b->host, b->cap, hipHostMallocDefault) == hipSuccess;
        if (ok && hipHostGetDevicePointer((void **)&b->host_dev, b->host, 0) != hipSuccess) { (void)hipHostFree(b->host); ok = false; }
        if (ok && hipMalloc((void **)&b->dev, b->cap) != hipSuccess) { (void)hipHostFree(b->host); ok = false; }
        if (ok && hipEventCreateWithFlags(&b->ev, hipEventDisableTiming) != hipSuccess) {
            (void)hipFree(b->dev); (void)hipHostFree(b->host); ok = false;
        }
    }
    if (!ok) {
        delete b;
        std::lock_guard<std::mutex> lk(g_mu);
        g_block_count--;
        return nullptr;
    }
    return b;
}

// Blocks that a recording of a call takes with it (Workspace::detach) are no longer the pool's: they
// do not count towards kMaxBlocks until they come back, or a process with many recordings would find
// the pool "full" for good and wait for the GPU at every call that stages something.
static void blocks_leave_pool(size_t n)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_block_count -= (int)n;
}
static void blocks_rejoin_pool(size_t n)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_block_count += (int)n;
}

static void release_block(Block *b, hipStream_t stream)
{
    if (!b) return;
    b->pending = (hipEventRecord(b->ev, stream) == hipSuccess);
    std::lock_guard<std::mutex> lk(g_mu);
    g_free.push_back(b);
}

// Large device-only scratch (saved accumulators of eager sessions), cached the same way: a
// buffer goes back to the cache with an event and is handed out again once that event is done.
struct DevBuf {
    int device = -1;
    char *ptr = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};
static std::vector<DevBuf *> g_devbufs;
static constexpr size_t kDevCacheLimit = (size_t)8 << 30;     // beyond this, idle buffers are freed

static DevBuf *acquire_devbuf(int device, size_t bytes)
{
    DevBuf *wait_for = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        DevBuf *best = nullptr;
        int n_busy = 0;
        for (DevBuf *b : g_devbufs) {
            if (b->device != device || b->cap < bytes) continue;
            if (b->pending) {
                if (hipEventQuery(b->ev) != hipSuccess) {
                    (void)hipGetLastError();
                    if (!wait_for) wait_for = b;          // release order: the oldest one
                    ++n_busy;
                    continue;
                }
                b->pending = false;
            }
            if (!best || b->cap < best->cap) best = b;
        }
        if (best) {
            g_devbufs.erase(std::find(g_devbufs.begin(), g_devbufs.end(), best));
            return best;
        }
        // two buffers in flight are enough to overlap one session's tail with the next one's
        // start; beyond that, wait for the oldest instead of growing
        if (wait_for && n_busy >= 2) g_devbufs.erase(std::find(g_devbufs.begin(), g_devbufs.end(), wait_for));
        else wait_for = nullptr;
    }
    if (wait_for) {
        if (hipEventSynchronize(wait_for->ev) != hipSuccess) (void)hipGetLastError();
        wait_for->pending = false;
        return wait_for;
    }
    DevBuf *b = new (std::nothrow) DevBuf;
    if (!b) return nullptr;
    b->device = device;
    b->cap = bytes;
    if (hipMalloc((void **)&b->ptr, bytes) != hipSuccess) { (void)hipGetLastError(); delete b; return nullptr; }
    if (hipEventCreateWithFlags(&b->ev, hipEventDisableTiming) != hipSuccess) { (void)hipFree(b->ptr); delete b; return nullptr; }
    return b;
}

static void release_devbuf(DevBuf *b, hipStream_t stream)
{
    if (!b) return;
    b->pending = (hipEventRecord(b->ev, stream) == hipSuccess);
    std::lock_guard<std::mutex> lk(g_mu);
    g_devbufs.push_back(b);
    size_t total = 0;
    for (DevBuf *x : g_devbufs) total += x->cap;
    for (size_t i = 0; i < g_devbufs.size() && total > kDevCacheLimit;) {
        DevBuf *x = g_devbufs[i];
        if (x->pending && hipEventQuery(x->ev) != hipSuccess) { (void)hipGetLastError(); ++i; continue; }
        total -= x->cap;
        (void)hipEventDestroy(x->ev);
        (void)hipFree(x->ptr);
        delete x;
        g_devbufs.erase(g_devbufs.begin() + i);
    }
}

// Carries up to kPokeVectors * 16 bytes from the kernel arguments to device memory: how programs
// and tables reach the static scratch without a staging buffer.
constexpr int kPokeVectors = 240;
struct PokeArgs {
    uint4 *dst;
    int n;
    int pad;
    uint4 data[kPokeVectors];
};
static_assert(sizeof(PokeArgs) <= 4096, "these argument blocks stay within 4 KiB, which every runtime takes");

__global__ __launch_bounds__(256) void poke_kernel(PokeArgs a)
{
    const int i = (int)threadIdx.x;
    if (i < a.n) a.dst[i] = a.data[i];
}

static bool poke(hipStream_t stream, void *dst, const void *src, size_t bytes)
{
    const char *from = (const char *)src;
    char *to = (char *)dst;
    while (bytes > 0) {
        PokeArgs a;
        const size_t now = bytes < sizeof a.data ? bytes : sizeof a.data;
        a.dst = (uint4 *)to;
        a.n = (int)((now + 15) / 16);
        a.pad = 0;
        std::memset(&a.data[(size_t)a.n - 1], 0, sizeof(uint4));        // the last vector may be partly filled
        std::memcpy(a.data, from, now);
        hipLaunchKernelGGL(poke_kernel, dim3(1), dim3(256), 0, stream, a);
        if (hipGetLastError() != hipSuccess) return false;
        from += now;
        to += now;
        bytes -= now;
    }
    return true;
}

// Copies n_vec 16-byte vectors from pinned host memory (as the device addresses it) to device memory:
// for a few KiB a kernel that reads over the host link starts sooner and costs the host less than a
// copy-engine transfer queued ahead of the kernels that need the data (workload 5's 12 KiB table: the
// call that has to stage it 24 -> 16 us).
__global__ __launch_bounds__(256) void pull_kernel(uint4 *dst, const uint4 *src, size_t n_vec)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}
constexpr size_t kPullMaxBytes = 64 * 1024;

// Bump allocator over a list of blocks; everything staged is copied to the
// device with one copy per stage() call, ordered on the stream.
//
// Static mode (static_base given): every request is served from one caller-given stretch of
// device memory, nothing is allocated, and staged data travels through kernel arguments. A
// request that does not fit fails, and error() then says HOP_ERR_TOO_LARGE.
class Workspace {
public:
    Workspace(int device, hipStream_t stream, char *static_base = nullptr, size_t static_cap = 0)
        : device_(device), stream_(stream), static_base_(static_base), static_cap_(static_base ? static_cap : 0) {}
    Workspace(const Workspace &) = delete;
    Workspace &operator=(const Workspace &) = delete;
    ~Workspace() { for (Block *b : blocks_) release_block(b, stream_); }

    bool is_static() const { return static_base_ != nullptr; }
    // Switches to static mode on the caller's memory; only while nothing has been taken yet.
    bool make_static(char *base, size_t cap)
    {
        if (!blocks_.empty() || is_static() || !base) return false;
        static_base_ = base;
        static_cap_ = cap;
        used_ = 0;
        return true;
    }
    // Hands the blocks over to the caller (who releases them later): what was staged stays valid.
    std::vector<Block *> detach()
    {
        std::vector<Block *> out;
        out.swap(blocks_);
        used_ = 0;
        return out;
    }
    // device bytes of the blocks held
    size_t held_bytes() const
    {
        size_t total = 0;
        for (const Block *b : blocks_) total += b->cap;
        return total;
    }
    // why the last request failed
    int error() const { return capture_denied_ ? HOP_ERR_CAPTURE : too_large_ ? HOP_ERR_TOO_LARGE : HOP_ERR_NOMEM; }
    // Whether the stream is being captured into a graph. Then nothing may come from the cached blocks: they
    // go back to the cache when the call or session ends and are written again by later calls, while a
    // replay of the graph would still copy from them and point its kernels at them.
    bool capturing()
    {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream_, &cap) != hipSuccess) { (void)hipGetLastError(); return false; }
        capture_denied_ = cap != hipStreamCaptureStatusNone;
        return capture_denied_;
    }
    // bytes a request of any kind may still take in static mode
    size_t static_left() const { return static_cap_ - used_; }

    // Copies `bytes` from src to device memory (16-byte aligned); returns the device address or null.
    void *stage(const void *src, size_t bytes)
    {
        size_t need = (bytes + 255) & ~(size_t)255;
        if (is_static()) {
            void *d = scratch(bytes);
            if (d && !poke(stream_, d, src, bytes)) return nullptr;
            return d;
        }
        if (capturing()) return nullptr;
        if (blocks_.empty() || used_ + need > blocks_.back()->cap) {
            Block *b = acquire_block(device_, need);
            if (!b) return nullptr;
            blocks_.push_back(b);
            used_ = 0;
        }
        Block *b = blocks_.back();
        std::memcpy(b->host + used_, src, bytes);
        if (bytes <= kPullMaxBytes) {
            const size_t n_vec = (bytes + 15) / 16;           // requests are rounded up to 256 bytes: the tail is the block's
            hipLaunchKernelGGL(pull_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, stream_, (uint4 *)(b->dev + used_),
                               (const uint4 *)(b->host_dev + used_), n_vec);
            if (hipGetLastError() != hipSuccess) return nullptr;
        } else if (hipMemcpyAsync(b->dev + used_, b->host + used_, bytes, hipMemcpyHostToDevice, stream_) != hipSuccess) {
            return nullptr;
        }
        void *d = b->dev + used_;
        used_ += need;
        return d;
    }

    // Copies `bytes` from src into pinned host memory and returns the address at which kernels
    // read it in place (over the host link): for small tables read once by few workgroups this is
    // cheaper than a copy engine transfer queued ahead of the kernel.
    const void *stage_in_place(const void *src, size_t bytes)
    {
        size_t need = (bytes + 255) & ~(size_t)255;
        if (is_static()) return stage(src, bytes);        // no pinned memory here: a copy on the device
        if (capturing()) return nullptr;
        if (blocks_.empty() || used_ + need > blocks_.back()->cap) {
            Block *b = acquire_block(device_, need);
            if (!b) return nullptr;
            blocks_.push_back(b);
            used_ = 0;
        }
        Block *b = blocks_.back();
        std::memcpy(b->host + used_, src, bytes);
        const void *d = b->host_dev + used_;
        used_ += need;
        return d;
    }

    // Makes sure the next `bytes` of stage()/scratch() requests come from one block.
    bool reserve(size_t bytes)
    {
        if (is_static()) {
            too_large_ = used_ + bytes > static_cap_;
            return !too_large_;
        }
        if (capturing()) return false;
        if (!blocks_.empty() && used_ + bytes <= blocks_.back()->cap) return true;
        Block *b = acquire_block(device_, bytes);
        if (!b) return false;
        blocks_.push_back(b);
        used_ = 0;
        return true;
    }

    // Uninitialised device scratch (256-byte aligned), valid until the workspace is released.
    void *scratch(size_t bytes)
    {
        size_t need = (bytes + 255) & ~(size_t)255;
        if (is_static()) {
            if (need > static_cap_ - used_) { too_large_ = true; return nullptr; }
            void *d = static_base_ + used_;
            used_ += need;
            return d;
        }
        if (capturing()) return nullptr;
        if (blocks_.empty() || used_ + need > blocks_.back()->cap) {
            Block *b = acquire_block(device_, need);
            if (!b) return nullptr;
            blocks_.push_back(b);
            used_ = 0;
        }
        void *d = blocks_.back()->dev + used_;
        used_ += need;
        return d;
    }

private:
    int device_;
    hipStream_t stream_;
    std::vector<Block *> blocks_;
    size_t used_ = 0;
    char *static_base_ = nullptr;
    size_t static_cap_ = 0;
    bool capture_denied_ = false;
    bool too_large_ = false;
};

}  // namespace hop
