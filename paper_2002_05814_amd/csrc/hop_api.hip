// C ABI of the reduce library (include/hop.h): argument checks, the degree choice and its
// calibration, the static scratch of the entry point that allocates nothing, the recordings of
// repeated small calls, and the entry points themselves. The scheduler is in hop_plan.hpp, the
// back ends that turn its launches into kernel launches in hop_gpu_backend.hpp, the cached
// workspaces in hop_workspace.hpp.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "hop_bcast.hpp"
#include "hop_gpu_backend.hpp"
#include "hop_kernels.h"
#include "hop_plan.hpp"
#include "hop_workspace.hpp"

namespace hop {

// ----------------------------------------------------------------------------
// scratch for callers that cannot allocate (hop_reduce_noalloc)
// ----------------------------------------------------------------------------

// One array per GPU the library runs on, held until the process ends. Host code never uses the
// array's name as an address: static_scratch() asks the runtime where the current device keeps
// its copy, once per device, and everything else (kernel arguments, the bump allocator below)
// works with that pointer.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxStaticDevices = 64;
static char *g_scratch_ptr[kMaxStaticDevices];

static int static_scratch(int device, char **ptr)
{
    if (device < 0 || device >= kMaxStaticDevices) return HOP_ERR_DEVICE;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {     // the current device's copy
            (void)hipGetLastError();
            return HOP_ERR_DEVICE;
        }
        g_scratch_ptr[device] = (char *)p;
    }
    *ptr = g_scratch_ptr[device];
    return HOP_OK;
}

// ----------------------------------------------------------------------------
// argument checks shared by the entry points
// ----------------------------------------------------------------------------

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

static int check_shape(int n, size_t object_bytes, int k, int op, int dtype, size_t chunk_bytes, int tree_degree,
                       Shape *shape)
{
    if (n < 1 || k < 1 || k > n) return HOP_ERR_INVALID;
    if (op < HOP_SUM || op > HOP_MAX || dtype < HOP_F32 || dtype > HOP_I32) return HOP_ERR_INVALID;
    if (chunk_bytes == 0 || chunk_bytes % 16 != 0 || tree_degree < 0) return HOP_ERR_INVALID;
    if (object_bytes % (size_t)elem_bytes(dtype) != 0) return HOP_ERR_INVALID;
    shape->object_bytes = object_bytes;
    shape->chunk_bytes = chunk_bytes;
    shape->n_chunks = object_bytes ? (int64_t)((object_bytes + chunk_bytes - 1) / chunk_bytes) : 1;
    return HOP_OK;
}

static int check_order(int n, const int32_t *ready_order)
{
    if (!ready_order) return HOP_OK;
    std::vector<char> seen(n, 0);
    for (int t = 0; t < n; ++t) {
        int i = ready_order[t];
        if (i < 0 || i >= n || seen[i]) return HOP_ERR_INVALID;
        seen[i] = 1;
    }
    return HOP_OK;
}

static int check_buffers(const void *const *objs, int n, void *const *dsts, int n_dst, size_t object_bytes)
{
    if (!objs || !dsts || n_dst < 1) return HOP_ERR_INVALID;
    for (int j = 0; j < n_dst; ++j) {
        if (!dsts[j]) return HOP_ERR_INVALID;
        if (!aligned16(dsts[j])) return HOP_ERR_ALIGN;
    }
    for (int i = 0; i < n; ++i) {
        if (!objs[i]) return HOP_ERR_INVALID;
        if (!aligned16(objs[i])) return HOP_ERR_ALIGN;
        for (int j = 0; j < n_dst; ++j) {
            const char *a = (const char *)objs[i], *b = (const char *)dsts[j];
            if (object_bytes && a < b + object_bytes && b < a + object_bytes) return HOP_ERR_INVALID;   // result would overwrite a source
        }
    }
    return HOP_OK;
}

// Destinations must not overlap each other (nor be the same buffer twice): sorted by address,
// neighbours suffice.
static int check_disjoint(void *const *dsts, int n_dst, size_t object_bytes)
{
    try {
        std::vector<uintptr_t> at((size_t)n_dst);
        for (int j = 0; j < n_dst; ++j) at[(size_t)j] = (uintptr_t)dsts[j];
        std::sort(at.begin(), at.end());
        for (size_t j = 1; j < at.size(); ++j)
            if (at[j] == at[j - 1] || at[j] - at[j - 1] < object_bytes) return HOP_ERR_INVALID;
        return HOP_OK;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

// The two constants of the cost model of section 3.4.2 (Eq. 1): L, the latency one more tree level
// costs, and B, the bandwidth at which a node takes in an object. The paper's runtime measures both
// (section 4); here calibrate() measures them on the device (what one more dependent launch costs,
// and the rate at which the reduce kernel streams objects in) and keeps them per device. Until a
// device has been calibrated the figures below stand in (typical MI355X values), so that the
// host-only planning calls, which never touch a device, have something to work with.
static const double kDefaultLatency = 3e-6;     // seconds
static const double kDefaultBandwidth = 6.5e12; // bytes per second
constexpr int kMaxCalibratedDevices = 64;
static double g_latency[kMaxCalibratedDevices], g_bandwidth[kMaxCalibratedDevices];     // 0 = not measured
static int g_calibrated_last = -1;              // the device calibrated last: what host-only planning uses

static void model_constants(int device, double *L, double *B)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (device < 0) device = g_calibrated_last;
    const bool have = device >= 0 && device < kMaxCalibratedDevices && g_latency[device] > 0;
    *L = have ? g_latency[device] : kDefaultLatency;
    *B = have ? g_bandwidth[device] : kDefaultBandwidth;
}

// argmin of Eq. 1 over the paper's candidates {1, 2, k} (section 4). Candidates whose predicted
// time lies within 2 % of the best count as equal; among equals the tree with the fewest
// accumulator levels wins (the reduce kernels hold fewer vectors per lane the more levels a tree
// needs), then the smaller degree.
static int pick_degree(int k, size_t object_bytes, double L, double B)
{
    if (k <= 2) return 1;
    if (!(L > 0) || !(B > 0)) {
        double l0, b0;
        model_constants(-1, &l0, &b0);
        if (!(L > 0)) L = l0;
        if (!(B > 0)) B = b0;
    }
    const int cand[3] = {1, 2, k};
    double t[3], best_t = 0;
    for (int i = 0; i < 3; ++i) {
        t[i] = tree_cost(k, cand[i], (double)object_bytes, L, B);
        if (i == 0 || t[i] < best_t) best_t = t[i];
    }
    int best = -1, best_depth = 0;
    for (int i = 0; i < 3; ++i) {
        if (t[i] > best_t * 1.02) continue;
        const int depth = cand[i] == 2 ? full_tree_depth(k, 2) : 1;       // a chain and a star need one level
        if (best < 0 || depth < best_depth) { best = i; best_depth = depth; }
    }
    return cand[best];
}

// Measures L and B on the current device (a few hundred microseconds of GPU time, 320 MiB of scratch
// allocated and freed again) and keeps them for the tree_degree = 0 calls on that device.
static int calibrate(double *latency_s, double *bytes_per_s)
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device >= kMaxCalibratedDevices) return HOP_ERR_DEVICE;
    constexpr size_t kBytes = (size_t)64 << 20;
    constexpr int kSources = 4, kTiny = 32;
    char *buf = nullptr;
    hipStream_t stream = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = HOP_OK;
    double L = 0, B = 0;
    if (hipMalloc((void **)&buf, kBytes * (kSources + 1)) != hipSuccess) { (void)hipGetLastError(); return HOP_ERR_NOMEM; }
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess || hipEventCreate(&e0) != hipSuccess ||
        hipEventCreate(&e1) != hipSuccess)
        rc = HOP_ERR_DEVICE;
    if (rc == HOP_OK && hipMemsetAsync(buf, 0, kBytes * (kSources + 1), stream) != hipSuccess) rc = HOP_ERR_DEVICE;
    if (rc == HOP_OK) {
        DevEntry steps[kSources];
        for (int i = 0; i < kSources; ++i) steps[i] = DevEntry{buf + (size_t)(i + 1) * kBytes, i == 0 ? (1u << 8) : 0u, 0};
        float ms = 0;
        // L: dependent launches of the smallest reduce (one vector), back to back
        for (int pass = 0; pass < 2 && rc == HOP_OK; ++pass) {
            if (hipEventRecord(e0, stream) != hipSuccess) rc = HOP_ERR_DEVICE;
            for (int i = 0; i < kTiny && rc == HOP_OK; ++i)
                if (launch_reduce(stream, HOP_F32, HOP_SUM, 1, steps, nullptr, kSources, buf, 0, 16) != hipSuccess) rc = HOP_ERR_DEVICE;
            if (rc == HOP_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                                 hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
                rc = HOP_ERR_DEVICE;
            L = (double)ms * 1e-3 / kTiny;              // the second pass counts (the first loads the kernel)
        }
        // B: the reduce kernel over four 64 MiB objects, the fastest of three launches
        for (int pass = 0; pass < 4 && rc == HOP_OK; ++pass) {
            if (hipEventRecord(e0, stream) != hipSuccess ||
                launch_reduce(stream, HOP_F32, HOP_SUM, 1, steps, nullptr, kSources, buf, 0, kBytes) != hipSuccess ||
                hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
                rc = HOP_ERR_DEVICE;
            else if (pass > 0 && ms > 0) B = std::max(B, (double)kBytes * (kSources + 1) / ((double)ms * 1e-3));
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (stream) { (void)hipStreamSynchronize(stream); (void)hipStreamDestroy(stream); }
    (void)hipFree(buf);
    if (rc != HOP_OK) { (void)hipGetLastError(); return rc; }
    if (!(L > 0) || !(B > 0)) return HOP_ERR_DEVICE;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_latency[device] = L;
        g_bandwidth[device] = B;
        g_calibrated_last = device;
    }
    if (latency_s) *latency_s = L;
    if (bytes_per_s) *bytes_per_s = B;
    return HOP_OK;
}

// The degree for tree_degree = 0 on the current device: Eq. 1 with that device's measured constants,
// which are taken on the first such call unless the stream is being captured (then, and if the
// measurement fails, with what is there).
static int auto_degree(int device, int k, size_t object_bytes, hipStream_t stream)
{
    bool have;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        have = device >= 0 && device < kMaxCalibratedDevices && g_latency[device] > 0;
    }
    if (!have && k > 2) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) (void)calibrate(nullptr, nullptr);
        else (void)hipGetLastError();
    }
    double L, B;
    model_constants(device, &L, &B);
    return pick_degree(k, object_bytes, L, B);
}

// Launches over more than this many bytes per object (that is, of at least 8 MiB) keep partial results
// while a participant can still fail. Below, keeping costs too much of every launch for what a repair
// would save: the kernel that keeps partials works one step at a time, which is the fast shape only for
// long ranges (12 fp32 inputs, per launch: 3-4 MiB +40 %, 6 MiB +25 %, 8-32 MiB +12-18 %, the extra bytes
// being 15 %).
static constexpr size_t kRetainAboveBytes = ((size_t)8 << 20) - 1;

static void default_retention(Scheduler &s, const Shape &shape, int dtype)
{
    s.set_retention(true, (int64_t)(kRetainAboveBytes / shape.chunk_bytes) + 1, elem_bytes(dtype));
}

// ----------------------------------------------------------------------------
// repeated calls
// ----------------------------------------------------------------------------

// What is remembered from call to call. A failure-free hop_reduce over small inputs is bound by the
// host: checking, planning, cutting the program and building its records take longer than the kernels
// run. Two levels:
//  - Recordings (CachedCall). A caller that repeats a call with the same objects, order and shape (a
//    serving loop) gets the launches of the first call again: they are recorded once, together with the
//    staged programs and the scratch they refer to, and enqueued again with the new destination.
//    Bounded: kMaxCachedCalls recordings holding kMaxCachedScratchTotal bytes of scratch, the least
//    recently used ones make room.
//  - Shapes (CallShape), for the same kind of call over OTHER buffers (a serving loop that gets fresh
//    buffers for every request): what the scheduler and the chain planner made of the shape - the
//    one-launch form of the program but for the objects' addresses - is kept under the key without the
//    addresses. A call that finds it fills in its addresses and launches, planning nothing. Only calls
//    whose whole work was one launch of that form are kept (all-reduces too: the copy follows).
// hop_shutdown frees both.

// The part of a call that decides its schedule: everything but the addresses.
struct CallKey {
    int device = 0, n = 0, k = 0, op = 0, dtype = 0;
    size_t object_bytes = 0, chunk_bytes = 0;
    int64_t degree = 0;
    bool identity_order = true;                  // ready_order was NULL
    std::vector<int32_t> order;
};
// The same of a call in progress (nothing copied).
struct CallView {
    int device, n, k, op, dtype;
    size_t object_bytes, chunk_bytes;
    int64_t degree;
    const int32_t *ready_order;
    const void *const *objs;

    bool scalars_match(const CallKey &c) const
    {
        return c.device == device && c.n == n && c.k == k && c.op == op && c.dtype == dtype && c.object_bytes == object_bytes &&
               c.chunk_bytes == chunk_bytes && c.degree == degree && c.identity_order == (ready_order == nullptr);
    }
    bool order_matches(const CallKey &c) const
    {
        return !ready_order || std::memcmp(c.order.data(), ready_order, sizeof(int32_t) * (size_t)n) == 0;
    }
    CallKey key() const
    {
        CallKey c;
        c.device = device; c.n = n; c.k = k; c.op = op; c.dtype = dtype;
        c.object_bytes = object_bytes; c.chunk_bytes = chunk_bytes; c.degree = degree;
        c.identity_order = ready_order == nullptr;
        if (ready_order) c.order.assign(ready_order, ready_order + n);
        return c;
    }
};

struct CachedCall {
    CallKey key;
    std::vector<const void *> objs;
    std::vector<RecordedLaunch> launches;
    std::vector<Block *> blocks;
    hop_info_t info = {};
    int status = HOP_OK;
    hipStream_t last_stream = nullptr;
    hipEvent_t ev = nullptr;
    bool in_use = false;
    uint64_t stamp = 0;
    size_t held = 0;                    // device bytes of `blocks`
};
struct CallShape {
    CallKey key;
    ChainSkeleton skeleton;
    hop_info_t info = {};
    int status = HOP_OK;
    uint64_t stamp = 0;
};
static std::vector<CachedCall *> g_calls;
static std::vector<std::shared_ptr<CallShape>> g_shapes;
static uint64_t g_call_stamp = 0;
static size_t g_calls_held = 0;                                       // device bytes of the blocks the recordings hold
static constexpr size_t kMaxCachedCalls = 128;          // a serving loop may rotate through many sets of buffers
static constexpr size_t kMaxCachedShapes = 32;
static constexpr size_t kMaxCachedInputBytes = (size_t)64 << 20;      // larger calls are bound by the kernels ...
static constexpr size_t kMaxCachedObjectBytes = (size_t)256 << 10;    // ... unless their objects are small: planning takes about
                                                                      // 20 ns per input, the kernels object_bytes / 6.5 TB/s
static constexpr size_t kMaxCachedScratch = (size_t)32 << 20;         // a recording keeps the scratch its launches use
static constexpr size_t kMaxCachedScratchTotal = (size_t)1 << 30;     // ... all recordings together (device bytes; as many pinned)

static void free_cached_call(CachedCall *c)
{
    blocks_rejoin_pool(c->blocks.size());
    for (Block *b : c->blocks) release_block(b, c->last_stream);
    if (c->ev) (void)hipEventDestroy(c->ev);
    delete c;
}

static bool nobody_fails(const int64_t *fail_mask, int n, int64_t n_chunks)
{
    if (!fail_mask) return true;
    for (int i = 0; i < n; ++i)
        if (fail_mask[i] >= 0 && fail_mask[i] < n_chunks) return false;
    return true;
}

// Whether this call may be remembered at all: failure-free, bound by the host, allowed to allocate, and
// not under graph capture (a recording's hand-over between streams uses an event from outside the capture).
static bool rememberable(int n, int k, size_t object_bytes, const int64_t *fail_mask, int64_t n_chunks, bool no_alloc,
                         hipStream_t stream)
{
    if (no_alloc || object_bytes == 0) return false;
    if (object_bytes > kMaxCachedInputBytes / (size_t)k && object_bytes > kMaxCachedObjectBytes) return false;
    if (!nobody_fails(fail_mask, n, n_chunks)) return false;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cap == hipStreamCaptureStatusNone;
}

// The recording of exactly this call, marked in use (one thread at a time replays a recording), or null.
static CachedCall *take_recording(const CallView &v)
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (CachedCall *c : g_calls) {
        if (c->in_use || !v.scalars_match(c->key)) continue;
        // the objects first: recordings of the same shape over other buffers differ in the first pointer
        if (std::memcmp(c->objs.data(), v.objs, sizeof(void *) * (size_t)v.n) != 0 || !v.order_matches(c->key)) continue;
        c->in_use = true;
        c->stamp = ++g_call_stamp;
        return c;
    }
    return nullptr;
}

// Enqueues a recording's launches again, with this call's destination.
static int replay_recording(CachedCall *hit, const CallView &v, void *const *dsts, int n_dst, hipStream_t stream, hop_info_t *info)
{
    // the objects and the order were checked when the call was recorded; the destination is new
    int rc = check_buffers(v.objs, v.n, dsts, n_dst, v.object_bytes);
    if (rc >= 0 && hit->last_stream != stream) {
        // the recording's scratch is shared by its uses: a use on another stream follows the last one
        if (!hit->ev && hipEventCreateWithFlags(&hit->ev, hipEventDisableTiming) != hipSuccess) rc = HOP_ERR_DEVICE;
        if (rc >= 0 && hipEventRecord(hit->ev, hit->last_stream) == hipSuccess) {
            if (hipStreamWaitEvent(stream, hit->ev, 0) != hipSuccess) rc = HOP_ERR_DEVICE;
        } else {
            (void)hipGetLastError();        // the stream of the last use is gone: its work is done
        }
    }
    for (size_t i = 0; rc >= 0 && i < hit->launches.size(); ++i)
        if (replay_launch(hit->launches[i], stream, dsts[0]) != hipSuccess) rc = HOP_ERR_DEVICE;
    if (rc >= 0) {
        hit->last_stream = stream;
        if (info) *info = hit->info;
        rc = hit->status;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    hit->in_use = false;
    return rc;
}

// Keeps what a call's launches need to be enqueued again; the least recently used recordings make room,
// for the new one and for what it holds.
static void remember_recording(const CallView &v, LaunchRecorder &rec, GpuBackend &be, const hop_info_t &info, int status,
                               hipStream_t stream)
{
    CachedCall *c = new CachedCall;
    c->key = v.key();
    c->objs.assign(v.objs, v.objs + v.n);
    c->launches.swap(rec.launches);
    c->held = be.held_bytes();
    c->blocks = be.detach_blocks();
    blocks_leave_pool(c->blocks.size());
    c->info = info;
    c->status = status;
    c->last_stream = stream;
    std::vector<CachedCall *> victims;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        c->stamp = ++g_call_stamp;
        g_calls.push_back(c);
        g_calls_held += c->held;
        while (g_calls.size() > kMaxCachedCalls || g_calls_held > kMaxCachedScratchTotal) {
            size_t at = g_calls.size();
            for (size_t i = 0; i < g_calls.size(); ++i)
                if (!g_calls[i]->in_use && g_calls[i] != c && (at == g_calls.size() || g_calls[i]->stamp < g_calls[at]->stamp)) at = i;
            if (at == g_calls.size()) break;
            victims.push_back(g_calls[at]);
            g_calls_held -= g_calls[at]->held;
            g_calls.erase(g_calls.begin() + (long)at);
        }
    }
    for (CachedCall *victim : victims) free_cached_call(victim);
}

static std::shared_ptr<CallShape> find_shape(const CallView &v)
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (const std::shared_ptr<CallShape> &c : g_shapes)
        if (v.scalars_match(c->key) && v.order_matches(c->key)) {
            c->stamp = ++g_call_stamp;
            return c;
        }
    return nullptr;
}

static void remember_shape(const CallView &v, const ChainSkeleton &sk, const hop_info_t &info, int status)
{
    auto c = std::make_shared<CallShape>();
    c->key = v.key();
    c->skeleton = sk;
    c->info = info;
    c->status = status;
    std::lock_guard<std::mutex> lk(g_mu);
    c->stamp = ++g_call_stamp;
    g_shapes.push_back(c);
    if (g_shapes.size() > kMaxCachedShapes) {
        size_t at = 0;
        for (size_t i = 1; i < g_shapes.size(); ++i)
            if (g_shapes[i]->stamp < g_shapes[at]->stamp) at = i;
        g_shapes.erase(g_shapes.begin() + (long)at);
    }
}

static int reduce_common(void *const *dsts, int n_dst, const void *const *objs, int n, size_t object_bytes,
                         const int32_t *ready_order, int k, int op, int dtype, size_t chunk_bytes,
                         int tree_degree, const int64_t *fail_mask, void *stream_, hop_info_t *info,
                         bool no_alloc = false)
{
    const hipStream_t stream = (hipStream_t)stream_;
    Shape shape;
    int rc = check_shape(n, object_bytes, k, op, dtype, chunk_bytes, tree_degree, &shape);
    if (rc < 0) return rc;
    if (!objs || !dsts) return HOP_ERR_INVALID;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return HOP_ERR_DEVICE;
    const int64_t d = tree_degree > 0 ? tree_degree : auto_degree(device, k, object_bytes, stream);
    const CallView view{device, n, k, op, dtype, object_bytes, chunk_bytes, d, ready_order, objs};
    const bool shapeable = rememberable(n, k, object_bytes, fail_mask, shape.n_chunks, no_alloc, stream);
    const bool cacheable = shapeable && n_dst == 1;       // recordings hold reduce launches only; shapes serve all-reduces too
    if (cacheable)
        if (CachedCall *hit = take_recording(view)) return replay_recording(hit, view, dsts, n_dst, stream, info);
    const std::shared_ptr<CallShape> known = shapeable ? find_shape(view) : nullptr;
    if (!known && (rc = check_order(n, ready_order)) < 0) return rc;      // a known shape's order was checked before
    if ((rc = check_buffers(objs, n, dsts, n_dst, object_bytes)) < 0) return rc;
    char *static_base = nullptr;
    if (no_alloc && (rc = static_scratch(device, &static_base)) < 0) return rc;
    try {
        GpuBackend be(device, stream, objs, n, std::vector<void *>(dsts, dsts + n_dst), shape, op, dtype, k, d, static_base,
                      kStaticScratchBytes);
        LaunchRecorder rec;
        hop_info_t my_info = {};
        bool planned = true;
        if (known) {
            // the shape's one launch with this call's addresses; anything in the way (an address that cannot be
            // told from an offset, no room) sends the call down the whole path
            if (cacheable) set_launch_recorder(&rec);
            rc = be.launch_skeleton(known->skeleton, 0, object_bytes);
            set_launch_recorder(nullptr);
            if (rc == HOP_OK && n_dst > 1 && (rc = be.copy_rest(0, object_bytes)) < 0) return rc;
            if (rc == HOP_OK) {
                planned = false;
                my_info = known->info;
                rc = known->status;
            } else if (rc < 0 && rc != HOP_ERR_INVALID) {
                return rc;
            } else {
                rec = LaunchRecorder();
            }
        }
        if (planned) {
            Scheduler s(n, k, shape.n_chunks, d, &be);
            default_retention(s, shape, dtype);
            if (cacheable) set_launch_recorder(&rec);
            rc = replay_reduce(s, n, shape.n_chunks, ready_order, fail_mask, &my_info);
            set_launch_recorder(nullptr);
            if (shapeable && !known && rc >= 0)
                if (const ChainSkeleton *sk = be.sole_skeleton(my_info.n_launches)) remember_shape(view, *sk, my_info, rc);
        }
        if (info) *info = my_info;
        if (cacheable && rc >= 0 && !rec.unusable && !rec.launches.empty() && be.held_bytes() <= kMaxCachedScratch)
            remember_recording(view, rec, be, my_info, rc, stream);
        return rc;
    } catch (const std::bad_alloc &) {
        set_launch_recorder(nullptr);
        return HOP_ERR_NOMEM;
    }
}

}  // namespace hop

// ----------------------------------------------------------------------------
// C ABI
// ----------------------------------------------------------------------------

using namespace hop;

// Broadcast back ends: enqueue 1-to-1 chunk-range copies, or only record them.
class GpuBcastBackend : public BcastBackend {
public:
    GpuBcastBackend(hipStream_t stream, const Shape &shape) : stream_(stream), shape_(shape) {}
    std::vector<void *> ptrs;                    // device address of every copy, by copy id
    std::vector<hop_bcast_copy_t> log;
    int copy(int from, int to, int64_t c0, int64_t c1) override
    {
        log.push_back({from, to, c0, c1});
        hipError_t e = launch_copy(stream_, ptrs[(size_t)from], nullptr, 1, shape_.begin(c0), shape_.end(c1),
                                   ptrs[(size_t)to]);
        return e == hipSuccess ? HOP_OK : HOP_ERR_DEVICE;
    }

private:
    hipStream_t stream_;
    Shape shape_;
};

class RecordingBcastBackend : public BcastBackend {
public:
    std::vector<hop_bcast_copy_t> log;
    int copy(int from, int to, int64_t c0, int64_t c1) override
    {
        log.push_back({from, to, c0, c1});
        return HOP_OK;
    }
};

struct hop_bcast {
    std::unique_ptr<GpuBcastBackend> gpu;
    std::unique_ptr<RecordingBcastBackend> rec;
    std::unique_ptr<BcastScheduler> sched;
    size_t object_bytes = 0;
    std::vector<hop_bcast_copy_t> &log() { return gpu ? gpu->log : rec->log; }
};

struct hop_session {
    std::unique_ptr<GpuBackend> be;             // sessions that enqueue work
    std::unique_ptr<RecordingBackend> rec;      // host-only sessions (hop_plan_session_begin)
    std::unique_ptr<Scheduler> sched;
    size_t chunk_bytes = 16;
    int dtype = HOP_F32;
};

static void copy_record(const RecordingBackend &be, hop_plan_launch_t *launches, int launch_capacity, int *n_launches,
                        hop_plan_entry_t *entries, int entry_capacity, int *n_entries)
{
    if (n_launches) *n_launches = (int)be.launches.size();
    if (n_entries) *n_entries = (int)be.entries.size();
    for (int i = 0; launches && i < launch_capacity && i < (int)be.launches.size(); ++i) launches[i] = be.launches[i];
    for (int i = 0; entries && i < entry_capacity && i < (int)be.entries.size(); ++i) {
        entries[i].obj = be.entries[i].obj;
        entries[i].level = be.entries[i].level;
        entries[i].set = be.entries[i].set;
        entries[i].n_fold = be.entries[i].n_fold;
        entries[i].save = be.entries[i].save;
        entries[i].save_level = be.entries[i].save_level;
        entries[i].reserved = 0;
    }
}


extern "C" {

int hop_reduce(void *dst, const void *const *objs, int n, size_t object_bytes, const int32_t *ready_order,
               int k, hop_op_t op, hop_dtype_t dtype, size_t chunk_bytes, int tree_degree,
               const int64_t *fail_mask, void *stream, hop_info_t *info)
{
    if (!dst) return HOP_ERR_INVALID;
    void *dsts[1] = {dst};
    return reduce_common(dsts, 1, objs, n, object_bytes, ready_order, k, (int)op, (int)dtype, chunk_bytes,
                         tree_degree, fail_mask, stream, info);
}

int hop_reduce_noalloc(void *dst, const void *const *objs, int n, size_t object_bytes, const int32_t *ready_order,
                       int k, hop_op_t op, hop_dtype_t dtype, size_t chunk_bytes, int tree_degree,
                       const int64_t *fail_mask, void *stream, hop_info_t *info)
{
    if (!dst) return HOP_ERR_INVALID;
    void *dsts[1] = {dst};
    return reduce_common(dsts, 1, objs, n, object_bytes, ready_order, k, (int)op, (int)dtype, chunk_bytes,
                         tree_degree, fail_mask, stream, info, true);
}

size_t hop_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int hop_allreduce(void *const *dsts, int n_dst, const void *const *objs, int n, size_t object_bytes,
                  const int32_t *ready_order, int k, hop_op_t op, hop_dtype_t dtype, size_t chunk_bytes,
                  int tree_degree, const int64_t *fail_mask, void *stream, hop_info_t *info)
{
    if (!dsts || n_dst < 1) return HOP_ERR_INVALID;
    int rc = check_disjoint(dsts, n_dst, object_bytes);
    if (rc < 0) return rc;
    return reduce_common(dsts, n_dst, objs, n, object_bytes, ready_order, k, (int)op, (int)dtype, chunk_bytes,
                         tree_degree, fail_mask, stream, info);
}

int hop_broadcast(void *const *dsts, int n_dst, const void *src, size_t object_bytes, size_t chunk_bytes,
                  void *stream)
{
    if (n_dst < 0 || (n_dst > 0 && !dsts) || chunk_bytes == 0 || chunk_bytes % 16 != 0) return HOP_ERR_INVALID;
    if (n_dst == 0 || object_bytes == 0) return HOP_OK;
    if (!src) return HOP_ERR_INVALID;
    if (!aligned16(src)) return HOP_ERR_ALIGN;
    for (int j = 0; j < n_dst; ++j) {
        if (!dsts[j]) return HOP_ERR_INVALID;
        if (!aligned16(dsts[j])) return HOP_ERR_ALIGN;
        const char *a = (const char *)src, *b = (const char *)dsts[j];
        if (a < b + object_bytes && b < a + object_bytes) return HOP_ERR_INVALID;
    }
    {
        int rc = check_disjoint(dsts, n_dst, object_bytes);
        if (rc < 0) return rc;
    }
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return HOP_ERR_DEVICE;
    try {
        // The whole source is present, so every chunk is ready at once: one launch covers them all. Up to
        // kInlineDsts destinations ride in the kernel arguments, a longer table is staged in device memory.
        Workspace ws(device, (hipStream_t)stream);
        void *const *table = nullptr;
        if (n_dst > kInlineDsts) {
            table = (void *const *)ws.stage(dsts, (size_t)n_dst * sizeof(void *));
            if (!table) return HOP_ERR_NOMEM;
        }
        hipError_t e = launch_copy((hipStream_t)stream, src, table, n_dst, 0, object_bytes, nullptr, common_residue(dsts, n_dst), dsts);
        return e == hipSuccess ? HOP_OK : HOP_ERR_DEVICE;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_bcast_begin(hop_bcast_t **b, const void *src, size_t object_bytes, size_t chunk_bytes, void *stream)
{
    if (!b || chunk_bytes == 0 || chunk_bytes % 16 != 0) return HOP_ERR_INVALID;
    *b = nullptr;
    if (src && !aligned16(src)) return HOP_ERR_ALIGN;
    Shape shape;
    shape.object_bytes = object_bytes;
    shape.chunk_bytes = chunk_bytes;
    shape.n_chunks = object_bytes ? (int64_t)((object_bytes + chunk_bytes - 1) / chunk_bytes) : 1;
    try {
        std::unique_ptr<hop_bcast> h(new hop_bcast);
        h->object_bytes = object_bytes;
        BcastBackend *be;
        if (src) {
            h->gpu.reset(new GpuBcastBackend((hipStream_t)stream, shape));
            h->gpu->ptrs.push_back(const_cast<void *>(src));
            be = h->gpu.get();
        } else {
            h->rec.reset(new RecordingBcastBackend);
            be = h->rec.get();
        }
        h->sched.reset(new BcastScheduler(shape.n_chunks, be));
        *b = h.release();
        return HOP_OK;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_bcast_source_ready(hop_bcast_t *b, int64_t chunks_ready_total)
{
    if (!b) return HOP_ERR_INVALID;
    return b->sched->source_ready(chunks_ready_total);
}

int hop_bcast_join(hop_bcast_t *b, void *dst, int *sender)
{
    if (!b) return HOP_ERR_INVALID;
    try {
        if (b->gpu) {
            if (!dst) return HOP_ERR_INVALID;
            if (!aligned16(dst)) return HOP_ERR_ALIGN;
            for (void *p : b->gpu->ptrs) {
                const char *x = (const char *)p, *y = (const char *)dst;
                if (b->object_bytes && x < y + b->object_bytes && y < x + b->object_bytes) return HOP_ERR_INVALID;
            }
            b->gpu->ptrs.push_back(dst);
        }
        return b->sched->join(sender);
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_bcast_fail(hop_bcast_t *b, int copy)
{
    if (!b) return HOP_ERR_INVALID;
    return b->sched->fail(copy);
}

int hop_bcast_step(hop_bcast_t *b, int64_t max_chunks)
{
    if (!b || max_chunks < 0) return HOP_ERR_INVALID;
    try {
        return b->sched->step(max_chunks);
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_bcast_sender(hop_bcast_t *b, int copy)
{
    if (!b || copy < 0 || copy >= b->sched->n_copies()) return HOP_ERR_INVALID;
    return b->sched->sender_of(copy);
}

int hop_bcast_finish(hop_bcast_t *b, hop_bcast_info_t *info, hop_bcast_copy_t *log, int log_capacity, int *n_log)
{
    if (!b) return HOP_ERR_INVALID;
    int rc;
    try {
        rc = b->sched->drain();
        if (rc >= 0) rc = b->sched->all_complete() ? HOP_OK : HOP_PARTIAL;
        if (info) {
            info->n_receivers = b->sched->n_copies() - 1;
            info->n_failed = b->sched->n_failed();
            info->n_resumed = b->sched->n_resumed();
            info->n_complete = 0;
            for (int id = 1; id < b->sched->n_copies(); ++id)
                info->n_complete += !b->sched->failed(id) && b->sched->complete(id);
            info->chunks_copied = b->sched->chunks_copied();
        }
        std::vector<hop_bcast_copy_t> &l = b->log();
        if (n_log) *n_log = (int)l.size();
        for (int i = 0; log && i < log_capacity && i < (int)l.size(); ++i) log[i] = l[(size_t)i];
    } catch (const std::bad_alloc &) {
        rc = HOP_ERR_NOMEM;
    }
    delete b;
    return rc;
}

int hop_session_begin(hop_session_t **s, void *dst, const void *const *objs, int n, size_t object_bytes, int k,
                      hop_op_t op, hop_dtype_t dtype, size_t chunk_bytes, int tree_degree, void *stream)
{
    if (!s || !dst) return HOP_ERR_INVALID;
    *s = nullptr;
    Shape shape;
    int rc = check_shape(n, object_bytes, k, (int)op, (int)dtype, chunk_bytes, tree_degree, &shape);
    if (rc < 0) return rc;
    void *dsts[1] = {dst};
    if ((rc = check_buffers(objs, n, dsts, 1, object_bytes)) < 0) return rc;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return HOP_ERR_DEVICE;
    const int64_t d = tree_degree > 0 ? tree_degree : auto_degree(device, k, object_bytes, (hipStream_t)stream);
    try {
        std::unique_ptr<hop_session> h(new hop_session);
        h->be.reset(new GpuBackend(device, (hipStream_t)stream, objs, n, std::vector<void *>(1, dst), shape,
                                   (int)op, (int)dtype, k, d));
        h->sched.reset(new Scheduler(n, k, shape.n_chunks, d, h->be.get()));
        default_retention(*h->sched, shape, (int)dtype);
        h->chunk_bytes = chunk_bytes;
        h->dtype = (int)dtype;
        *s = h.release();
        return HOP_OK;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_session_ready(hop_session_t *s, int obj, int64_t chunks_ready_total)
{
    if (!s) return HOP_ERR_INVALID;
    try {
        int rc = s->sched->on_ready(obj, chunks_ready_total);
        return rc < 0 ? rc : s->sched->pump();
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_session_ready_after(hop_session_t *s, int obj, int64_t chunks_ready_total, void *event)
{
    if (!s) return HOP_ERR_INVALID;
    // the wait is enqueued at once, ahead of whatever this or a later notification launches
    if (event && s->be && !s->be->wait_for((hipEvent_t)event)) return HOP_ERR_DEVICE;
    return hop_session_ready(s, obj, chunks_ready_total);
}

int hop_session_fail(hop_session_t *s, int obj)
{
    if (!s) return HOP_ERR_INVALID;
    try {
        int rc = s->sched->on_fail(obj);
        return rc < 0 ? rc : s->sched->pump();
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_session_finish(hop_session_t *s, hop_info_t *info)
{
    if (!s) return HOP_ERR_INVALID;
    int rc;
    try {
        rc = s->sched->finish(info);
    } catch (const std::bad_alloc &) {
        rc = HOP_ERR_NOMEM;
    }
    delete s;
    return rc;
}

int hop_session_set_eager(hop_session_t *s, int min_steps)
{
    if (!s || min_steps < 0) return HOP_ERR_INVALID;
    s->sched->set_eager(min_steps);
    return HOP_OK;
}

int hop_session_set_workspace(hop_session_t *s, void *device_memory, size_t bytes)
{
    if (!s || !device_memory || bytes < 256) return HOP_ERR_INVALID;
    if (((uintptr_t)device_memory & 255u) != 0) return HOP_ERR_ALIGN;
    if (!s->be) return HOP_OK;                       // host-only sessions have no scratch
    return s->be->use_workspace(device_memory, bytes) ? HOP_OK : HOP_ERR_INVALID;
}

int hop_session_set_retention(hop_session_t *s, int on)
{
    if (!s) return HOP_ERR_INVALID;
    s->sched->set_retention(on != 0, (int64_t)(kRetainAboveBytes / s->chunk_bytes) + 1, elem_bytes(s->dtype));
    return HOP_OK;
}

int hop_session_set_adaptive(hop_session_t *s, int on)
{
    if (!s) return HOP_ERR_INVALID;
    s->sched->set_adaptive(on != 0);
    if (on && s->be) s->be->track_idle();
    return HOP_OK;
}

int64_t hop_session_chunks_final(hop_session_t *s)
{
    if (!s) return HOP_ERR_INVALID;
    return s->sched->chunks_final();
}

int hop_plan_session_begin(hop_session_t **s, int n, size_t object_bytes, int k, hop_dtype_t dtype,
                           size_t chunk_bytes, int tree_degree)
{
    if (!s) return HOP_ERR_INVALID;
    *s = nullptr;
    Shape shape;
    int rc = check_shape(n, object_bytes, k, HOP_SUM, (int)dtype, chunk_bytes, tree_degree, &shape);
    if (rc < 0) return rc;
    const int64_t d = tree_degree > 0 ? tree_degree : pick_degree(k, object_bytes, 0, 0);
    try {
        std::unique_ptr<hop_session> h(new hop_session);
        h->rec.reset(new RecordingBackend);
        h->sched.reset(new Scheduler(n, k, shape.n_chunks, d, h->rec.get()));
        default_retention(*h->sched, shape, (int)dtype);
        h->chunk_bytes = chunk_bytes;
        h->dtype = (int)dtype;
        *s = h.release();
        return HOP_OK;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_plan_session_finish(hop_session_t *s, hop_info_t *info, hop_plan_launch_t *launches, int launch_capacity,
                            int *n_launches, hop_plan_entry_t *entries, int entry_capacity, int *n_entries)
{
    if (!s || !s->rec) return HOP_ERR_INVALID;
    int rc;
    try {
        rc = s->sched->finish(info);
        copy_record(*s->rec, launches, launch_capacity, n_launches, entries, entry_capacity, n_entries);
    } catch (const std::bad_alloc &) {
        rc = HOP_ERR_NOMEM;
    }
    delete s;
    return rc;
}

int hop_plan_reduce(int n, size_t object_bytes, const int32_t *ready_order, int k, hop_dtype_t dtype,
                    size_t chunk_bytes, int tree_degree, const int64_t *fail_mask, hop_info_t *info,
                    hop_plan_launch_t *launches, int launch_capacity, int *n_launches,
                    hop_plan_entry_t *entries, int entry_capacity, int *n_entries)
{
    Shape shape;
    int rc = check_shape(n, object_bytes, k, HOP_SUM, (int)dtype, chunk_bytes, tree_degree, &shape);
    if (rc < 0) return rc;
    if ((rc = check_order(n, ready_order)) < 0) return rc;
    const int64_t d = tree_degree > 0 ? tree_degree : pick_degree(k, object_bytes, 0, 0);
    try {
        RecordingBackend be;
        Scheduler s(n, k, shape.n_chunks, d, &be);
        default_retention(s, shape, (int)dtype);
        rc = replay_reduce(s, n, shape.n_chunks, ready_order, fail_mask, info);
        copy_record(be, launches, launch_capacity, n_launches, entries, entry_capacity, n_entries);
        return rc;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_plan_split(const hop_plan_entry_t *entries, int n_entries, int want_steps, int min_run, int max_run,
                   hop_plan_entry_t *top, int top_capacity, int *n_top,
                   hop_plan_entry_t *sub_entries, int sub_capacity, int *n_sub_entries,
                   int32_t *sub_begin, int32_t *sub_pass, int sub_table_capacity, int *n_subs, int *n_passes)
{
    if (!entries || n_entries < 0 || min_run < 1 || max_run < min_run || want_steps < 0) return HOP_ERR_INVALID;
    try {
        std::vector<Entry> prog(n_entries);
        for (int i = 0; i < n_entries; ++i) prog[i] = {entries[i].obj, entries[i].level, entries[i].set, entries[i].n_fold};
        MultiPlan mp;
        const bool ok = plan_passes(prog, (size_t)want_steps, min_run, max_run, mp);
        const std::vector<Entry> &flat = mp.steps;
        std::vector<int32_t> begins(mp.begin);
        if (begins.empty()) begins.push_back(0);
        if (n_top) *n_top = (int)mp.top.size();
        if (n_sub_entries) *n_sub_entries = (int)flat.size();
        if (n_subs) *n_subs = (int)mp.n_subs();
        if (n_passes) *n_passes = mp.n_passes;
        auto put = [](hop_plan_entry_t *dst, int cap, const std::vector<Entry> &src) {
            for (int i = 0; dst && i < cap && i < (int)src.size(); ++i) {
                dst[i].obj = src[i].obj; dst[i].level = src[i].level; dst[i].set = src[i].set; dst[i].n_fold = src[i].n_fold;
            }
        };
        put(top, top_capacity, mp.top);
        put(sub_entries, sub_capacity, flat);
        for (int i = 0; sub_begin && i < sub_table_capacity && i < (int)begins.size(); ++i) sub_begin[i] = begins[i];
        for (int i = 0; sub_pass && i < sub_table_capacity && i < (int)mp.n_subs(); ++i) sub_pass[i] = mp.height[(size_t)i];
        return ok ? HOP_OK : HOP_PARTIAL;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_plan_chains(const hop_plan_entry_t *entries, int n_entries, int min_cut, int max_items,
                    int32_t *items, int item_capacity, int *n_items,
                    int32_t *chain_begin, int32_t *chain_pass, int table_capacity, int *n_chains, int *n_passes)
{
    if (!entries || n_entries < 0 || min_cut < 1 || max_items < 2) return HOP_ERR_INVALID;
    try {
        std::vector<Entry> prog(n_entries);
        for (int i = 0; i < n_entries; ++i) {
            prog[i] = {entries[i].obj, entries[i].level, entries[i].set, entries[i].n_fold};
            prog[i].save = entries[i].save;
        }
        ChainPlan cp;
        const bool ok = plan_chains(prog, min_cut, max_items, cp);
        if (n_items) *n_items = (int)cp.items.size();
        if (n_chains) *n_chains = (int)cp.n_chains();
        if (n_passes) *n_passes = cp.n_passes;
        for (int i = 0; items && i < item_capacity && i < (int)cp.items.size(); ++i) items[i] = cp.items[(size_t)i];
        for (int i = 0; chain_begin && i < table_capacity && i < (int)cp.begin.size(); ++i) chain_begin[i] = cp.begin[(size_t)i];
        for (int i = 0; chain_pass && i < table_capacity && i < (int)cp.n_chains(); ++i) chain_pass[i] = cp.pass[(size_t)i];
        return ok ? HOP_OK : HOP_PARTIAL;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_plan_slots(int k, int tree_degree, int32_t *node_of_slot)
{
    if (k < 1 || tree_degree < 1 || !node_of_slot) return HOP_ERR_INVALID;
    try {
        Tree t;
        t.build(k, tree_degree);
        std::memcpy(node_of_slot, t.node_of_slot.data(), sizeof(int32_t) * (size_t)k);
        return HOP_OK;
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

int hop_pick_degree(int k, size_t object_bytes, double latency_s, double bytes_per_s)
{
    if (k < 1) return HOP_ERR_INVALID;
    return pick_degree(k, object_bytes, latency_s, bytes_per_s);
}

int hop_calibrate(double *latency_s, double *bytes_per_s)
{
    try {
        return calibrate(latency_s, bytes_per_s);
    } catch (const std::bad_alloc &) {
        return HOP_ERR_NOMEM;
    }
}

size_t hop_workspace_bytes(int n, int k, size_t object_bytes, size_t chunk_bytes, int tree_degree, hop_dtype_t dtype,
                           int n_dst, int policy)
{
    Shape shape;
    if (n_dst < 0 || check_shape(n, object_bytes, k, HOP_SUM, (int)dtype, chunk_bytes, tree_degree, &shape) < 0) return 0;
    try {
        const int64_t d = tree_degree > 0 ? tree_degree : pick_degree(k, object_bytes, 0, 0);
        auto blocks = [](size_t bytes) { return bytes == 0 ? (size_t)0 : ((bytes + kMinBlock - 1) / kMinBlock) * kMinBlock; };
        auto round256 = [](size_t bytes) { return (bytes + 255) & ~(size_t)255; };
        const size_t n_elems = object_bytes / (size_t)elem_bytes((int)dtype);
        // staged program (longer than the kernel arguments hold) and destination table
        size_t staged = 0;
        if (k > kInlineEntries) staged += round256((size_t)k * sizeof(DevEntry));
        if (n_dst - 1 > kInlineDsts) staged += round256((size_t)(n_dst - 1) * sizeof(void *));
        size_t total = blocks(staged);
        // the cut into sub-programs of a call over many small objects: their partial results and records
        // the program as chains in one launch: a table of one record per chain (fewer chains than inputs)
        if ((size_t)k >= kChainWantSteps && object_bytes > 0 && std::min(object_bytes, shape.chunk_bytes) <= kChainWideMaxBytes)
            total += blocks(round256((size_t)k * kChainRecordWords * sizeof(uint64_t)));
        if ((size_t)k >= kSplitWantSteps && object_bytes > 0 && std::min(object_bytes, shape.chunk_bytes) <= split_max_bytes((int)dtype)) {
            Tree tr;
            tr.shape(k, d);
            std::vector<int32_t> occ((size_t)k, 0);
            std::vector<Entry> prog;
            compile_program(tr, occ, prog);
            MultiPlan mp;
            if (plan_passes(prog, kSplitWantSteps, kSplitMinRun, kSplitMaxRun, mp)) {
                // bf16: 4-byte accumulators in whole blocks of 1 KiB of the object, wherever the range starts
                const size_t longest = std::min(object_bytes, split_max_bytes((int)dtype));
                const size_t partials = (dtype == HOP_BF16 ? ((longest + 1023) / 1024 + 1) * 2048 : round256(longest)) * mp.n_subs();
                if (partials <= kSplitMaxScratch)
                    total = std::max(total, blocks(partials + (mp.steps.size() + mp.n_subs() * 2 + mp.top.size()) * sizeof(DevEntry) + 512));
            }
        }
        const size_t level_stride = round256(n_elems * 4);
        if (policy & HOP_WS_EAGER) {
            // saved accumulators: one array of 4-byte values per level the tree can need, plus one staged program
            // segment per launch (at most k steps each, one 256 KiB block at a time)
            total += level_stride * (size_t)std::min(HOP_MAX_DEPTH, std::max(1, full_tree_depth(k, d)));
            total += blocks(round256((size_t)k * sizeof(DevEntry)));
        }
        if ((policy & HOP_WS_FAILURES) && object_bytes > kRetainAboveBytes) {
            const size_t runs = kept_subtrees(k, d, elem_bytes((int)dtype), kMaxKept).size();
            const size_t kept_stride = (((object_bytes + 15) / 16 + 63) / 64) * 1024 * (size_t)(4 / elem_bytes((int)dtype));
            if (runs > 0 && kept_stride <= ((size_t)16 << 30) / runs) total += kept_stride * runs;
        }
        return total;
    } catch (const std::bad_alloc &) {
        return 0;
    }
}

int hop_shutdown(void)
{
    {
        // recorded calls first: their blocks go back to the cache that is emptied below
        std::vector<CachedCall *> calls;
        {
            std::lock_guard<std::mutex> lk(g_mu);
            calls.swap(g_calls);
            g_calls_held = 0;
            g_shapes.clear();
        }
        for (CachedCall *c : calls) free_cached_call(c);
    }
    std::lock_guard<std::mutex> lk(g_mu);
    int rc = HOP_OK;
    for (Block *b : g_free) {
        if (b->pending && hipEventSynchronize(b->ev) != hipSuccess) rc = HOP_ERR_DEVICE;
        (void)hipEventDestroy(b->ev);
        (void)hipFree(b->dev);
        (void)hipHostFree(b->host);
        delete b;
        g_block_count--;
    }
    g_free.clear();
    for (DevBuf *b : g_devbufs) {
        if (b->pending && hipEventSynchronize(b->ev) != hipSuccess) rc = HOP_ERR_DEVICE;
        (void)hipEventDestroy(b->ev);
        (void)hipFree(b->ptr);
        delete b;
    }
    g_devbufs.clear();
    return rc;
}

const char *hop_kernel_config(void) { return kernel_config(); }

const char *hop_strerror(int status)
{
    switch (status) {
    case HOP_OK: return "ok";
    case HOP_PARTIAL: return "fewer than k objects survived; all survivors were reduced";
    case HOP_ERR_INVALID: return "invalid argument";
    case HOP_ERR_ALIGN: return "device buffer not 16-byte aligned";
    case HOP_ERR_NO_SURVIVOR: return "no object survived";
    case HOP_ERR_DEVICE: return "HIP call failed";
    case HOP_ERR_NOMEM: return "out of memory";
    case HOP_ERR_DEPTH: return "reduce tree needs more live partial results than the kernels hold";
    case HOP_ERR_CAPTURE: return "the stream is being captured into a graph and the call would need memory from the library's caches";
    case HOP_ERR_TOO_LARGE: return "the call needs more device scratch than the static array of the no-allocation entry point holds";
    default: return "unknown status";
    }
}

}  // extern "C"
