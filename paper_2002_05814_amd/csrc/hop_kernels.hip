// gfx950 kernels of the chunked N-way reduce: a bandwidth-bound multi-input
// streaming reduce that evaluates the tree expression in registers, and a
// chunked one-to-many copy.
//
// The reduce is the elementwise ReduceOp of the paper's Table 1 applied in the
// order fixed by the reduce tree of section 3.4.2; the copy is the data
// movement of the broadcast of section 3.4.1. Both are pure streaming work:
// every input byte comes from HBM once, with 128-bit loads, nothing is staged
// through LDS and no matrix unit is involved.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "hop_device.hpp"
#include "hop_kernels.h"
#include "hop_launch_shape.h"

namespace hop {

// ----------------------------------------------------------------------------
// launch helpers
// ----------------------------------------------------------------------------

constexpr size_t kMaxGrid = 1u << 22;

static unsigned grid_for(size_t n_vec, size_t tile_vecs)
{
    size_t tiles = (n_vec + tile_vecs - 1) / tile_vecs;
    if (tiles > kMaxGrid) tiles = kMaxGrid;      // the kernels loop over tiles beyond the grid
    return (unsigned)(tiles < 1 ? 1 : tiles);
}

int elem_bytes(int dtype) { return dtype == HOP_BF16 ? 2 : 4; }

const char *kernel_config()
{
    return "reduce: 64 lanes/workgroup, 4|2|1 vectors/lane by accumulator depth, unroll 1; below 768 4-KiB tiles: 1 KiB "
           "tiles, unroll 8; below 2048: 2 KiB per workgroup, unroll 2, in two pieces 16 KiB apart; from 2048: 1 KiB "
           "pieces 64 KiB apart, one per vector (the 2 KiB shape instead if the rounds of resident waves would be less "
           "than 80 % full); kernels with 4 vectors/lane: 8 waves per CU from 5120 tiles; bf16 at "
           "depth 5..8 from 768 tiles: 2 vectors/lane, unroll 2 (pieces 64 KiB apart from 2048 tiles); groups of 8 plain steps marked by the host; "
           "nontemporal loads+stores, programs <= 128 steps in kernel arguments; vector grids start at a 128-byte boundary of "
           "the sources (reduce) or destinations (copies); "
           "copy to one destination: 64 lanes/workgroup, 8 contiguous vectors/lane; from 5120 8-KiB tiles 4 vectors/lane in "
           "1 KiB pieces 64 KiB apart, 10 waves per CU; nontemporal; "
           "to several: one 4 KiB tile and one destination per workgroup, destination-major within spans of 4096 tiles, "
           "cached loads, nontemporal stores, 12 waves per CU (no limit for >= 128 MiB to < 8 destinations); "
           "launches that keep or read partial results: one step at a time, 4|2|1 vectors/lane, pieces 64 KiB apart from 2048 "
           "tiles, 8 waves per CU from 5120 tiles, partials as 4-byte accumulators indexed like the elements, nontemporal; "
           "programs of 48 steps or more over at most 64 KiB: one launch, 256 lanes per 64-byte column, chains of at most 23 items "
           "folded by teams of 4 lanes with all their loads in flight, values in LDS, tables of up to 256 chains in the kernel arguments, "
           "four columns in a row per die; above 64 KiB up to 768 KiB: 512 lanes per 1 KiB column, a wave per chain";
}

static thread_local LaunchRecorder *tl_recorder = nullptr;

void set_launch_recorder(LaunchRecorder *r) { tl_recorder = r; }

static void not_recordable()
{
    if (tl_recorder) tl_recorder->unusable = true;
}

// Launch of a reduce kernel whose only parameter is its argument block (ReduceArgs first in it).
template <class Args>
static hipError_t enqueue(void (*kernel)(Args), dim3 grid, unsigned lds, hipStream_t stream, const Args &a, bool writes_result,
                          unsigned threads = kThreads)
{
    hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, stream, a);
    const hipError_t e = hipGetLastError();
    if (tl_recorder && e == hipSuccess) {
        RecordedLaunch r;
        r.kernel = (const void *)kernel;
        r.grid_x = grid.x;
        r.grid_y = grid.y;
        r.lds = lds;
        r.threads = threads;
        r.writes_result = writes_result;
        r.args.assign((const unsigned char *)&a, (const unsigned char *)&a + sizeof a);
        tl_recorder->launches.push_back(std::move(r));
    }
    return e;
}

hipError_t replay_launch(RecordedLaunch &l, hipStream_t stream, void *dst)
{
    // the result pointer is replaced in the recorded block itself (the runtime copies the block at the launch;
    // the caller lets one thread at a time use a recording)
    if (l.args.size() < sizeof(ReduceArgs)) return hipErrorInvalidValue;
    unsigned char *block = l.args.data();
    if (l.writes_result) std::memcpy(block + offsetof(ReduceArgs, dst), &dst, sizeof dst);
    void *params[1] = {block};
    return hipLaunchKernel(l.kernel, dim3(l.grid_x, l.grid_y), dim3(l.threads), params, l.lds, stream);
}

static Launcher pick(int dtype, int op, int depth)
{
    typedef Launcher (*fn)(int);
    static const fn table[3][3] = {{launcher_0_0, launcher_0_1, launcher_0_2},
                                   {launcher_1_0, launcher_1_1, launcher_1_2},
                                   {launcher_2_0, launcher_2_1, launcher_2_2}};
    return table[dtype][op](depth);
}

static void fill_range(ReduceArgs &a, int dtype, size_t byte_begin, size_t byte_end)
{
    a.spill = nullptr;
    a.level_stride = 0;
    a.n_restore = 0;
    a.n_save = 0;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail = (int)(((byte_end - byte_begin) % 16) / elem_bytes(dtype));
    a.piece_stride_log2 = -1;
    a.lead_vecs = 0;
}

// Workgroups of one wave that the whole device holds at once for a kernel launched without dynamic
// LDS (by its register use), asked of the runtime once per kernel; 0 if it cannot be told.
static size_t chip_slots(const void *kernel)
{
    static std::mutex mu;
    static std::vector<std::pair<const void *, size_t>> known;
    std::lock_guard<std::mutex> lk(mu);
    for (const auto &k : known)
        if (k.first == kernel) return k.second;
    size_t slots = 0;
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, 0) == hipSuccess &&
        hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && per_cu > 0 && cus > 0)
        slots = (size_t)per_cu * (size_t)cus;
    else
        (void)hipGetLastError();
    known.emplace_back(kernel, slots);
    return slots;
}

hipError_t launch_reduce(hipStream_t stream, int dtype, int op, int depth, const DevEntry *host_steps,
                         const DevEntry *dev_prog, int n_entries, void *dst, size_t byte_begin,
                         size_t byte_end, bool mixed)
{
    if (byte_end <= byte_begin || n_entries <= 0) return hipSuccess;
    const Launcher l = pick(dtype, op, depth);
    if (mixed && (!l.dev_small_mixed || !l.inl_small_mixed)) return hipErrorInvalidValue;
    ReduceArgsInline a;
    a.base.prog = dev_prog;
    a.base.n_entries = n_entries;
    a.base.dst = dst;
    a.base.sub_entries = 0;
    fill_range(a.base, dtype, byte_begin, byte_end);
    if (host_steps && a.base.n_vec > 0) a.base.lead_vecs = lead_vectors(host_steps, n_entries, byte_begin);
    // shape by the amount of work, measured in 4 KiB tiles of the range
    const size_t tiles4k = (a.base.n_vec + 255) / 256;
    // bf16 with 5..8 accumulator levels (2 vectors per lane) needs more loads in flight than one
    // source at a time gives it: two sources in flight, the pieces 64 KiB apart, no cap (64 inputs of
    // 32 MiB in a binary tree: 81 % of the HBM peak, against 59-63 % for one source at a time and
    // 70-79 %, depending on how the objects lie, for 1 KiB tiles with 8 sources in flight)
    const bool deep_bf16 = dtype == HOP_BF16 && depth > 4 && depth <= kDeepBf16MaxDepth;
    int shape = (tiles4k < kSmallLaunchTiles || mixed) ? 0 : (tiles4k < kMidLaunchTiles || deep_bf16) ? 1 : 2;
    const bool inl = n_entries <= kInlineEntries;
    const size_t n_all = a.base.n_vec + (size_t)a.base.lead_vecs;
    // strided: whole groups of (vpt << stride) pieces, one workgroup per 2^stride-th of a group
    auto grid_of = [&](int vpt, int stride_log2) {
        return stride_log2 < 0 ? grid_for(n_all, (size_t)kThreads * vpt)
                               : grid_for(n_all, ((size_t)kThreads * vpt) << stride_log2) << stride_log2;
    };
    // LDS the kernels never touch: it only caps the number of resident waves per compute unit
    const unsigned lds = (shape == 2 && l.vpt == 4 && tiles4k >= kCapLaunchTiles) ? kLargeLdsBytes : 0;
    if (shape == 2 && lds == 0 && l.vpt >= 2) {
        // One wave per workgroup and equal work per wave: a launch that needs 1.25 rounds of resident
        // waves takes as long as one that needs 2 (200 inputs of 10 MiB, fp32: 67 % of the HBM peak
        // where 8 MiB and 14 MiB reach 85 %). If the last round of the large shape would be poorly
        // filled, the 2 KiB shape with its shorter waves takes the launch (81 % in that example).
        const size_t slots = chip_slots(inl ? (const void *)l.inl : (const void *)l.dev);
        const size_t wgs = grid_of(l.vpt, kPieceStrideLog2);
        if (slots > 0 && wgs > slots) {
            const size_t rounds = (wgs + slots - 1) / slots;
            if ((double)wgs < kMinRoundFill * (double)(rounds * slots)) shape = 1;
        }
    }
    const int vpt = shape == 0 ? 1 : shape == 1 ? (l.vpt < kMidVecs ? l.vpt : kMidVecs) : l.vpt;
    const int stride_log2 = vpt < 2 ? -1 : (shape == 2 || tiles4k >= kMidLaunchTiles) ? kPieceStrideLog2
                            : shape == 1 ? kMidPieceStrideLog2 : -1;
    a.base.piece_stride_log2 = stride_log2;
    const unsigned grid = grid_of(vpt, stride_log2);
    if (inl) {
        for (int i = 0; i < n_entries; ++i) a.steps[i] = host_steps[i];
        for (int i = n_entries; i < kInlineEntries; ++i) a.steps[i] = DevEntry{nullptr, 0, 0};
        return enqueue(mixed ? l.inl_small_mixed : shape == 0 ? l.inl_small : shape == 1 ? l.inl_mid : l.inl, dim3(grid), lds,
                       stream, a, true);
    }
    if (!dev_prog) return hipErrorInvalidValue;
    return enqueue(mixed ? l.dev_small_mixed : shape == 0 ? l.dev_small : shape == 1 ? l.dev_mid : l.dev, dim3(grid), lds, stream,
                   a.base, true);
}

hipError_t launch_reduce_segment(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_prog,
                                 int n_entries, void *dst, char *spill, size_t level_stride, int n_restore,
                                 int n_save, size_t byte_begin, size_t byte_end, int lead_vecs)
{
    if (byte_end <= byte_begin) return hipSuccess;
    if ((n_entries > 0 && !dev_prog) || n_entries < 0 || (n_entries == 0 && n_restore < 1) || n_restore < 0 || n_save < 0 || n_restore > depth || n_save > depth ||
        ((n_restore > 0 || n_save > 0) && !spill))
        return hipErrorInvalidValue;
    const Launcher l = pick(dtype, op, depth);
    ReduceArgs a;
    a.prog = dev_prog;
    a.n_entries = n_entries;
    a.dst = dst;
    a.sub_entries = 0;
    fill_range(a, dtype, byte_begin, byte_end);
    a.spill = spill;
    a.level_stride = level_stride;
    a.n_restore = n_restore;
    a.n_save = n_save;
    if (a.n_vec > 0 && lead_vecs > 0 && lead_vecs < 8) a.lead_vecs = lead_vecs;
    // long ranges as in launch_reduce: pieces 64 KiB apart, and few resident waves for the 4-vector kernels
    const size_t tiles4k = (a.n_vec + 255) / 256;
    const bool strided = l.vpt >= 2 && tiles4k >= kMidLaunchTiles;
    a.piece_stride_log2 = strided ? kPieceStrideLog2 : -1;
    const unsigned lds = (l.vpt == 4 && tiles4k >= kCapLaunchTiles) ? kLargeLdsBytes : 0;
    const size_t n_all = a.n_vec + (size_t)a.lead_vecs;
    const unsigned grid = !strided ? grid_for(n_all, (size_t)kThreads * l.vpt)
                                   : grid_for(n_all, ((size_t)kThreads * l.vpt) << kPieceStrideLog2) << kPieceStrideLog2;
    not_recordable();
    hipLaunchKernelGGL(l.seg, dim3(grid), dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

// Resident waves per compute unit for the launches that keep or reuse partial results (4 vectors per
// lane, two steps' loads in flight per wave).
constexpr int kKeptWavesPerCU = 8;
constexpr unsigned kKeptLdsBytes = kLdsBytesPerCU / kKeptWavesPerCU / 256 * 256;

hipError_t launch_reduce_kept(hipStream_t stream, int dtype, int op, int depth, const DevEntry *host_steps,
                              const DevEntry *dev_prog, int n_entries, void *dst, char *kept, size_t level_stride,
                              size_t byte_begin, size_t byte_end)
{
    if (byte_end <= byte_begin || n_entries <= 0) return hipSuccess;
    if (!host_steps || !kept) return hipErrorInvalidValue;
    const Launcher l = pick(dtype, op, depth);
    ReduceArgsInline a;
    a.base.prog = dev_prog;
    a.base.n_entries = n_entries;
    a.base.dst = dst;
    a.base.sub_entries = 0;
    fill_range(a.base, dtype, byte_begin, byte_end);
    a.base.spill = kept;
    a.base.level_stride = level_stride;
    if (a.base.n_vec > 0) a.base.lead_vecs = lead_vectors(host_steps, n_entries, byte_begin);
    // shaped like the long whole-program launches: pieces 64 KiB apart, few resident waves for the
    // kernels that hold 4 vectors per lane
    const size_t tiles4k = (a.base.n_vec + 255) / 256;
    const bool strided = l.vpt >= 2 && tiles4k >= kMidLaunchTiles;
    a.base.piece_stride_log2 = strided ? kPieceStrideLog2 : -1;
    const unsigned lds = (l.vpt == 4 && tiles4k >= kCapLaunchTiles) ? kKeptLdsBytes : 0;
    const size_t n_all = a.base.n_vec + (size_t)a.base.lead_vecs;
    const unsigned grid = !strided ? grid_for(n_all, (size_t)kThreads * l.vpt)
                                   : grid_for(n_all, ((size_t)kThreads * l.vpt) << kPieceStrideLog2) << kPieceStrideLog2;
    not_recordable();
    if (n_entries <= kInlineEntries) {
        for (int i = 0; i < n_entries; ++i) a.steps[i] = host_steps[i];
        hipLaunchKernelGGL(l.kept_inl, dim3(grid), dim3(kThreads), lds, stream, a);
    } else {
        if (!dev_prog) return hipErrorInvalidValue;
        hipLaunchKernelGGL(l.kept, dim3(grid), dim3(kThreads), lds, stream, a.base);
    }
    return hipGetLastError();
}

hipError_t launch_reduce_subs(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_records,
                              int sub_entries, int n_subs, size_t byte_begin, size_t byte_end, bool mixed)
{
    if (byte_end <= byte_begin || n_subs <= 0) return hipSuccess;
    if (!dev_records || n_subs > 65535 || sub_entries < 2 || sub_entries > kMaxSubSteps + 1) return hipErrorInvalidValue;
    static_assert(kMaxSubSteps + 1 <= kThreads, "one lane per entry of a record");
    const Launcher l = pick(dtype, op, depth);
    if (mixed && !l.dev_small_mixed) return hipErrorInvalidValue;
    ReduceArgs a;
    a.prog = dev_records;
    a.n_entries = 0;
    a.dst = nullptr;
    fill_range(a, dtype, byte_begin, byte_end);
    a.sub_entries = sub_entries;
    const unsigned grid = grid_for(a.n_vec, (size_t)kThreads);
    return enqueue(mixed ? l.dev_small_mixed : l.dev_small, dim3(grid, (unsigned)n_subs), 0, stream, a, false);
}

// bf16: whole blocks of 64 vectors (1 KiB of the object, 2 KiB of accumulators), so that the layout of a kept
// partial result, which is defined on the object's byte offsets, holds inside the range's own array
size_t split_partial_bytes(int dtype, size_t byte_begin, size_t byte_end)
{
    if (dtype != HOP_BF16) return (byte_end - byte_begin + 255) & ~(size_t)255;
    const size_t first = byte_begin / 1024, last = (byte_end + 1023) / 1024;
    return (last - first) * 2048;
}

size_t split_partial_base_offset(int dtype, size_t byte_begin)
{
    return dtype != HOP_BF16 ? byte_begin : byte_begin / 1024 * 2048;
}

size_t chain_value_bytes(int dtype, bool wide)
{
    return (size_t)(wide ? kChainWideLanes : kChainLanes) * (dtype == HOP_BF16 ? 8 : 4) * 4;
}

// LDS that one workgroup of the wide form may take: kChainWideLdsBytes where the device gives a workgroup
// that much (asked once; a launch that is refused all the same takes it back), else what the narrow form has.
static std::atomic<size_t> g_wide_lds{0};
static size_t wide_lds_bytes()
{
    size_t v = g_wide_lds.load(std::memory_order_relaxed);
    if (v) return v;
    int dev = 0, per_block = 0;
    v = kChainLdsBytes;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess &&
        (size_t)per_block >= kChainWideLdsBytes)
        v = kChainWideLdsBytes;
    else
        (void)hipGetLastError();
    g_wide_lds.store(v, std::memory_order_relaxed);
    return v;
}

int chain_slots_max(int dtype, bool wide)
{
    return (int)((wide ? wide_lds_bytes() : kChainLdsBytes) / chain_value_bytes(dtype, wide)) - 1;     // one place is the identity's
}

// Tables ride in the kernel arguments until a launch with such an argument block is refused.
static std::atomic<bool> g_inline_tables{true};

bool chain_table_inline(int n_chains)
{
    return g_inline_tables.load(std::memory_order_relaxed) && n_chains >= 1 &&
           (size_t)n_chains * kChainRecordWords <= (size_t)kChainInlineWordsLarge;
}

template <int WORDS>
static hipError_t launch_chains_inline(void (*kernel)(ChainArgsInline<WORDS>), unsigned grid, unsigned lds, hipStream_t stream,
                                       const ChainArgs &base, const uint64_t *host_table, size_t n_words, int threads)
{
    static thread_local ChainArgsInline<WORDS> a;          // tens of KiB: not on the stack of every caller
    a.base = base;
    std::memcpy(a.table, host_table, n_words * sizeof(uint64_t));
    return enqueue(kernel, dim3(grid), lds, stream, a, true, threads);
}

hipError_t launch_reduce_chains(hipStream_t stream, int dtype, int op, const uint64_t *dev_table, int n_chains,
                                int n_slots, const uint32_t *pass_begin, int n_passes, void *dst,
                                size_t byte_begin, size_t byte_end, const uint64_t *host_table, bool wide)
{
    if (byte_end <= byte_begin) return hipSuccess;
    if ((!dev_table && !host_table) || !pass_begin || n_chains < 1 || n_passes < 1 || n_passes > kMaxChainPasses || n_slots < 0 ||
        n_slots > chain_slots_max(dtype, wide) || pass_begin[0] != 0 || pass_begin[n_passes] != (uint32_t)n_chains)
        return hipErrorInvalidValue;
    const Launcher l = pick(dtype, op, 1);
    ChainArgs a;
    a.base.prog = (const DevEntry *)dev_table;
    a.base.n_entries = n_passes;
    a.base.dst = dst;
    a.base.sub_entries = 0;
    fill_range(a.base, dtype, byte_begin, byte_end);
    a.identity_at = (uint32_t)((size_t)n_slots * chain_value_bytes(dtype, wide));
    for (int p = 0; p <= kMaxChainPasses; ++p) a.pass_begin[p] = pass_begin[p < n_passes ? p : n_passes];
    const size_t lanes = wide ? kChainWideLanes : kChainLanes;
    const int threads = wide ? kChainWideThreads : kChainThreads;
    const size_t n_cols = (a.base.n_vec + lanes - 1) / lanes;
    const size_t grid = n_cols + ((size_t)a.base.n_tail + lanes - 1) / lanes;
    if (grid > kMaxGrid) return hipErrorInvalidValue;       // one column per workgroup: the kernel does not loop
    const unsigned lds = (unsigned)(((size_t)n_slots + 1) * chain_value_bytes(dtype, wide));
    if (host_table && chain_table_inline(n_chains)) {
        const size_t n_words = (size_t)n_chains * kChainRecordWords;
        const int size = n_words <= (size_t)kChainInlineWordsSmall ? 0 : n_words <= (size_t)kChainInlineWordsMid ? 1 : 2;
        const hipError_t e =
            size == 0 ? launch_chains_inline(wide ? l.chains_wide_inl_small : l.chains_inl_small, (unsigned)grid, lds, stream, a, host_table, n_words, threads)
            : size == 1 ? launch_chains_inline(wide ? l.chains_wide_inl_mid : l.chains_inl_mid, (unsigned)grid, lds, stream, a, host_table, n_words, threads)
                        : launch_chains_inline(wide ? l.chains_wide_inl_large : l.chains_inl_large, (unsigned)grid, lds, stream, a, host_table, n_words, threads);
        if (e == hipSuccess) return e;
        if (lds > kChainLdsBytes) {
            // more LDS than the narrow form ever asks for: that, not the argument block, may be what was refused
            g_wide_lds.store(kChainLdsBytes, std::memory_order_relaxed);
            return e;
        }
        g_inline_tables.store(false, std::memory_order_relaxed);      // this runtime refuses the argument block
    }
    if (!dev_table) return hipErrorInvalidValue;            // the caller stages the table and calls again
    const hipError_t e = enqueue(wide ? l.chains_wide : l.chains, dim3((unsigned)grid), lds, stream, a, true, threads);
    if (e != hipSuccess && lds > kChainLdsBytes) g_wide_lds.store(kChainLdsBytes, std::memory_order_relaxed);
    return e;
}

// One destination: every vector is read once (non-temporal) and stored once; 8 contiguous
// vectors per lane in flight, and from 40 MiB 4 vectors per lane in 1 KiB pieces 64 KiB apart
// at 10 waves per CU (256 MiB: 6.47 -> 6.73 TB/s read + write, 64 MiB: 5.94 -> 6.14; at 16 MiB
// the contiguous uncapped kernel is the fastest). Several destinations: the fan-out kernel, one 4 KiB tile and one destination
// per workgroup, the source served from L2 after its first read, 12 resident waves per CU (10
// and 12 measured alike, 6 and no limit 12-15 % slower). Measured on MI355X with the source not
// in any cache beforehand, 16 / 64 / 256 MiB to 63 destinations: 151 / 592 / 2460 us against
// 187 / 768 / 3170 us for a kernel that reads a tile once and stores it to every destination in
// turn; to 8 destinations: 22 / 82 / 401 us against 25 / 114 / 481 us. Spans of 32 MiB (4 MiB
// per XCD, the whole L2) were 40 % slower than spans of 16 MiB. A source of 128 MiB or more
// going to fewer than 8 destinations is read from HBM for a large part of the run, which wants
// more waves in flight: no limit there (256 MiB to 2: 140 us against 152 us).
constexpr int kCopyVpt = 8;
constexpr int kLongCopyVpt = 4;
constexpr unsigned kCopyCapTiles = 5120;       // 8 KiB tiles: from 40 MiB per object
constexpr int kCopyWavesPerCU = 10;
constexpr unsigned kCopyLdsBytes = kLdsBytesPerCU / kCopyWavesPerCU / 256 * 256;
static_assert(kLdsBytesPerCU / kCopyLdsBytes == kCopyWavesPerCU, "cap must come out as intended");
constexpr int kFanoutVpt = 4;
constexpr unsigned kFanoutSpanTiles = 4096;    // 4 KiB tiles: 16 MiB of the source, 2 MiB per XCD
constexpr unsigned kFanoutMaxBlocks = 1u << 30;
constexpr int kFanoutMaxDst = (int)(kFanoutMaxBlocks / kFanoutSpanTiles);
constexpr int kFanoutWavesPerCU = 12;
constexpr unsigned kFanoutLdsBytes = kLdsBytesPerCU / kFanoutWavesPerCU / 256 * 256;
static_assert(kLdsBytesPerCU / kFanoutLdsBytes == kFanoutWavesPerCU, "cap must come out as intended");
constexpr int kFanoutFewDst = 8;
constexpr size_t kFanoutLongBytes = (size_t)128 << 20;
static_assert(kFanoutSpanTiles % 8 == 0, "a tile must meet the same XCD for every destination");

hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end, void *dst0, unsigned dst_residue, void *const *host_dsts)
{
    not_recordable();
    if (n_dst != 1) dst0 = nullptr;
    if (dst0) dst_residue = (unsigned)((uintptr_t)dst0 & 127);
    if (byte_end <= byte_begin || n_dst <= 0) return hipSuccess;
    const bool inl = !dst0 && host_dsts && n_dst <= kInlineDsts;
    if (!dst0 && !inl && !dsts) return hipErrorInvalidValue;
    if (n_dst == 1 && inl) { dst0 = host_dsts[0]; dst_residue = (unsigned)((uintptr_t)dst0 & 127); }
    CopyArgsInline ai;
    CopyArgs &a = ai.base;
    a.src = src;
    a.dst0 = dst0;
    a.dsts = dsts;
    a.n_dst = n_dst;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail_bytes = (int)((byte_end - byte_begin) % 16);
    a.n_tiles = 0;
    a.span_tiles = 0;
    a.piece_stride_log2 = -1;
    // where the destinations (most of them) are 128-byte aligned; the table is in device memory, so
    // the caller passes the residue it saw when it built the table
    a.lead_vecs = a.n_vec > 0 ? (int)((((uintptr_t)dst_residue + byte_begin) >> 4) & 7) : 0;
    if (n_dst >= 2 && n_dst <= kFanoutMaxDst) {
        // whole spans per launch, as many as keep the grid below kFanoutMaxBlocks (one launch
        // unless the copy is enormous); the bytes beyond the last whole vector go with the last
        constexpr size_t kTileVecs = (size_t)kThreads * kFanoutVpt;
        const size_t spans_per_launch = kFanoutMaxBlocks / ((size_t)kFanoutSpanTiles * (size_t)n_dst);
        const size_t tiles_per_launch = spans_per_launch * kFanoutSpanTiles;
        if ((a.n_vec + 8 + kTileVecs - 1) / kTileVecs > tiles_per_launch) a.lead_vecs = 0;    // several launches: plain grid
        const size_t tiles = (a.n_vec + (size_t)a.lead_vecs + kTileVecs - 1) / kTileVecs;
        a.span_tiles = kFanoutSpanTiles;
        const unsigned lds = (n_dst < kFanoutFewDst && byte_end - byte_begin >= kFanoutLongBytes) ? 0 : kFanoutLdsBytes;
        size_t done = 0;
        do {
            const size_t now = tiles - done < tiles_per_launch ? tiles - done : tiles_per_launch;
            const bool last = done + now == tiles;
            CopyArgs part = a;
            part.byte_begin = byte_begin + done * kTileVecs * 16;
            part.n_vec = last ? a.n_vec + (size_t)a.lead_vecs - done * kTileVecs - (size_t)part.lead_vecs : now * kTileVecs;
            part.n_tail_bytes = last ? a.n_tail_bytes : 0;
            part.n_tiles = (unsigned)now;
            const size_t grid = (now < 1 ? 1 : now) * (size_t)n_dst;     // one workgroup at least, for the tail bytes
            if (now == 0) part.n_tiles = 1;                              // its only tile is empty: n_vec == 0
            if (inl) {
                CopyArgsInline pi;
                pi.base = part;
                pi.base.dsts = nullptr;
                for (int i = 0; i < kInlineDsts; ++i) pi.dsts[i] = i < n_dst ? host_dsts[i] : nullptr;
                hipLaunchKernelGGL((fanout_kernel_inline<kFanoutVpt, kThreads>), dim3((unsigned)grid), dim3(kThreads), lds, stream, pi);
            } else {
                hipLaunchKernelGGL((fanout_kernel<kFanoutVpt, kThreads>), dim3((unsigned)grid), dim3(kThreads), lds, stream, part);
            }
            done += now;
        } while (done < tiles);
        return hipGetLastError();
    }
    const size_t n_all = a.n_vec + (size_t)a.lead_vecs;
    const unsigned grid = grid_for(n_all, (size_t)kThreads * kCopyVpt);
    if (grid >= kCopyCapTiles) {
        // long copies, like long reduces, run faster with few resident waves and with a wave's
        // vectors apart (256 MiB one-to-one: 77 % -> 84 % of the HBM peak)
        a.piece_stride_log2 = kPieceStrideLog2;
        const unsigned g = grid_for(n_all, ((size_t)kThreads * kLongCopyVpt) << kPieceStrideLog2) << kPieceStrideLog2;
        hipLaunchKernelGGL((copy_kernel<kLongCopyVpt, kThreads>), dim3(g), dim3(kThreads), kCopyLdsBytes, stream, a);
    } else {
        hipLaunchKernelGGL((copy_kernel<kCopyVpt, kThreads>), dim3(grid), dim3(kThreads), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace hop
