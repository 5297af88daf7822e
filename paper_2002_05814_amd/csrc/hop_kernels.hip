// gfx950 kernels of the chunked N-way reduce: a bandwidth-bound multi-input
// streaming reduce that evaluates the tree expression in registers, and a
// chunked one-to-many copy.
//
// The reduce is the elementwise ReduceOp of the paper's Table 1 applied in the
// order fixed by the reduce tree of section 3.4.2; the copy is the data
// movement of the broadcast of section 3.4.1. Both are pure streaming work:
// every input byte is read once with 128-bit loads, nothing is staged through
// LDS and no matrix unit is involved.
#include <hip/hip_runtime.h>
#include <stdint.h>

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
    return "reduce: 64 lanes/workgroup, 4|2|1 vectors/lane by accumulator depth, unroll 1, one 4 KiB tile per "
           "workgroup (2 KiB tiles, unroll 2 below 2048 tiles; 1 KiB tiles, unroll 8 below 768); kernels with 4 vectors/lane: "
           "8 waves per CU from 4096 tiles, and from 12288 tiles (bf16 at depth 5..8: from 4096) 1 KiB tiles, unroll 8, 10 waves per CU; nontemporal loads+stores, programs <= 128 steps in "
           "kernel arguments; "
           "copy: 64 lanes/workgroup, 8 vectors/lane, 10 waves per CU from 5120 tiles, nontemporal";
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
}

hipError_t launch_reduce(hipStream_t stream, int dtype, int op, int depth, const DevEntry *host_steps,
                         const DevEntry *dev_prog, int n_entries, void *dst, size_t byte_begin,
                         size_t byte_end)
{
    if (byte_end <= byte_begin || n_entries <= 0) return hipSuccess;
    const Launcher l = pick(dtype, op, depth);
    ReduceArgsInline a;
    a.base.prog = dev_prog;
    a.base.n_entries = n_entries;
    a.base.dst = dst;
    a.base.subs = nullptr;
    fill_range(a.base, dtype, byte_begin, byte_end);
    // shape by the amount of work, measured in 4 KiB tiles of the range
    const size_t tiles4k = (a.base.n_vec + 255) / 256;
    // bf16 with 5..8 accumulator levels is bound by its unpacking arithmetic at 2 vectors per lane
    // (64 inputs in a binary tree: 56 % of the HBM peak at any size); one vector per lane with 8
    // sources in flight keeps it at 77-80 %
    const bool deep_bf16 = dtype == HOP_BF16 && depth > 4 && depth <= kStreamMaxDepth && tiles4k >= kCapLaunchTiles;
    const bool stream_shape = (tiles4k >= kStreamLaunchTiles && l.vpt == 4 && depth <= kStreamMaxDepth) || deep_bf16;
    const int shape = (tiles4k < kSmallLaunchTiles || stream_shape) ? 0 : tiles4k < kMidLaunchTiles ? 1 : 2;
    const int vpt = shape == 0 ? 1 : shape == 1 ? (l.vpt < kMidVecs ? l.vpt : kMidVecs) : l.vpt;
    // LDS the kernels never touch: it only caps the number of resident waves per compute unit
    const unsigned lds = stream_shape ? kStreamLdsBytes
                         : (shape == 2 && vpt == 4 && tiles4k >= kCapLaunchTiles) ? kLargeLdsBytes : 0;
    const unsigned grid = grid_for(a.base.n_vec, (size_t)kThreads * vpt);
    if (n_entries <= kInlineEntries) {
        for (int i = 0; i < n_entries; ++i) a.steps[i] = host_steps[i];
        hipLaunchKernelGGL(shape == 0 ? l.inl_small : shape == 1 ? l.inl_mid : l.inl, dim3(grid), dim3(kThreads), lds,
                           stream, a);
    } else {
        if (!dev_prog) return hipErrorInvalidValue;
        hipLaunchKernelGGL(shape == 0 ? l.dev_small : shape == 1 ? l.dev_mid : l.dev, dim3(grid), dim3(kThreads), lds,
                           stream, a.base);
    }
    return hipGetLastError();
}

hipError_t launch_reduce_segment(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_prog,
                                 int n_entries, void *dst, char *spill, size_t level_stride, int n_restore,
                                 int n_save, size_t byte_begin, size_t byte_end)
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
    a.subs = nullptr;
    fill_range(a, dtype, byte_begin, byte_end);
    a.spill = spill;
    a.level_stride = level_stride;
    a.n_restore = n_restore;
    a.n_save = n_save;
    const unsigned grid = grid_for(a.n_vec, (size_t)kThreads * l.vpt);
    hipLaunchKernelGGL(l.seg, dim3(grid), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_reduce_subs(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_prog,
                              const SubLaunch *dev_subs, int n_subs, size_t byte_begin, size_t byte_end)
{
    if (byte_end <= byte_begin || n_subs <= 0) return hipSuccess;
    if (!dev_prog || !dev_subs || n_subs > 65535) return hipErrorInvalidValue;
    const Launcher l = pick(dtype, op, depth);
    ReduceArgs a;
    a.prog = dev_prog;
    a.n_entries = 0;
    a.dst = nullptr;
    a.subs = dev_subs;
    fill_range(a, dtype, byte_begin, byte_end);
    const unsigned grid = grid_for(a.n_vec, (size_t)kThreads);
    hipLaunchKernelGGL(l.dev_small, dim3(grid, (unsigned)n_subs), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

// The copy is write-bound; longer bursts per destination pay: 8 vectors per lane
// (8 KiB per wave and destination) beat 1, 2 and 4 in sweeps with 63 destinations,
// as did keeping all destinations in one workgroup rather than splitting them.
constexpr int kCopyVpt = 8;
constexpr unsigned kCopyCapTiles = 5120;       // 8 KiB tiles: from 40 MiB per object
constexpr int kCopyWavesPerCU = 10;
constexpr unsigned kCopyLdsBytes = kLdsBytesPerCU / kCopyWavesPerCU / 256 * 256;
static_assert(kLdsBytesPerCU / kCopyLdsBytes == kCopyWavesPerCU, "cap must come out as intended");

hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end, void *dst0)
{
    if (byte_end <= byte_begin || n_dst <= 0) return hipSuccess;
    if (!dsts && (n_dst != 1 || !dst0)) return hipErrorInvalidValue;
    CopyArgs a;
    a.src = src;
    a.dst0 = dst0;
    a.dsts = dsts;
    a.n_dst = n_dst;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail_bytes = (int)((byte_end - byte_begin) % 16);
    const unsigned grid = grid_for(a.n_vec, (size_t)kThreads * kCopyVpt);
    // long copies, like long reduces, run faster with few resident waves (256 MiB one-to-one:
    // 77 % -> 82 % of the HBM peak; 64 MiB to 8 destinations: 63 % -> 67 %; 16 MiB to 63: unchanged)
    const unsigned lds = grid >= kCopyCapTiles ? kCopyLdsBytes : 0;
    hipLaunchKernelGGL((copy_kernel<kCopyVpt, kThreads>), dim3(grid), dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace hop
