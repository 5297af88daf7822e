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

namespace hop {

// ----------------------------------------------------------------------------
// launch helpers
// ----------------------------------------------------------------------------

// Launch shape, from sweeps on MI355X over the 64 MiB x 12, 256 MiB x 31 and
// 16 MiB x 64 workloads: one wave per workgroup, each wave owning a tile of
// 4 KiB per source (4 vectors per lane, all four loads of a source in flight
// together), one tile per workgroup so that the dispatcher keeps every CU
// supplied with fresh waves. Deeper accumulator stacks take fewer vectors per
// lane to stay inside the register file.
constexpr int kThreads = 64;
constexpr int kUnroll = 1;
constexpr size_t kMaxGrid = 1u << 22;

template <int DT, int D> struct VecPerLane {
    static constexpr int W = Traits<DT>::W;
    static constexpr int value = (D * W <= 32) ? 4 : (D * W <= 64) ? 2 : 1;
};

// Launches that cover few tiles (small objects, short chunk runs) cannot fill the
// chip with 4 KiB tiles; they use 1 KiB tiles (one vector per lane) with 16 sources
// in flight per lane instead, which shortens the dependent-load chain per wave.
constexpr int kSmallUnroll = 16;
constexpr size_t kSmallLaunchTiles = 2048;   // below this many 4 KiB tiles the small shape is used

struct Launcher {
    void (*dev)(ReduceArgs);
    void (*inl)(ReduceArgsInline);
    void (*dev_small)(ReduceArgs);
    void (*inl_small)(ReduceArgsInline);
    int vpt;
};

template <int DT, int OP, int D> static Launcher make_launcher()
{
    constexpr int V = VecPerLane<DT, D>::value;
    return {reduce_kernel<DT, OP, D, V, kUnroll, kThreads>, reduce_kernel_inline<DT, OP, D, V, kUnroll, kThreads>,
            reduce_kernel<DT, OP, D, 1, kSmallUnroll, kThreads>,
            reduce_kernel_inline<DT, OP, D, 1, kSmallUnroll, kThreads>, V};
}
template <int DT, int OP> static Launcher pick_depth(int depth)
{
    if (depth <= 1) return make_launcher<DT, OP, 1>();
    if (depth <= 2) return make_launcher<DT, OP, 2>();
    if (depth <= 4) return make_launcher<DT, OP, 4>();
    if (depth <= 8) return make_launcher<DT, OP, 8>();
    return make_launcher<DT, OP, 16>();
}
template <int DT> static Launcher pick_op(int op, int depth)
{
    switch (op) {
    case HOP_SUM: return pick_depth<DT, HOP_SUM>(depth);
    case HOP_MIN: return pick_depth<DT, HOP_MIN>(depth);
    default:      return pick_depth<DT, HOP_MAX>(depth);
    }
}

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
           "workgroup (1 KiB tiles, unroll 16 below 2048 tiles), nontemporal loads+stores, programs <= 32 steps in "
           "kernel arguments; "
           "copy: 64 lanes/workgroup, 8 vectors/lane, nontemporal";
}

static Launcher pick(int dtype, int op, int depth)
{
    switch (dtype) {
    case HOP_F32:  return pick_op<HOP_F32>(op, depth);
    case HOP_BF16: return pick_op<HOP_BF16>(op, depth);
    default:       return pick_op<HOP_I32>(op, depth);
    }
}

static void fill_range(ReduceArgs &a, int dtype, size_t byte_begin, size_t byte_end)
{
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
    const bool small = grid_for(a.base.n_vec, (size_t)kThreads * l.vpt) < kSmallLaunchTiles;
    const unsigned grid = grid_for(a.base.n_vec, (size_t)kThreads * (small ? 1 : l.vpt));
    if (n_entries <= kInlineEntries) {
        for (int i = 0; i < n_entries; ++i) a.steps[i] = host_steps[i];
        for (int i = n_entries; i < kInlineEntries; ++i) a.steps[i] = DevEntry{nullptr, 0, 0};
        hipLaunchKernelGGL(small ? l.inl_small : l.inl, dim3(grid), dim3(kThreads), 0, stream, a);
    } else {
        if (!dev_prog) return hipErrorInvalidValue;
        hipLaunchKernelGGL(small ? l.dev_small : l.dev, dim3(grid), dim3(kThreads), 0, stream, a.base);
    }
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

hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end)
{
    if (byte_end <= byte_begin || n_dst <= 0) return hipSuccess;
    CopyArgs a;
    a.src = src;
    a.dsts = dsts;
    a.n_dst = n_dst;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail_bytes = (int)((byte_end - byte_begin) % 16);
    const unsigned grid = grid_for(a.n_vec, (size_t)kThreads * kCopyVpt);
    hipLaunchKernelGGL((copy_kernel<kCopyVpt, kThreads>), dim3(grid), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace hop
