// Launch shape of the reduce kernels and the table of instantiations, shared by
// hop_kernels.hip (which launches) and hop_kernels_inst.hip (which instantiates).
#pragma once

#include "hop_kernels.h"

namespace hop {

// Launch shape, from sweeps on MI355X over the 64 MiB x 12, 256 MiB x 31 and
// 16 MiB x 64 workloads: one wave per workgroup, each wave owning a tile of
// 4 KiB per source (4 vectors per lane, all four loads of a source in flight
// together), one tile per workgroup so that the dispatcher keeps every CU
// supplied with fresh waves. Deeper accumulator stacks take fewer vectors per
// lane to stay inside the register file.
constexpr int kThreads = 64;
constexpr int kUnroll = 1;

// Launches that cover few tiles (small objects, short chunk runs) cannot fill the
// chip with 4 KiB tiles; they use 1 KiB tiles (one vector per lane) with 8 sources
// in flight per lane instead, which shortens the dependent-load chain per wave.
constexpr int kSmallUnroll = 8;
constexpr size_t kSmallLaunchTiles = 768;    // below this many 4 KiB tiles the small shape is used
// In between, 2 KiB tiles with two sources in flight: finer work granularity than the large
// shape (whose few thousand long-lived waves quantise badly at these sizes), fewer
// dependent rounds than the small one. From sweeps over 0.25..24 MiB objects.
constexpr int kMidVecs = 2;
constexpr int kMidUnroll = 2;
constexpr size_t kMidLaunchTiles = 2048;     // below this many 4 KiB tiles (and above the small limit)

// W = accumulators per 16-byte vector (4 for 32-bit elements, 8 for bf16)
// bf16 (W = 8) steps down one notch earlier than the 32-bit types: at equal accumulator count its
// unpacking temporaries cost occupancy (236 VGPRs at D = 4, 4 vectors), which showed as a wave
// quantisation dip around 10 MiB objects and no gain at 256 MiB.
template <int W, int D> struct VecPerLane {
    static constexpr int value = (D * W <= 16) ? 4 : (D * W <= 32) ? (W == 8 ? 2 : 4) : (D * W <= 64) ? 2 : 1;
};

struct Launcher {
    void (*dev)(ReduceArgs);
    void (*inl)(ReduceArgsInline);
    void (*dev_small)(ReduceArgs);
    void (*inl_small)(ReduceArgsInline);
    void (*dev_mid)(ReduceArgs);
    void (*inl_mid)(ReduceArgsInline);
    void (*seg)(ReduceArgs);
    int vpt;
};

// One per (element type, op): the kernels for the smallest instantiated depth >= depth.
Launcher launcher_0_0(int depth); Launcher launcher_0_1(int depth); Launcher launcher_0_2(int depth);
Launcher launcher_1_0(int depth); Launcher launcher_1_1(int depth); Launcher launcher_1_2(int depth);
Launcher launcher_2_0(int depth); Launcher launcher_2_1(int depth); Launcher launcher_2_2(int depth);

}  // namespace hop
