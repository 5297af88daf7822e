// Launch shape of the reduce kernels and the table of instantiations, shared by
// hop_kernels.hip (which launches) and hop_kernels_inst.hip (which instantiates).
#pragma once

#include "hop_kernels.h"

namespace hop {

// Basic shape, from sweeps on MI355X over the 64 MiB x 12, 256 MiB x 31 and
// 16 MiB x 64 workloads: one wave per workgroup, one tile per workgroup (the
// dispatcher keeps the CUs supplied with fresh waves; persistent grids and
// larger workgroups were slower), each wave owning a tile of up to 4 KiB per
// source (4 vectors per lane, the four loads of a source in flight together).
// Deeper accumulator stacks take fewer vectors per lane to stay inside the
// register file. The size of the launch then decides tile size, loads in flight
// and how many waves may be resident (below).
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
// Resident waves. Once the result store joins the read streams, the memory system runs best with
// few waves in flight per compute unit, each with several loads outstanding; kernels that need few
// registers otherwise fill a CU with 20+ waves and lose 5-10 points of bandwidth (a chain over
// 12 x 64 MiB fp32: 72 % of the HBM peak uncapped, 79-84 % capped). The cap is an LDS allocation
// per workgroup that the kernels never touch. It applies to the kernels that hold 4 vectors per
// lane (shallow accumulator stacks); those with fewer (deep stacks, bf16 from depth 3) already hold
// few waves through their register use, and capping them further only costs (measured).
//  - from 48 MiB per object: the 1 KiB-tile kernel with 8 sources in flight at 10 waves per CU (9 measured a little faster still on the
//    two large workloads, 7 much slower: 10 keeps a margin)
//    (12 x 64 MiB fp32, degree 4: 79 % -> 83-85 %; gains of 3..10 points in sweeps over chains,
//    stars and trees of 4..64 inputs of 64..512 MiB, fp32, int32 and bf16);
//  - from 16 MiB: 4 KiB tiles at 8 waves per CU (12 x 16 MiB fp32: 70 % -> 75 %; 32 inputs: 72 % ->
//    83 %); below that a launch fits in one round of uncapped waves and a cap would split it in two.
constexpr size_t kCapLaunchTiles = 4096;      // 4 KiB tiles; below: uncapped
constexpr int kLargeWavesPerCU = 8;
constexpr size_t kStreamLaunchTiles = 12288;  // from this many 4 KiB tiles: 1 KiB tiles, 8 sources in flight
constexpr int kStreamMaxDepth = 8;
constexpr int kStreamWavesPerCU = 10;
constexpr unsigned kLdsBytesPerCU = 160 * 1024;
constexpr unsigned kStreamLdsBytes = kLdsBytesPerCU / kStreamWavesPerCU / 256 * 256;   // per workgroup
constexpr unsigned kLargeLdsBytes = kLdsBytesPerCU / kLargeWavesPerCU / 256 * 256;
static_assert(kLdsBytesPerCU / kStreamLdsBytes == kStreamWavesPerCU, "cap must come out as intended");
static_assert(kLdsBytesPerCU / kLargeLdsBytes == kLargeWavesPerCU, "cap must come out as intended");
static_assert(kStreamLdsBytes <= 64 * 1024 && kLargeLdsBytes <= 64 * 1024, "needs no opt-in for large dynamic LDS");

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
