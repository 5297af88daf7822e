// Launch shape of the reduce kernels and the table of instantiations, shared by
// hop_kernels.hip (which launches) and hop_kernels_inst.hip (which instantiates).
#pragma once

#include "hop_kernels.h"

namespace hop {

// Basic shape, from sweeps on MI355X over the 64 MiB x 12, 256 MiB x 31 and
// 16 MiB x 64 workloads: one wave per workgroup, one tile per workgroup (the
// dispatcher keeps the CUs supplied with fresh waves; persistent grids and
// larger workgroups were slower), each wave owning up to 4 KiB per source
// (4 vectors per lane, the four loads of a source in flight together).
// Deeper accumulator stacks take fewer vectors per lane to stay inside the
// register file. The size of the launch then decides tile size, loads in flight,
// where a wave's vectors lie and how many waves may be resident (below).
constexpr int kThreads = 64;
constexpr int kUnroll = 1;

// Launches that cover few tiles (small objects, short chunk runs) cannot fill the
// chip with 4 KiB tiles; they use 1 KiB tiles (one vector per lane) with 8 sources
// in flight per lane instead, which shortens the dependent-load chain per wave.
constexpr int kSmallUnroll = 8;
static_assert(kSmallUnroll == kRunSteps, "runs are marked for the group size of the small shape");
constexpr size_t kSmallLaunchTiles = 768;    // below this many 4 KiB tiles the small shape is used
// In between, 2 KiB per wave with two sources in flight: finer work granularity than the large
// shape (whose few thousand long-lived waves quantise badly at these sizes), fewer
// dependent rounds than the small one. From sweeps over 0.25..24 MiB objects.
constexpr int kMidVecs = 2;
constexpr int kMidUnroll = 2;
constexpr size_t kMidLaunchTiles = 2048;     // below this many 4 KiB tiles (and above the small limit)
// Where a wave's vectors lie. The loads a wave has in flight together should not sit side by side:
// with its 4 vectors per lane in four 1 KiB pieces 64 KiB apart (instead of one contiguous 4 KiB) the
// same kernel moves 31 x 256 MiB at 88 % of the HBM peak instead of 78 %, 12 x 64 MiB at 85 % instead
// of 79 %, 4 x 128 MiB at 82 % instead of 78 %; 16 KiB apart measures about the same, 4 KiB and
// 256 KiB apart clearly less. Consecutive workgroups still cover consecutive pieces, so the chip as a
// whole streams through every source front to back. The 2 KiB shape gains 3-5 points with its two
// pieces 16 KiB apart. The alternative of keeping several sources in flight at the same offset
// (1 KiB tiles, 8 sources) depends on how the sources lie relative to each other: 70 % to 83 % for
// 31 x 256 MiB as the distance between consecutive objects varies by a few KiB; pieces of one source
// at a time do not (85-86 % for every placement tried).
constexpr int kMidPieceStrideLog2 = 4;        // 2 KiB per wave: the two pieces lie 16 KiB apart
constexpr int kPieceStrideLog2 = 6;           // up to 4 KiB per wave: the pieces lie 64 KiB apart
// Resident waves. Once the result store joins the read streams, the memory system runs best with
// few waves in flight per compute unit; kernels that need few registers otherwise fill a CU with
// 20+ waves and lose 5-10 points of bandwidth. The cap is an LDS allocation per workgroup that the
// kernels never touch. It applies to the kernels that hold 4 vectors per lane (shallow accumulator
// stacks), from 20 MiB per object: 8 waves per CU (7 is a little faster for some shapes and much slower
// for others, 10 and 12 lose 2-3 points); those with fewer vectors already hold few waves through
// their register use, and capping them further only costs (measured). Up to 16 MiB a launch fits in
// one round of uncapped waves and a cap would split it in two (12 inputs of 18 MiB: 77 % uncapped,
// 74 % capped; of 22 MiB: 78 % and 82 %).
constexpr double kMinRoundFill = 0.80;        // uncapped large launches: least fill of the rounds of resident waves
constexpr size_t kCapLaunchTiles = 5120;      // 4 KiB tiles; below: uncapped
constexpr int kLargeWavesPerCU = 8;
// bf16 with 5..8 accumulator levels keeps the 2 KiB shape (two sources in flight) at every size.
constexpr int kDeepBf16MaxDepth = 8;
constexpr unsigned kLdsBytesPerCU = 160 * 1024;
constexpr unsigned kLargeLdsBytes = kLdsBytesPerCU / kLargeWavesPerCU / 256 * 256;      // per workgroup
static_assert(kLdsBytesPerCU / kLargeLdsBytes == kLargeWavesPerCU, "cap must come out as intended");
static_assert(kLargeLdsBytes <= 64 * 1024, "needs no opt-in for large dynamic LDS");

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
    void (*dev_small_mixed)(ReduceArgs);           // bf16 only (else null): steps may read partial results
    void (*inl_small_mixed)(ReduceArgsInline);
    void (*dev_mid)(ReduceArgs);
    void (*inl_mid)(ReduceArgsInline);
    void (*seg)(ReduceArgs);
    void (*kept)(ReduceArgs);
    void (*kept_inl)(ReduceArgsInline);
    void (*chains)(ChainArgs);
    void (*chains_inl_small)(ChainArgsInline<kChainInlineWordsSmall>);
    void (*chains_inl_mid)(ChainArgsInline<kChainInlineWordsMid>);
    void (*chains_inl_large)(ChainArgsInline<kChainInlineWordsLarge>);
    void (*chains_wide)(ChainArgs);
    void (*chains_wide_inl_small)(ChainArgsInline<kChainInlineWordsSmall>);
    void (*chains_wide_inl_mid)(ChainArgsInline<kChainInlineWordsMid>);
    void (*chains_wide_inl_large)(ChainArgsInline<kChainInlineWordsLarge>);
    int vpt;
};

// One per (element type, op): the kernels for the smallest instantiated depth >= depth.
Launcher launcher_0_0(int depth); Launcher launcher_0_1(int depth); Launcher launcher_0_2(int depth);
Launcher launcher_1_0(int depth); Launcher launcher_1_1(int depth); Launcher launcher_1_2(int depth);
Launcher launcher_2_0(int depth); Launcher launcher_2_1(int depth); Launcher launcher_2_2(int depth);

}  // namespace hop
