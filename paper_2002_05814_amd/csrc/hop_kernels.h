// Launch interface between the host scheduler's GPU back end and the gfx950
// kernels (hop_kernels.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/hop.h"
#include "hop_program.h"

namespace hop {

// Programs of at most this many steps travel inside the kernel arguments
// (no separate host-to-device copy, steps read straight from the argument
// segment; measured 4 us per call from C against 21 us through the staging
// path); longer ones are staged in device memory.
constexpr int kInlineEntries = 128;

// Several independent sub-programs evaluated by a single launch (grid dimension y): the launch's
// program memory holds gridDim.y records of sub_entries entries each, a SubHeader and then the
// sub-program's steps (at most kMaxSubSteps, the rest of the record is padding). A workgroup
// fetches its whole record with one vector load, lane i entry i, and takes the steps from
// the lanes afterwards: one trip to the program's memory instead of one per group of steps, which
// matters because these programs are read in place from pinned host memory.
struct SubHeader {
    void *dst;                 // where the sub-program's result goes
    uint32_t n_entries;        // its number of steps
    uint32_t flags;            // kSubStoresAccumulators or 0
};
// The sub-program's result is stored as accumulator-typed values, 4 bytes per element in the layout of a
// kept partial result, not as elements (bf16: what later sub-programs and the top read with kPartialBit).
constexpr uint32_t kSubStoresAccumulators = 1u;
static_assert(sizeof(SubHeader) == sizeof(DevEntry), "a header takes one entry");
constexpr int kMaxSubSteps = 63;   // header + steps fit the 64 lanes of a wave

struct ReduceArgs {
    const DevEntry *prog;      // device memory, n_entries steps (unused by the inline variant)
    int n_entries;
    void *dst;                 // result
    size_t byte_begin;         // first byte of the object range this launch covers
    size_t n_vec;              // full 16-byte vectors in the range
    int n_tail;                // elements after the last full vector (object end only)
    int sub_entries;           // > 0: prog holds gridDim.y sub-program records of this many entries (see SubHeader)
    int lead_vecs;             // the workgroups' grid of vectors starts this many vectors before byte_begin, where
                               // the sources are 128-byte aligned; the vectors in front of the range are skipped
    int piece_stride_log2;     // < 0: a workgroup's vectors are contiguous; s >= 0: its VPT pieces of one vector
                               // per lane lie 2^s pieces apart (see reduce_body)
    // segment launches only (reduce_kernel_seg): where accumulators live between segments
    char *spill;               // level L's array starts at spill + L * level_stride
    size_t level_stride;
    int n_restore;             // levels read back before the first step
    int n_save;                // levels written after the last step; 0 = store the result to dst instead
};

struct ReduceArgsInline {
    ReduceArgs base;
    DevEntry steps[kInlineEntries];
};
static_assert(sizeof(ReduceArgsInline) <= 4096, "these argument blocks stay within 4 KiB, which every runtime takes");

// A long program over a short byte range, evaluated by one launch as chains (see plan_chains in
// hop_plan.hpp): a workgroup of kChainThreads lanes owns a column of kChainLanes 16-byte vectors
// of the objects; its lanes form kChainTeams teams of kChainLanes, each team folds one chain at a
// time, and the chains' values live in LDS between the passes (kChainLanes x W accumulators per
// value that is still needed; W = accumulators per vector). The table in device memory holds one
// record of kChainRecordWords 8-byte words per chain, in pass order: word 0 = where the value goes,
// as a byte offset into the workgroup's LDS (bits 0..31; kChainFinal: it is the result and goes to
// dst); words 1..kChainMaxItems = the items, each the address of an object (never below 2^32) or
// the LDS byte offset of a chain's value, and behind the last item the offset of the identity value
// (identity_at) up to the end of the record, so that loads and folds need not look at a count.
constexpr int kChainLanes = 4;
constexpr int kChainColumnRun = 4;       // columns in a row that one die's workgroups take
constexpr int kChainTeams = 64;
constexpr int kChainThreads = kChainLanes * kChainTeams;
// The wide form of the same: a team is a whole wave (a column of 64 vectors = 1 KiB of the objects, a value
// 1 KiB of LDS for 32-bit elements), 8 chains side by side. For ranges of hundreds of KiB.
constexpr int kChainWideLanes = 64;
constexpr int kChainWideTeams = 8;
constexpr int kChainWideThreads = kChainWideLanes * kChainWideTeams;
constexpr int kChainMaxItems = 23;
constexpr int kChainRecordWords = kChainMaxItems + 1;
constexpr int kMaxChainPasses = 24;
constexpr uint32_t kChainFinal = 0xffffffffu;
constexpr size_t kChainLdsBytes = 64 * 1024;
constexpr size_t kChainWideLdsBytes = 128 * 1024;  // the wide form, where the device gives a workgroup that much
struct ChainArgs {
    ReduceArgs base;           // prog = the table, n_entries = number of passes, dst / byte_begin / n_vec / n_tail as usual
    uint32_t identity_at;      // LDS byte offset of the identity value (behind the chains' values)
    uint32_t pass_begin[kMaxChainPasses + 1];      // pass p evaluates the chains [pass_begin[p], pass_begin[p + 1])
};
// The same with the table inside the kernel arguments. This runtime takes argument blocks far beyond
// the 4 KiB of older ones (64 KiB were tried); a launch that is refused falls back to the staged table
// for good (launch_reduce_chains). Three sizes, so that a small table does not cost a large copy (the
// runtime copies the whole block at every launch: 4 KiB more cost the host about 0.5 us).
template <int WORDS> struct ChainArgsInline {
    ChainArgs base;
    alignas(16) uint64_t table[WORDS];
};
constexpr int kChainInlineWordsSmall = 1536;       // 64 chains, 12 KiB
constexpr int kChainInlineWordsMid = 3072;         // 128 chains, 24 KiB
constexpr int kChainInlineWordsLarge = 6144;       // 256 chains, 48 KiB

struct CopyArgs {
    const void *src;
    void *dst0;                // the only destination when dsts is null
    void *const *dsts;         // device table, or null
    int n_dst;
    size_t byte_begin;
    size_t n_vec;
    int n_tail_bytes;
    int piece_stride_log2;     // copy kernel only: < 0 contiguous vectors per workgroup, else pieces 2^s apart
    int lead_vecs;             // the grid of vectors starts this many vectors before byte_begin, where the
                               // destinations are 128-byte aligned; vectors in front of the range are skipped
    unsigned n_tiles;          // fan-out kernel only: tiles in this launch
    unsigned span_tiles;       // fan-out kernel only: tiles per span
};

// Destination tables of at most this many entries travel inside the kernel arguments
// (no staging copy in front of the copy kernel); longer ones are staged in device memory.
constexpr int kInlineDsts = 64;
struct CopyArgsInline {
    CopyArgs base;
    void *dsts[kInlineDsts];
};
static_assert(sizeof(CopyArgsInline) <= 4096, "these argument blocks stay within 4 KiB, which every runtime takes");

int elem_bytes(int dtype);

// Recording of kernel launches, for calls that will be repeated with the same arguments: while a
// recorder is installed on the calling thread, every whole-program reduce launch (launch_reduce,
// launch_reduce_subs, launch_reduce_chains) is also written down - kernel, grid, workgroup size, LDS, the argument block - and can be
// enqueued again later with replay_launch, with another result buffer if the launch wrote the
// caller's result. Launches of any other kind mark the recording unusable.
struct RecordedLaunch {
    const void *kernel;
    unsigned grid_x, grid_y, lds, threads;
    bool writes_result;                 // the argument block's ReduceArgs::dst is the caller's destination
    std::vector<unsigned char> args;
};
struct LaunchRecorder {
    std::vector<RecordedLaunch> launches;
    bool unusable = false;
};
void set_launch_recorder(LaunchRecorder *r);          // per host thread; nullptr = none
hipError_t replay_launch(RecordedLaunch &l, hipStream_t stream, void *dst);       // one thread at a time per recording

// Launch shape of the kernels, as text.
const char *kernel_config();

// Reduce the byte range [byte_begin, byte_end) of the objects named by the
// program into dst. depth = accumulator levels the program uses
// (1..HOP_MAX_DEPTH). host_steps = the n_entries steps in host memory; when
// there are more than kInlineEntries of them, dev_prog must hold the same
// steps in device memory. Every other pointer is a device pointer.
hipError_t launch_reduce(hipStream_t stream, int dtype, int op, int depth, const DevEntry *host_steps,
                         const DevEntry *dev_prog, int n_entries, void *dst, size_t byte_begin,
                         size_t byte_end, bool mixed = false);

// Steps [0, n_entries) of dev_prog as one segment of a longer program: n_restore accumulator
// levels are read back from the spill area first; then n_save levels are written to it, or, if
// n_save is 0, the result goes to dst. The spill area holds, per level, one array of 4-byte
// accumulators indexed like the object's elements; levels are level_stride bytes apart.
hipError_t launch_reduce_segment(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_prog,
                                 int n_entries, void *dst, char *spill, size_t level_stride, int n_restore,
                                 int n_save, size_t byte_begin, size_t byte_end, int lead_vecs = 0);

// A whole program (n_entries steps in device memory) some of whose steps read kept partial results
// (kPartialBit) or store one (aux): `kept` is the area of the kept partials, one array of 4-byte
// accumulators per partial, indexed like the object's elements, level_stride bytes apart.
// host_steps = the steps in host memory; with more than kInlineEntries of them dev_prog must hold them too.
hipError_t launch_reduce_kept(hipStream_t stream, int dtype, int op, int depth, const DevEntry *host_steps,
                              const DevEntry *dev_prog, int n_entries, void *dst, char *kept, size_t level_stride,
                              size_t byte_begin, size_t byte_end);

// The same for n_subs independent sub-programs at once: dev_records holds n_subs records of
// sub_entries entries (SubHeader, steps, padding; 2 <= sub_entries <= kMaxSubSteps + 1); every
// sub-program covers the same byte range and needs at most `depth` accumulator levels.
// mixed (bf16 only): steps may carry kPartialBit. Headers may carry kSubStoresAccumulators either way (bf16).
hipError_t launch_reduce_subs(hipStream_t stream, int dtype, int op, int depth, const DevEntry *dev_records,
                              int sub_entries, int n_subs, size_t byte_begin, size_t byte_end, bool mixed = false);
// Bytes of one partial result of a cut program over [byte_begin, byte_end) of the objects, and how far in
// front of its first byte the address lies that the kernels take as its base (they address sources by the
// object's byte offset). 32-bit elements: the range itself. bf16: 4-byte accumulators in the layout of a
// kept partial result, whose blocks of 64 vectors start at multiples of 1 KiB of the object.
size_t split_partial_bytes(int dtype, size_t byte_begin, size_t byte_end);
size_t split_partial_base_offset(int dtype, size_t byte_begin);

// The program as chains in one launch: dev_table as described at ChainArgs (n_chains records, written for
// values of chain_value_bytes(dtype) bytes each) or, for tables that ride in the kernel arguments, host_table (the
// same in host memory), n_slots = values alive at most at one time; the identity
// value takes the place behind them. hipErrorInvalidValue if that is more LDS than a workgroup gets.
// wide: the form with 1 KiB columns (the table written for its values and its kChainWideTeams teams).
hipError_t launch_reduce_chains(hipStream_t stream, int dtype, int op, const uint64_t *dev_table, int n_chains,
                                int n_slots, const uint32_t *pass_begin, int n_passes, void *dst,
                                size_t byte_begin, size_t byte_end, const uint64_t *host_table = nullptr, bool wide = false);
// Whether a table of n_chains records rides in the kernel arguments (then launch_reduce_chains needs
// host_table only, else dev_table).
bool chain_table_inline(int n_chains);
// LDS bytes of one chain's value, and the number of values a launch_reduce_chains may keep alive at
// one time, for this element type.
size_t chain_value_bytes(int dtype, bool wide = false);
int chain_slots_max(int dtype, bool wide = false);

// Copy [byte_begin, byte_end) of src into the same range of n_dst destinations: dst0 if n_dst == 1
// and dst0 is given; else the table host_dsts (host memory) if it has at most kInlineDsts entries
// (it then rides in the kernel arguments); else the device table dsts.
// dst_residue: address modulo 128 of the table's destinations (of most of them, if they
// differ; see common_residue), used to start the stores at whole lines; dst0's own otherwise.
hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end, void *dst0 = nullptr, unsigned dst_residue = 0,
                       void *const *host_dsts = nullptr);

// The address modulo 128 that most of n (16-byte aligned) host-visible pointers share.
inline unsigned common_residue(void *const *p, int n)
{
    int count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < n; ++i) count[((uintptr_t)p[i] >> 4) & 7]++;
    int best = 0;
    for (int r = 1; r < 8; ++r)
        if (count[r] > count[best]) best = r;
    return (unsigned)best * 16;
}

}  // namespace hop
