// Launch interface between the host scheduler's GPU back end and the gfx950
// kernels (hop_kernels.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/hop.h"

namespace hop {

// One accumulator-program step as the kernel reads it (16 bytes, so that a
// step is one scalar 128-bit load): the source object's base address and
// ctl = level | set << 8 | n_fold << 16.
struct DevEntry {
    const void *src;
    uint32_t ctl;
    uint32_t reserved;
};
static_assert(sizeof(DevEntry) == 16, "program steps are 16 bytes");

struct ReduceArgs {
    const DevEntry *prog;      // device memory, n_entries steps
    int n_entries;
    void *dst;                 // result
    void *const *extra_dsts;   // device table of n_extra further destinations (allreduce), or null
    int n_extra;
    size_t byte_begin;         // first byte of the object range this launch covers
    size_t n_vec;              // full 16-byte vectors in the range
    int n_tail;                // elements after the last full vector (object end only)
};

struct CopyArgs {
    const void *src;
    void *const *dsts;         // device table
    int n_dst;
    size_t byte_begin;
    size_t n_vec;
    int n_tail_bytes;
};

// Workgroups per compute unit for the grid-stride loops.
constexpr int kReduceBlocksPerCu = 8;
constexpr int kCopyBlocksPerCu = 8;

int elem_bytes(int dtype);

// Reduce the byte range [byte_begin, byte_end) of the objects named by the
// program into dst (and the extra destinations). depth = accumulator levels
// the program uses (1..HOP_MAX_DEPTH). All pointers are device pointers.
hipError_t launch_reduce(hipStream_t stream, int dtype, int op, int depth, const DevEntry *prog,
                         int n_entries, void *dst, void *const *extra_dsts, int n_extra,
                         size_t byte_begin, size_t byte_end, int n_cu);

// Copy [byte_begin, byte_end) of src into the same range of every destination.
hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end, int n_cu);

}  // namespace hop
