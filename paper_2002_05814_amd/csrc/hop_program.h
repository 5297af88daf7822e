// The accumulator program as the kernels read it, and the host-side marking of step groups.
// No HIP types here: the host-only tests include this file too.
#pragma once

#include <stddef.h>
#include <stdint.h>

namespace hop {

// One accumulator-program step as the kernel reads it (16 bytes, so that a
// step is one scalar 128-bit load): the source object's base address and
// ctl = level | set << 8 | run << 9 | partial << 10 | n_fold << 16 (run: see kRunBit;
// partial: see kPartialBit). aux is read only by the kernels that keep or reuse partial
// results: 0, or (1 + q) | save_level << 16 = once the folds of this step have come down to
// save_level, acc[save_level] is also stored as kept partial q.
struct DevEntry {
    const void *src;
    uint32_t ctl;
    uint32_t aux;
};
static_assert(sizeof(DevEntry) == 16, "program steps are 16 bytes");

// Bit 9 of ctl, set by mark_runs on the first step of a group of kRunSteps steps (groups counted
// from the first step of a program or sub-program) when every step of the group is a plain
// "combine into the accumulator of this level": no set, no fold, one level. The kernel that walks
// programs in groups of kRunSteps then takes the group without looking at the other control words,
// which is most of the per-step instruction count for programs over many small objects (a node
// with 16 leaf children is a run of 16 such steps). Kernels with other group sizes ignore the bit.
constexpr uint32_t kRunBit = 1u << 9;
// Bit 10 of ctl: src is not an object but an array of accumulator-typed values, one per element
// (4 bytes each whatever the element type): a kept partial result.
constexpr uint32_t kPartialBit = 1u << 10;
constexpr int kRunSteps = 8;
inline void mark_runs(DevEntry *steps, size_t n)
{
    for (size_t t = 0; t + kRunSteps <= n; t += kRunSteps) {
        bool plain = true;
        for (int u = 0; u < kRunSteps; ++u)
            plain = plain && (steps[t + u].ctl & ~0xffu) == 0 && (steps[t + u].ctl & 0xffu) == (steps[t].ctl & 0xffu);
        if (plain) steps[t].ctl |= kRunBit;
    }
}

// Vectors between the last 128-byte boundary of the sources and the start of the range: the residue
// most of the program's sources share (objects from one allocator usually share it). The kernels
// start their grid of vectors that many vectors before the range.
inline int lead_vectors(const DevEntry *host_steps, int n_entries, size_t byte_begin)
{
    int count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < n_entries; ++i) count[(((uintptr_t)host_steps[i].src + byte_begin) >> 4) & 7]++;
    int best = 0;
    for (int r = 1; r < 8; ++r)
        if (count[r] > count[best]) best = r;
    return best;
}

}  // namespace hop
