// The back ends the chunk scheduler sends its launches to: the GPU back end, which turns them into
// kernel launches on the caller's stream (whole programs, segments with saved accumulators,
// launches that keep or reuse partial results, sub-programs for many small objects, the copies of an
// allreduce), and the recording back end behind the host-only planning calls.
// Included by hop_api.hip only.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "hop_kernels.h"
#include "hop_plan.hpp"
#include "hop_workspace.hpp"

namespace hop {

// ----------------------------------------------------------------------------
// back ends
// ----------------------------------------------------------------------------

struct Shape {
    size_t object_bytes = 0, chunk_bytes = 0;
    int64_t n_chunks = 1;
    size_t begin(int64_t c) const { return (size_t)c * chunk_bytes; }
    size_t end(int64_t c) const { size_t e = (size_t)c * chunk_bytes; return e < object_bytes ? e : object_bytes; }
};

// When a long program over few output tiles is cut into sub-programs with partial results in memory
// (GpuBackend::launch_split), and when it is evaluated as chains in one launch (launch_chains); the
// measurements behind the numbers stand at those functions.
constexpr size_t kSplitWantSteps = 128;             // shorter programs are not worth extra launches
constexpr int kSplitMaxRun = kMaxSubSteps;          // longest sub-program: a record fits the lanes of a wave
constexpr size_t kSplitMaxBytes = 768u << 10;       // above, a wave's walk through the whole program is hidden behind the streaming
constexpr size_t kSplitMaxBytesBf16 = 512u << 10;   // bf16's partial results are twice the range: the cut stops paying earlier
inline size_t split_max_bytes(int dtype) { return dtype == HOP_BF16 ? kSplitMaxBytesBf16 : kSplitMaxBytes; }
constexpr int kSplitMinRun = 4;
constexpr size_t kSplitMaxScratch = 256u << 20;     // partial results of all sub-programs
constexpr size_t kChainWantSteps = 48;              // shorter programs: one wave per tile walks them as fast
constexpr size_t kChainMaxBytes = 64u << 10;        // at most 1024 columns
constexpr int kChainMinCut = 4;
constexpr size_t kChainMaxWork = 3072;              // columns x rounds
constexpr size_t kChainWideMaxBytes = 768u << 10;   // the wide form: ranges above kChainMaxBytes up to this
constexpr size_t kChainWideEarlyBytes = 32u << 10;  // bf16 (two narrow workgroups per compute unit, not three): the wide form
constexpr size_t kChainWideEarlySteps = 384;        // already from here on for programs up to this length

class GpuBackend : public Backend {
public:
    // static_base != nullptr: all device scratch comes from [static_base, static_base + static_cap) and
    // nothing is allocated (the back end of hop_reduce_noalloc)
    GpuBackend(int device, hipStream_t stream, const void *const *objs, int n, std::vector<void *> dsts,
               const Shape &shape, int op, int dtype, int k, int64_t degree, char *static_base = nullptr,
               size_t static_cap = 0)
        : ws_(device, stream, static_base, static_cap), stream_(stream), objs_(objs, objs + n), dsts_(std::move(dsts)), shape_(shape),
          op_(op), dtype_(dtype), k_(k), degree_(degree), device_(device), library_scratch_(static_base != nullptr)
    {
        if (dsts_.size() > 1) extra_residue_ = common_residue(dsts_.data() + 1, (int)dsts_.size() - 1);
    }

    ~GpuBackend() override
    {
        release_devbuf(spill_buf_, stream_);
        release_devbuf(kept_buf_, stream_);
        if (busy_ev_) (void)hipEventDestroy(busy_ev_);
    }

    // From now on every byte of device scratch (staged programs, saved accumulators, kept partial results)
    // comes out of [base, base + bytes), memory of the caller's; possible only before anything was staged.
    bool use_workspace(void *base, size_t bytes)
    {
        if (spill_ || kept_ || dev_prog_ || dev_extra_ || library_scratch_) return false;
        return ws_.make_static((char *)base, bytes);
    }

    // the staged programs and scratch this back end's launches refer to, for a caller that will replay them
    std::vector<Block *> detach_blocks()
    {
        dev_prog_ = nullptr;
        dev_extra_ = nullptr;
        dev_version_ = 0;
        chain_version_ = 0;
        chain_table_ = nullptr;
        chain_host_table_.clear();
        return ws_.detach();
    }
    size_t held_bytes() const { return ws_.held_bytes(); }

    // Adaptive sessions ask whether the stream has worked off what this session launched: an event
    // is recorded behind every launch from now on.
    void track_idle() { track_idle_ = true; }
    bool idle() override
    {
        if (!busy_recorded_) return true;
        if (hipEventQuery(busy_ev_) == hipSuccess) return true;
        (void)hipGetLastError();
        return false;
    }

    // everything enqueued on the session's stream from now on runs after `ev` has completed
    bool wait_for(hipEvent_t ev) { return hipStreamWaitEvent(stream_, ev, 0) == hipSuccess; }

    // Memory for the partial results kept for failure repair: one array of 4-byte accumulators per
    // partial, each as long as the object has elements, from the library's cache of device buffers.
    // Refused without the right to allocate, and beyond kMaxKeptBytes.
    bool keep_partials(int n_partials) override
    {
        if (kept_) return true;
        if (n_partials < 1 || shape_.object_bytes == 0 || library_scratch_) return false;
        // 4 bytes per element, in blocks for 64 source vectors each (see kept_offset in the device code)
        const size_t n_blocks = ((shape_.object_bytes + 15) / 16 + 63) / 64;
        kept_stride_ = n_blocks * 1024 * (size_t)(4 / elem_bytes(dtype_));
        if (kept_stride_ > kMaxKeptBytes / (size_t)n_partials) return false;
        if (ws_.is_static()) {
            // a caller's workspace: the kept arrays come out of it if they fit (else nothing is kept)
            if (kept_stride_ * (size_t)n_partials + 256 > ws_.static_left()) return false;
            kept_ = (char *)ws_.scratch(kept_stride_ * (size_t)n_partials);
            if (!kept_) return false;
        } else {
            if (ws_.capturing()) return false;          // a graph cannot own cached memory: nothing is kept
            kept_buf_ = acquire_devbuf(device_, kept_stride_ * (size_t)n_partials);
            if (!kept_buf_) return false;
            kept_ = kept_buf_->ptr;
        }
        n_kept_ = n_partials;
        return true;
    }

    int launch(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1, bool final,
               int live_before, int live_after) override
    {
        const int rc = launch_work(prog, version, c0, c1, t0, t1, final, live_before, live_after);
        if (rc >= 0 && track_idle_) {
            if (!busy_ev_ && hipEventCreateWithFlags(&busy_ev_, hipEventDisableTiming) != hipSuccess) return HOP_ERR_DEVICE;
            if (hipEventRecord(busy_ev_, stream_) != hipSuccess) return HOP_ERR_DEVICE;
            busy_recorded_ = true;
        }
        return rc;
    }

private:
    int launch_work(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1, bool final,
                    int live_before, int live_after)
    {
        if (shape_.object_bytes == 0) return HOP_OK;
        if (t0 > 0 || !final) return launch_segment(prog, c0, c1, t0, t1, final, live_before, live_after);
        for (const Entry &e : prog)
            if (e.obj < 0 || e.save >= 0) return launch_kept(prog, version, c0, c1);
        const size_t b0 = shape_.begin(c0), b1 = shape_.end(c1);
        if (wants_chains(prog.size(), b1 - b0)) {
            int rc = launch_chains(prog, version, b0, b1);
            if (rc != HOP_PARTIAL) {                // HOP_PARTIAL here = "no such form, use another path"
                if (rc < 0) return rc;
                return copy_to_other_destinations(b0, b1);
            }
        }
        if (wants_split(prog.size(), b1 - b0)) {
            int rc = launch_split(prog, b0, b1);
            if (rc != HOP_PARTIAL) {                // HOP_PARTIAL here = "not splittable, use the plain path"
                if (rc < 0) return rc;
                return copy_to_other_destinations(b0, b1);
            }
        }
        if (version != dev_version_) {
            staging_.resize(prog.size());
            depth_ = 1;
            for (size_t i = 0; i < prog.size(); ++i) {
                staging_[i] = resolve(prog[i], nullptr, 0, 0);
                depth_ = std::max(depth_, (int)prog[i].level + 1);
            }
            mark_runs(staging_.data(), staging_.size());
            dev_prog_ = nullptr;
            if ((int)staging_.size() > kInlineEntries) {      // short programs ride in the kernel arguments
                dev_prog_ = (const DevEntry *)ws_.stage(staging_.data(), staging_.size() * sizeof(DevEntry));
                if (!dev_prog_) return ws_.error();
            }
            dev_version_ = version;
        }
        // Storing to all destinations from the reduce kernel itself was measured slower than a reduce into
        // the first one followed by the copy (reads and 64-way writes interleaved: 492 us against 391 us
        // on 64 x 16 MiB).
        hipError_t e = launch_reduce(stream_, dtype_, op_, depth_, staging_.data(), dev_prog_, (int)prog.size(),
                                     dsts_[0], b0, b1);
        if (e != hipSuccess) return HOP_ERR_DEVICE;
        return copy_to_other_destinations(b0, b1);
    }

private:
    // Reduce followed by broadcast, chunk run by chunk run: the finished chunks have landed in the first
    // destination and the copy kernel carries them to the others while they are still cache-resident. Up
    // to kInlineDsts other destinations ride in the kernel arguments; more are staged once per call.
    int copy_to_other_destinations(size_t b0, size_t b1)
    {
        if (dsts_.size() < 2) return HOP_OK;
        const int n_other = (int)dsts_.size() - 1;
        if (n_other > kInlineDsts && !dev_extra_) {
            dev_extra_ = (void *const *)ws_.stage(dsts_.data() + 1, (size_t)n_other * sizeof(void *));
            if (!dev_extra_) return ws_.error();
        }
        const hipError_t e = launch_copy(stream_, dsts_[0], dev_extra_, n_other, b0, b1, nullptr, extra_residue_, dsts_.data() + 1);
        return e == hipSuccess ? HOP_OK : HOP_ERR_DEVICE;
    }

    // Steps [t0, t1) only: accumulators come from and/or go to the spill area, one array of 4-byte
    // accumulators per level, each as long as the object has elements. It is taken from the
    // library's cache when the first partial segment is launched and returned with the session.
    int launch_segment(const std::vector<Entry> &prog, int64_t c0, int64_t c1, int t0, int t1, bool final,
                       int live_before, int live_after)
    {
        const size_t b0 = shape_.begin(c0), b1 = shape_.end(c1);
        if (!spill_) {
            const size_t n_elems = shape_.object_bytes / (size_t)elem_bytes(dtype_);
            level_stride_ = (n_elems * 4 + 255) & ~(size_t)255;
            spill_levels_ = std::min(HOP_MAX_DEPTH, full_tree_depth(k_, degree_));
            if (ws_.is_static()) {
                // the library's own static scratch never holds object-sized arrays; a caller's workspace does
                if (library_scratch_) return HOP_ERR_TOO_LARGE;
                spill_ = (char *)ws_.scratch(level_stride_ * (size_t)spill_levels_);
                if (!spill_) return ws_.error();
            } else {
                if (ws_.capturing()) return ws_.error();
                spill_buf_ = acquire_devbuf(device_, level_stride_ * (size_t)spill_levels_);
                if (!spill_buf_) return HOP_ERR_NOMEM;
                spill_ = spill_buf_->ptr;
            }
        }
        int depth = 1;
        std::vector<DevEntry> steps((size_t)(t1 - t0));
        for (int t = t0; t < t1; ++t) {
            steps[(size_t)(t - t0)] = resolve(prog[(size_t)t], nullptr, 0, 0);
            depth = std::max(depth, (int)prog[(size_t)t].level + 1);
        }
        depth = std::max(depth, std::max(live_before, live_after));
        if (depth > spill_levels_) return HOP_ERR_DEPTH;
        const DevEntry *dev_steps = nullptr;           // t0 == t1: only move saved accumulators to the result
        if (!steps.empty()) {
            dev_steps = (const DevEntry *)ws_.stage(steps.data(), steps.size() * sizeof(DevEntry));
            if (!dev_steps) return ws_.error();
        }
        hipError_t e = launch_reduce_segment(stream_, dtype_, op_, depth, dev_steps, t1 - t0, dsts_[0], spill_,
                                             level_stride_, live_before, final ? 0 : live_after, b0, b1,
                                             steps.empty() ? 0 : lead_vectors(steps.data(), (int)steps.size(), b0));
        if (e != hipSuccess) return HOP_ERR_DEVICE;
        return final ? copy_to_other_destinations(b0, b1) : HOP_OK;
    }

    // A whole program some of whose steps read a kept partial result (obj = -(1 + q)) or store one
    // (save = q): the repair of a failure and the launches that prepare for one.
    static constexpr size_t kMaxKeptBytes = (size_t)16 << 30;

    int launch_kept(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1)
    {
        if (!kept_) return HOP_ERR_NOMEM;               // keep_partials was not asked, or said no
        const size_t b0 = shape_.begin(c0), b1 = shape_.end(c1);
        if (version != kept_version_) {
            kept_steps_.resize(prog.size());
            kept_depth_ = 1;
            for (size_t i = 0; i < prog.size(); ++i) {
                const Entry &e = prog[i];
                if (e.obj < 0 && -e.obj - 1 >= n_kept_) return HOP_ERR_INVALID;
                if (e.save >= n_kept_ || e.save_level > e.level) return HOP_ERR_INVALID;
                DevEntry d;
                d.src = e.obj >= 0 ? objs_[e.obj] : (const void *)(kept_ + (size_t)(-e.obj - 1) * kept_stride_);
                d.ctl = (uint32_t)e.level | ((uint32_t)e.set << 8) | ((uint32_t)e.n_fold << 16) | (e.obj < 0 ? kPartialBit : 0u);
                d.aux = e.save >= 0 ? ((uint32_t)e.save + 1u) | ((uint32_t)e.save_level << 16) : 0u;
                kept_steps_[i] = d;
                kept_depth_ = std::max(kept_depth_, (int)e.level + 1);
            }
            kept_dev_ = nullptr;
            if ((int)kept_steps_.size() > kInlineEntries) {       // short programs ride in the kernel arguments
                kept_dev_ = (const DevEntry *)ws_.stage(kept_steps_.data(), kept_steps_.size() * sizeof(DevEntry));
                if (!kept_dev_) return ws_.error();
            }
            kept_version_ = version;
        }
        hipError_t e = launch_reduce_kept(stream_, dtype_, op_, kept_depth_, kept_steps_.data(), kept_dev_, (int)prog.size(),
                                          dsts_[0], kept_, kept_stride_, b0, b1);
        if (e != hipSuccess) return HOP_ERR_DEVICE;
        return copy_to_other_destinations(b0, b1);
    }

    // Many inputs but few output tiles (the many-small-objects case): one wave per tile would walk
    // the whole program alone, so the independent subtrees are evaluated side by side first.
    // Partials are stored in the accumulation type, which for bf16 is not the element type: its
    // sub-programs store 4-byte accumulators in the layout of a kept partial result, and the steps that
    // read them say so (kernels instantiated for that: launch_reduce_subs and launch_reduce with mixed).
    // Measured (fp32 sums, 16-ary tree, inputs not in any cache): a wave that walks
    // a program alone takes about 0.15 us per step whatever the range, so the cut pays while that is more
    // than the time to stream the range - up to about 768 KiB: 4000 inputs of 256 KiB 212 us against 620
    // for the plain path, 1000 inputs of 1 MiB 212 us against 186. bf16, cut against plain: 128 inputs of 72 KiB
    // 15.1 against 21.9, of 512 KiB 22.8 against 24.2, of 768 KiB 32.3 against 25.5; 512 inputs of 128 KiB 27.0
    // against 81.4, of 768 KiB 90.9 against 99.5; 1000 of 256 KiB 76.7 against 185; 4000 of 128 KiB 125 against 792.

    bool wants_split(size_t n_steps, size_t range_bytes) const
    {
        return n_steps >= kSplitWantSteps && range_bytes <= split_max_bytes(dtype_);
    }

    int launch_split(const std::vector<Entry> &prog, size_t b0, size_t b1)
    {
        MultiPlan mp;
        if (!plan_passes(prog, kSplitWantSteps, kSplitMinRun, kSplitMaxRun, mp)) return HOP_PARTIAL;
        const bool mixed = dtype_ == HOP_BF16;
        const size_t part_bytes = split_partial_bytes(dtype_, b0, b1), part_off = split_partial_base_offset(dtype_, b0);
        const size_t n_subs = mp.n_subs();
        if (part_bytes * n_subs > kSplitMaxScratch || n_subs > 65535) return HOP_PARTIAL;
        // partials, then every sub-program as a record of equal length per pass: from one block
        struct PassInfo { size_t records_at; int sub_entries, n_subs, depth; };
        std::vector<PassInfo> passes(mp.n_passes, PassInfo{0, 2, 0, 1});
        for (size_t g = 0; g < n_subs; ++g) {
            PassInfo &pi = passes[(size_t)mp.height[g]];
            pi.sub_entries = std::max(pi.sub_entries, (int)(mp.begin[g + 1] - mp.begin[g]) + 1);
            pi.depth = std::max(pi.depth, (int)mp.depth[g]);
            pi.n_subs++;
        }
        size_t n_blob = mp.top.size();
        for (const PassInfo &pi : passes) {
            if (pi.sub_entries > kMaxSubSteps + 1) return HOP_PARTIAL;
            n_blob += (size_t)pi.sub_entries * (size_t)pi.n_subs;
        }
        const size_t need = part_bytes * n_subs + n_blob * sizeof(DevEntry) + 512;
        // without the right to allocate, a cut that does not fit beside the whole program (which the
        // plain path then has to stage) is not made
        if (ws_.is_static() && need + prog.size() * sizeof(DevEntry) + 256 > ws_.static_left()) return HOP_PARTIAL;
        if (!ws_.reserve(need)) return ws_.error();
        char *partials = (char *)ws_.scratch(part_bytes * n_subs);
        if (!partials) return ws_.error();
        // Kernels address sources and results by the object's byte offset, so a partial that holds
        // only [b0, b1) is passed as base - b0 (bf16: less the offset of b0's block of accumulators). Passes run in stream order: pass h reads what
        // passes < h wrote.
        // All passes' records, then the top program, travel in one copy.
        std::vector<DevEntry> blob;
        blob.reserve(n_blob);
        for (int pass = 0; pass < mp.n_passes; ++pass) {
            PassInfo &pi = passes[(size_t)pass];
            pi.records_at = blob.size();
            for (size_t g = 0; g < n_subs; ++g) {
                if (mp.height[g] != pass) continue;
                const size_t rec_at = blob.size();
                SubHeader h;
                h.dst = (void *)((uintptr_t)partials + g * part_bytes - part_off);
                h.n_entries = (uint32_t)(mp.begin[g + 1] - mp.begin[g]);
                h.flags = mixed ? kSubStoresAccumulators : 0u;
                DevEntry raw;
                std::memcpy(&raw, &h, sizeof raw);
                blob.push_back(raw);
                for (int32_t t = mp.begin[g]; t < mp.begin[g + 1]; ++t)
                    blob.push_back(resolve(mp.steps[(size_t)t], partials, part_bytes, part_off, mixed));
                mark_runs(blob.data() + rec_at + 1, blob.size() - rec_at - 1);
                blob.resize(rec_at + (size_t)pi.sub_entries, DevEntry{nullptr, 0, 0});
            }
        }
        const size_t top_at = blob.size();
        for (const Entry &e : mp.top) blob.push_back(resolve(e, partials, part_bytes, part_off, mixed));
        mark_runs(blob.data() + top_at, blob.size() - top_at);
        const DevEntry *dev = (const DevEntry *)ws_.stage_in_place(blob.data(), blob.size() * sizeof(DevEntry));
        if (!dev) return ws_.error();
        for (const PassInfo &pi : passes) {
            // the first pass reads objects only: the kernel without the registers for partial results does
            const bool reads_partials = mixed && &pi != &passes[0];
            if (launch_reduce_subs(stream_, dtype_, op_, pi.depth, dev + pi.records_at, pi.sub_entries, pi.n_subs, b0,
                                   b1, reads_partials) != hipSuccess)
                return HOP_ERR_DEVICE;
        }
        hipError_t e = launch_reduce(stream_, dtype_, op_, mp.top_depth, blob.data() + top_at, dev + top_at,
                                     (int)mp.top.size(), dsts_[0], b0, b1, mixed);
        return e == hipSuccess ? HOP_OK : HOP_ERR_DEVICE;
    }

    // Many inputs and a byte range so short that it gives at most a thousand 64-byte columns: one launch
    // in which every column's workgroup evaluates the program as chains, up to 64 of them side by side,
    // their values in LDS (no second launch, no partials in memory; the values are accumulator-typed,
    // so bf16 takes this path too). Measured on fp32 sums in a 16-ary tree, inputs not in any cache,
    // against the other paths, us per call: 128 inputs of 1-64 KiB 8.0-8.5 against 10.7-11.3; 1000 inputs of
    // 1-16 KiB 9.0-9.5 against 18.8-21.6, of 64 KiB 25.3 against 27.3; 4000 inputs of 1-16 KiB 15.5-23.5
    // against 19.6-33.6. It loses where the workgroups no longer run side by side (a workgroup is bound by
    // the latency of its few loads): 256 inputs of 256 KiB 28.8 against 19.3, 4000 of 64 KiB 109 against 67.
    // Hence the limit on columns x rounds, a round being 64 chains of one pass. (With each die's workgroups on
    // columns in a row, see chains_workgroup: 1000 inputs of 64 KiB 17.6, 4000 of 16 KiB 17.1, 256 of 64 KiB 8.8;
    // the same limits still came out best: 4000 of 64 KiB 72.8 as chains against 63.5, 4000 of 32 KiB 39.7
    // as chains against 44.5.)

    //
    // The wide form (a whole wave per chain, 1 KiB columns, 8 chains side by side) takes over above 64 KiB:
    // every load instruction then covers 1 KiB of one object, as in the streaming kernels, and a range of
    // 256 KiB is 256 workgroups instead of 4096. One launch where the cut into sub-programs needs two or
    // three, and no partial results in memory. fp32 sums, 16-ary tree, cold inputs, us per call, wide form
    // against the cut: 128 inputs of 128 KiB 8.4 / 12.8, of 256 KiB 8.4 / 14.1; 256 of 256 KiB 13.3 / 19.3;
    // 1000 of 128 KiB 34.6 / 38.7, of 256 KiB 48.5 / 59.9; 512 of 512 KiB 52.5 / 59.5; 128 / 256 / 512 / 1000 of
    // 768 KiB 25.8 / 42.1 / 76.9 / 139 against 29.5 / 46.4 / 84.1 / 156; at 1 MiB per object it loses against the
    // plain path (128 inputs: 32.9 / 24.3) or draws (256, 1000 inputs). bf16: 128 of 128 KiB 9.6 / 15.1, 256 of
    // 256 KiB 16.9 / 23.2, of 512 KiB 35.2 / 40.4. Programs with more values alive at one time than the LDS
    // holds (128 KiB: 127 of 1 KiB, bf16: 63 of 2 KiB; thousands of inputs) have no such form and are cut as before
    // (with 128 KiB instead of 64: fp32 2000 of 256 KiB 93 against 108, bf16 1000 of 256 KiB 54.2 against 79.5).

    bool wants_chains(size_t n_steps, size_t range_bytes) const
    {
        return n_steps >= kChainWantSteps && range_bytes <= kChainWideMaxBytes;
    }

    // bf16 from 32 KiB for programs of up to 384 steps: 128 / 256 inputs of 64 KiB 8.8 / 12.1 us wide against
    // 14.9 / 15.5 narrow (1000 inputs: 42.1 against 26.6; at 32 KiB the narrow form wins or draws for every count)
    bool takes_wide_form(size_t n_steps, size_t range_bytes) const
    {
        return range_bytes > kChainMaxBytes ||
               (dtype_ == HOP_BF16 && range_bytes > kChainWideEarlyBytes && n_steps <= kChainWideEarlySteps);
    }

    int launch_chains(const std::vector<Entry> &prog, uint64_t version, size_t b0, size_t b1)
    {
        const bool wide = takes_wide_form(prog.size(), b1 - b0);
        if (version != chain_version_ || wide != skeleton_.wide) {
            // the plan is made once per program and form; the table only when a launch is short enough to use it
            chain_version_ = version;
            chain_table_ = nullptr;
            chain_host_table_.clear();
            chain_usable_ = build_skeleton(prog, wide, skeleton_);
        }
        if (!chain_usable_) return HOP_PARTIAL;
        const int rc = launch_skeleton(skeleton_, b0, b1);
        if (rc == HOP_OK) ++chain_launches_;
        return rc;
    }

    bool build_skeleton(const std::vector<Entry> &prog, bool wide, ChainSkeleton &sk) const
    {
        ChainFormat f;
        f.min_cut = kChainMinCut;
        f.max_items = kChainMaxItems;
        f.record_words = kChainRecordWords;
        f.teams = wide ? kChainWideTeams : kChainTeams;
        f.max_passes = kMaxChainPasses;
        f.value_bytes = chain_value_bytes(dtype_, wide);
        f.max_values = chain_slots_max(dtype_, wide);
        f.result_mark = kChainFinal;
        const bool ok = build_chain_skeleton(prog, f, sk);
        sk.wide = wide;
        return ok;
    }

public:
    // One launch of a skeleton over [b0, b1) of this back end's objects: their addresses go into a copy of
    // the table, which is staged once per back end. HOP_PARTIAL if the launch is too long for this form
    // or an address cannot be told from a value's offset.
    int launch_skeleton(const ChainSkeleton &sk, size_t b0, size_t b1)
    {
        if (sk.wide) {
            if (!takes_wide_form(sk.n_steps, b1 - b0) || b1 - b0 > kChainWideMaxBytes) return HOP_PARTIAL;
        } else {
            const size_t columns = (b1 - b0 + 16 * kChainLanes - 1) / (16 * kChainLanes);
            if (b1 - b0 > kChainMaxBytes || columns * sk.rounds > kChainMaxWork) return HOP_PARTIAL;
        }
        if (!chain_table_ && chain_host_table_.empty()) {
            std::vector<uint64_t> table(sk.table);
            for (uint64_t &word : table) {
                if (!(word & kSkeletonObject)) continue;
                const size_t index = (size_t)(word & ~kSkeletonObject);
                if (index >= objs_.size()) return HOP_ERR_INVALID;
                word = (uint64_t)(uintptr_t)objs_[index];
                if ((word >> 32) == 0) return HOP_PARTIAL;         // would read as a value's offset
            }
            chain_host_table_.swap(table);
        }
        // a table of up to 256 chains rides in the kernel arguments; a longer one (or any, once the runtime has
        // refused such arguments) is staged once per back end
        for (int attempt = 0; attempt < 2; ++attempt) {
            const bool inl = chain_table_inline(sk.n_chains);
            if (!inl && !chain_table_) {
                // without the right to allocate, a table that does not fit beside the whole program (which the
                // plain path then has to stage) is not made
                const size_t bytes = chain_host_table_.size() * sizeof(uint64_t);
                if (ws_.is_static() && bytes + sk.n_steps * sizeof(DevEntry) + 512 > ws_.static_left()) return HOP_PARTIAL;
                chain_table_ = (const uint64_t *)ws_.stage(chain_host_table_.data(), bytes);
                if (!chain_table_) return ws_.error();
            }
            const hipError_t e = launch_reduce_chains(stream_, dtype_, op_, chain_table_, sk.n_chains, sk.n_slots,
                                                      sk.pass_begin.data(), (int)sk.pass_begin.size() - 1, dsts_[0], b0, b1,
                                                      inl ? chain_host_table_.data() : nullptr, sk.wide);
            if (e == hipSuccess) return HOP_OK;
            if (sk.wide && ((size_t)sk.n_slots + 1) * chain_value_bytes(dtype_, true) > kChainLdsBytes) {
                // a workgroup was refused that much LDS (the launcher asks for less from now on): another path
                (void)hipGetLastError();
                chain_usable_ = false;
                return HOP_PARTIAL;
            }
            if (!inl || chain_table_inline(sk.n_chains)) return HOP_ERR_DEVICE;
            (void)hipGetLastError();                               // refused as arguments: once more, staged
        }
        return HOP_ERR_DEVICE;
    }
    // the copy of [b0, b1) of the first destination to the others, for a caller that launched the reduce itself
    int copy_rest(size_t b0, size_t b1) { return copy_to_other_destinations(b0, b1); }
    // The skeleton of the program in force if every launch so far was one launch of it (a failure-free call
    // over many small objects), else null.
    const ChainSkeleton *sole_skeleton(int n_launches) const
    {
        return chain_usable_ && chain_launches_ == n_launches && n_launches > 0 ? &skeleton_ : nullptr;
    }

private:
    // partial q of a cut program lies at partials + q * part_bytes, and the kernels address it from part_off
    // bytes in front of that; partial_bit: its values are accumulators, not elements (bf16)
    DevEntry resolve(const Entry &e, const char *partials, size_t part_bytes, size_t part_off, bool partial_bit = false) const
    {
        DevEntry d;
        d.src = e.obj >= 0 ? objs_[e.obj]
                           : (const void *)((uintptr_t)partials + (size_t)(-e.obj - 1) * part_bytes - part_off);
        d.ctl = (uint32_t)e.level | ((uint32_t)e.set << 8) | ((uint32_t)e.n_fold << 16) |
                (e.obj < 0 && partial_bit ? kPartialBit : 0u);
        d.aux = 0;
        return d;
    }

    Workspace ws_;
    hipStream_t stream_;
    std::vector<const void *> objs_;
    std::vector<void *> dsts_;
    Shape shape_;
    int op_, dtype_, k_;
    int64_t degree_;
    std::vector<DevEntry> staging_;
    const DevEntry *dev_prog_ = nullptr;
    void *const *dev_extra_ = nullptr;
    unsigned extra_residue_ = 0;                // address modulo 128 shared by (most of) the other destinations
    uint64_t dev_version_ = 0;
    uint64_t chain_version_ = 0;                // the program whose one-launch form skeleton_ is
    const uint64_t *chain_table_ = nullptr;     // its table with this back end's objects, staged (null: not yet, or not needed)
    std::vector<uint64_t> chain_host_table_;    // the same in host memory
    ChainSkeleton skeleton_;
    bool chain_usable_ = false;
    int chain_launches_ = 0;
    int depth_ = 1;
    int device_;
    DevBuf *spill_buf_ = nullptr;
    char *spill_ = nullptr;
    size_t level_stride_ = 0;
    int spill_levels_ = 0;
    hipEvent_t busy_ev_ = nullptr;
    bool busy_recorded_ = false, track_idle_ = false;
    bool library_scratch_ = false;              // all scratch from the library's small static array (hop_reduce_noalloc)
    DevBuf *kept_buf_ = nullptr;                // partial results kept for failure repair
    char *kept_ = nullptr;
    size_t kept_stride_ = 0;
    int n_kept_ = 0;
    std::vector<DevEntry> kept_steps_;
    const DevEntry *kept_dev_ = nullptr;
    uint64_t kept_version_ = 0;
    int kept_depth_ = 1;
};

class RecordingBackend : public Backend {
public:
    int launch(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1, bool final,
               int live_before, int live_after) override
    {
        if (version != version_) {
            entry_begin_ = (int32_t)entries.size();
            entries.insert(entries.end(), prog.begin(), prog.end());
            version_ = version;
        }
        hop_plan_launch_t l;
        l.chunk_begin = c0;
        l.chunk_end = c1;
        l.entry_begin = entry_begin_;
        l.entry_end = (int32_t)(entry_begin_ + prog.size());
        l.step_begin = t0;
        l.step_end = t1;
        l.final = final ? 1 : 0;
        l.live_before = live_before;
        l.live_after = live_after;
        l.reserved = 0;
        launches.push_back(l);
        return HOP_OK;
    }
    std::vector<Entry> entries;
    std::vector<hop_plan_launch_t> launches;

private:
    uint64_t version_ = 0;
    int32_t entry_begin_ = 0;
};

}  // namespace hop
