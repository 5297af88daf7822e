// Host-side chunk scheduler of the MI355X reduce library: tree shape, slot
// assignment by arrival, per-chunk readiness, failure repair, and the
// translation of the tree into a flat accumulator program for the kernels.
// No HIP in this file: it is driven either by the GPU back end (hop_api.hip)
// or by a recording back end (hop_plan_reduce) that enqueues nothing.
//
// Paper passages: dynamic d-ary tree and in-order placement of arrivals,
// subset reduce (section 3.4.2); chunk-granular pipelining (section 3.3);
// removal and in-place replacement of a failed participant (section 3.5.2).
#pragma once

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>
#include <set>
#include <vector>

#include "../../include/hop.h"

namespace hop {

// One step of the per-element accumulator program (same meaning as
// hop_plan_entry_t): read the element of object `obj`, start or extend the
// partial result at `level`, then fold `n_fold` finished partials downwards.
//
// Two extensions serve the repair of failures (section 3.5.2: partial results that do not
// contain the failed object are kept). obj = -(1 + q) reads kept partial q, an array of
// accumulator-typed values, instead of an object. save = q >= 0: once the step's value is combined
// and the folds have come down to save_level, acc[save_level] is also stored as kept partial q;
// the remaining folds follow.
struct Entry {
    int32_t obj;
    uint8_t level;
    uint8_t set;
    uint16_t n_fold;
    int16_t save = -1;
    uint8_t save_level = 0;
    uint8_t reserved = 0;
};

// Complete d-ary tree on k nodes in level order; node_of_slot[t] is the node
// that the t-th arrival takes (generalised in-order traversal, section 3.4.2).
struct Tree {
    int k = 0;
    int64_t d = 1;
    std::vector<int32_t> node_of_slot, slot_of_node;

    int64_t child(int64_t j, int64_t c) const {
        int64_t x = d * j + c;
        return (x < k) ? x : -1;
    }

    // shape only: enough for compile_program, which walks the tree itself
    void shape(int k_, int64_t d_) { k = k_; d = d_; }

    void build(int k_, int64_t d_) {
        k = k_;
        d = d_;
        node_of_slot.assign(k, -1);
        slot_of_node.assign(k, -1);
        // Explicit stack: (node, next child to descend into). A chain (d = 1)
        // is k levels deep, so recursion is avoided.
        struct Frame { int64_t node; int64_t next; bool visited; };
        std::vector<Frame> st;
        st.push_back({0, 1, false});
        int t = 0;
        while (!st.empty()) {
            Frame &f = st.back();
            if (f.next == 1) {                       // first child's subtree comes first
                f.next = 2;
                int64_t c1 = child(f.node, 1);
                if (c1 >= 0) { st.push_back({c1, 1, false}); continue; }
            }
            if (!f.visited) {                        // then the node itself
                f.visited = true;
                node_of_slot[t] = (int32_t)f.node;
                slot_of_node[f.node] = t;
                ++t;
            }
            int64_t c = (f.next <= d) ? child(f.node, f.next) : -1;
            if (c >= 0) {                            // then children 2..d, left to right
                f.next++;
                st.push_back({c, 1, false});
                continue;
            }
            st.pop_back();
        }
    }
};

// Flattens the tree expression over the current occupants (-1 = empty
// position, contributes nothing; -2 = position not taken yet, shapes the
// program like an object) into accumulator steps. A node combines,
// left to right, [first child's partial, its own object, other children's
// partials]; the first child's partial is built in the parent's own
// accumulator, every later child that has children of its own in the next
// level and folded in when done, a later child without children (one object)
// is combined into the parent's accumulator at once.
// Returns the number of accumulator levels used (0 if nobody is in the tree).
// slot_of_step (may be null) receives, per step, the tree position (arrival rank) whose occupant it reads.
inline int compile_program(const Tree &tr, const std::vector<int32_t> &occupant, std::vector<Entry> &out,
                           std::vector<int32_t> *slot_of_step = nullptr)
{
    out.clear();
    if (slot_of_step) slot_of_step->clear();
    const int k = tr.k;
    const int64_t d = tr.d;
    if (d == 1 || k == 1) {
        // chain: plain left fold in arrival order
        for (int t = 0; t < k; ++t) {
            if (occupant[t] == -1) continue;
            out.push_back({occupant[t], 0, (uint8_t)out.empty(), 0});
            if (slot_of_step) slot_of_step->push_back(t);
        }
        return out.empty() ? 0 : 1;
    }
    // d >= 2: height <= log2(k), recursion is shallow. The walk is the in-order traversal
    // itself, so the next position in arrival order is simply a running counter. Most nodes
    // of a wide tree are leaves: they are emitted without a call.
    out.resize((size_t)k);
    if (slot_of_step) slot_of_step->resize((size_t)k);
    struct Walk {
        const int k; const int64_t d; const int32_t *occ; Entry *out; int n_out; int depth; int slot; int32_t *slots;
        void emit(const Entry &e) {
            if (slots) slots[n_out] = slot - 1;          // the position just read
            out[n_out++] = e;
        }
        bool leaf(int level) {
            const int32_t o = occ[slot++];
            if (o == -1) return false;
            emit(Entry{o, (uint8_t)level, 1, 0});
            if (level + 1 > depth) depth = level + 1;
            return true;
        }
        bool is_leaf(int64_t j) const { return d * j + 1 >= k; }
        bool node(int64_t j, int level) {
            bool started = false;
            const int64_t c1 = d * j + 1;
            if (c1 < k) started = is_leaf(c1) ? leaf(level) : node(c1, level);
            const int32_t o = occ[slot++];
            if (o != -1) {                    // an object, or a position still to be taken
                emit(Entry{o, (uint8_t)level, (uint8_t)!started, 0});
                if (level + 1 > depth) depth = level + 1;
                started = true;
            }
            for (int64_t c = 2; c <= d; ++c) {
                const int64_t ch = d * j + c;
                if (ch >= k) break;
                if (!started) {
                    started = is_leaf(ch) ? leaf(level) : node(ch, level);
                } else if (is_leaf(ch)) {
                    // a lone object joins its parent's partial directly: the same arithmetic as
                    // starting a partial of its own in the next level and folding it at once
                    const int32_t o = occ[slot++];
                    if (o != -1) emit(Entry{o, (uint8_t)level, 0, 0});
                } else if (node(ch, level + 1)) {     // at most log2(k) < 32 levels
                    out[n_out - 1].n_fold++;
                }
            }
            return started;
        }
    } w{k, d, occupant.data(), out.data(), 0, 0, 0, slot_of_step ? slot_of_step->data() : nullptr};
    w.node(0, 0);
    out.resize((size_t)w.n_out);
    if (slot_of_step) slot_of_step->resize((size_t)w.n_out);
    return w.depth;
}

// A long program cut into short independent ones. Every `set` step above level 0
// opens a run that ends at the step whose folds return below the run's level: a
// non-first-child subtree of the tree, an independent sub-expression. Cutting
// works bottom-up: every outermost run of min_run..max_run steps becomes a
// sub-program of its own (its steps with levels counted from the run's level,
// the fold out of the run dropped); in the program it came from, one step
// replaces it that combines the sub-program's stored partial into the level
// below - the same arithmetic as the dropped fold - and carries the folds that
// went further down. If what is left still has want_steps steps or more, it is
// cut again the same way (its runs now contain partials of the first cut), and
// so on: a tree of any depth becomes a few passes of many short programs. Pass
// h evaluates side by side all sub-programs cut in round h, which read only
// objects and partials of earlier passes; the top program comes last.
struct MultiPlan {
    std::vector<Entry> steps;                    // all sub-programs: sub g = steps[begin[g], begin[g + 1])
    std::vector<int32_t> begin;                  // n_subs() + 1 offsets
    std::vector<int32_t> height, depth;          // per sub-program: pass it runs in, accumulator levels
    std::vector<Entry> top;                      // obj >= 0: object; obj = -(1 + g): partial of sub-program g
    int top_depth = 0;
    int n_passes = 0;
    size_t n_subs() const { return height.size(); }
};

inline int program_depth(const std::vector<Entry> &p)
{
    int d = 0;
    for (const Entry &e : p) d = std::max(d, (int)e.level + 1);
    return d;
}

// Returns false (top = prog, no sub-programs) if nothing was cut or the program is malformed.
inline bool plan_passes(const std::vector<Entry> &prog, size_t want_steps, int min_run, int max_run, MultiPlan &mp)
{
    mp = MultiPlan();
    auto whole = [&]() {
        mp = MultiPlan();
        mp.top = prog;
        mp.top_depth = program_depth(prog);
        return false;
    };
    if (min_run < 1) min_run = 1;
    if (max_run < min_run) return whole();
    std::vector<Entry> cur(prog), next;
    std::vector<int32_t> run_end;
    mp.begin.push_back(0);
    for (int pass = 0; cur.size() >= want_steps && !cur.empty(); ++pass) {
        const int n = (int)cur.size();
        // where every run ends: at most one run is open per level at any time
        run_end.assign((size_t)n, -1);
        int32_t open[256];
        for (int l = 0; l < 256; ++l) open[l] = -1;
        for (int i = 0; i < n; ++i) {
            const Entry &e = cur[(size_t)i];
            if (e.n_fold > e.level) return whole();
            if (e.level >= 1) {
                if (e.set) {
                    if (open[e.level] >= 0) return whole();
                    open[e.level] = i;
                } else if (open[e.level] < 0) return whole();
            }
            for (int f = 0; f < (int)e.n_fold; ++f) {
                const int l = (int)e.level - f;
                if (open[l] < 0) return whole();
                run_end[(size_t)open[l]] = i;
                open[l] = -1;
            }
        }
        for (int l = 0; l < 256; ++l)
            if (open[l] >= 0) return whole();
        // outermost runs of suitable length leave; the rest stays, nested runs looked at in turn
        next.clear();
        next.reserve((size_t)n);
        bool any = false;
        for (int i = 0; i < n;) {
            const Entry &e = cur[(size_t)i];
            const int len = (e.set && e.level >= 1) ? run_end[(size_t)i] - i + 1 : 0;
            if (len < min_run || len > max_run) {
                next.push_back(e);
                ++i;
                continue;
            }
            const int base = e.level, end = run_end[(size_t)i];
            const int32_t g = (int32_t)mp.height.size();
            int depth = 1;
            for (int t = i; t <= end; ++t) {
                const Entry &x = cur[(size_t)t];
                const int rel = (int)x.level - base;
                mp.steps.push_back(Entry{x.obj, (uint8_t)rel, x.set, (uint16_t)std::min((int)x.n_fold, rel)});
                depth = std::max(depth, rel + 1);
            }
            const Entry &last = cur[(size_t)end];
            const int beyond = (int)last.n_fold - ((int)last.level - base) - 1;      // folds below the run's parent level
            next.push_back(Entry{-(1 + g), (uint8_t)(base - 1), 0, (uint16_t)beyond});
            mp.begin.push_back((int32_t)mp.steps.size());
            mp.height.push_back(pass);
            mp.depth.push_back(depth);
            mp.n_passes = pass + 1;
            any = true;
            i = end + 1;
        }
        if (!any) break;
        cur.swap(next);
    }
    if (mp.height.empty()) return whole();
    mp.top.swap(cur);
    mp.top_depth = program_depth(mp.top);
    return true;
}

// A program as chains: the form in which ONE workgroup can evaluate a long program over a narrow
// column of the objects with many lanes side by side. A chain is a left fold, value = item 0 (op)
// item 1 (op) ... in that order, of objects and of the values of other chains; the value of the
// last chain is the program's result. Every accumulator level of the program is such a fold: the
// steps that combine into it, and, where a fold of the level above lands in it, that level's value.
// A chain is cut where it first needs a value that is ready later than everything it holds so far
// (if it holds at least min_cut items by then): the front part becomes a chain of its own, evaluated
// earlier, and the rest starts from its value - the same arithmetic, since a chain's value is kept
// in the accumulation type. A chain that reaches max_items items is cut the same way (a long fold
// has no independent parts: its pieces follow each other, one pass each). pass[g] = 0 if chain g reads only objects, else 1 + the largest pass of
// the chains it reads: all chains of a pass are independent of each other.
struct ChainPlan {
    std::vector<int32_t> items;                  // obj >= 0: object; -(1 + g): value of chain g
    std::vector<int32_t> begin;                  // chain g = items[begin[g], begin[g + 1])
    std::vector<int32_t> pass;
    int n_passes = 0;
    int64_t critical_steps = 0;                  // items on the longest path: sum over passes of the longest chain
    size_t n_chains() const { return pass.size(); }
};

// Returns false if the program is malformed, reads kept partial results, or is a single object.
inline bool plan_chains(const std::vector<Entry> &prog, int min_cut, int max_items, ChainPlan &cp)
{
    cp = ChainPlan();
    if (max_items < 2) return false;
    cp.begin.push_back(0);
    struct Open {
        std::vector<int32_t> items;
        int avail = 0;                           // pass before which nothing of `items` is missing
    };
    int depth = 1;
    for (const Entry &e : prog) depth = std::max(depth, (int)e.level + 1);
    std::vector<Open> open((size_t)depth);
    cp.items.reserve(prog.size() + prog.size() / 2);
    cp.begin.reserve(prog.size() / 2 + 2);
    cp.pass.reserve(prog.size() / 2 + 1);
    auto avail_of = [&](int32_t item) { return item >= 0 ? 0 : cp.pass[(size_t)(-item - 1)] + 1; };
    auto emit = [&](Open &o) {
        const int32_t g = (int32_t)cp.pass.size();
        cp.items.insert(cp.items.end(), o.items.begin(), o.items.end());
        cp.begin.push_back((int32_t)cp.items.size());
        cp.pass.push_back(o.avail);
        return -(1 + g);
    };
    auto add = [&](Open &o, int32_t item) {
        const int a = avail_of(item);
        if ((a > o.avail && (int)o.items.size() >= std::max(min_cut, 2)) || (int)o.items.size() >= max_items) {
            const int32_t front = emit(o);
            o.items.assign(1, front);
            o.avail = avail_of(front);
        }
        o.items.push_back(item);
        o.avail = std::max(o.avail, a);
    };
    auto close = [&](Open &o) {                  // the level's value as one item
        const int32_t item = o.items.size() == 1 ? o.items[0] : emit(o);
        o.items.clear();
        o.avail = 0;
        return item;
    };
    for (const Entry &e : prog) {
        if (e.obj < 0 || e.save >= 0 || e.n_fold > e.level) return false;
        Open &o = open[e.level];
        if (e.set != o.items.empty()) return false;      // a level starts with set and only then
        add(o, e.obj);
        for (int f = 0; f < (int)e.n_fold; ++f) {
            const int l = (int)e.level - f;
            if (open[(size_t)l].items.empty() || open[(size_t)l - 1].items.empty()) return false;
            add(open[(size_t)l - 1], close(open[(size_t)l]));
        }
    }
    for (size_t l = 1; l < open.size(); ++l)
        if (!open[l].items.empty()) return false;
    if (open[0].items.size() < 2) return false;
    emit(open[0]);
    cp.n_passes = cp.pass.back() + 1;
    std::vector<int32_t> longest((size_t)cp.n_passes, 0);
    for (size_t g = 0; g < cp.n_chains(); ++g)
        longest[(size_t)cp.pass[g]] = std::max(longest[(size_t)cp.pass[g]], cp.begin[g + 1] - cp.begin[g]);
    for (int32_t len : longest) cp.critical_steps += len;
    return true;
}

// The one-launch form of a program, complete but for the objects' addresses: a table of one record of
// record_words 8-byte words per chain, in pass order. Word 0 of a record: where the chain's value goes,
// as a byte offset into the workgroup's array of values, or result_mark for the chain whose value is the
// result. Words 1..max_items: the items - kSkeletonObject | object index where an object's address
// belongs, or the byte offset of another chain's value - and behind the last item the offset of the
// identity value, which sits behind all values. A value's place is taken when its chain's pass starts and
// is free again from the pass after the one that reads it (every value is read exactly once).
constexpr uint64_t kSkeletonObject = 1ull << 63;
struct ChainSkeleton {
    std::vector<uint64_t> table;
    std::vector<uint32_t> pass_begin;            // pass p is the records [pass_begin[p], pass_begin[p + 1])
    int n_slots = 0, n_chains = 0;               // places for values (the identity takes place n_slots), records
    size_t rounds = 0;                           // chains a team folds one after the other, summed over the passes
    size_t n_steps = 0;                          // of the program it stands for
    bool wide = false;                           // written for the kernels' wide form (whole waves as teams, 1 KiB columns)
};
struct ChainFormat {
    int min_cut = 4, max_items = 23, record_words = 24, teams = 64, max_passes = 24, max_values = 1023;
    uint64_t value_bytes = 64;
    uint32_t result_mark = 0xffffffffu;
};

// False if the program has no such form (plan_chains), needs more passes or places than the format has, or
// would not pay: the longest path through the chains must be at most half the program.
inline bool build_chain_skeleton(const std::vector<Entry> &prog, const ChainFormat &f, ChainSkeleton &sk)
{
    sk = ChainSkeleton();
    if (f.record_words < f.max_items + 1 || f.teams < 1) return false;
    ChainPlan cp;
    if (!plan_chains(prog, f.min_cut, f.max_items, cp)) return false;
    if (cp.n_passes > f.max_passes || cp.critical_steps * 2 > (int64_t)prog.size()) return false;
    const size_t n_chains = cp.n_chains();
    std::vector<int> per_pass((size_t)cp.n_passes, 0);
    for (int32_t ps : cp.pass) per_pass[(size_t)ps]++;
    for (int cnt : per_pass) sk.rounds += (size_t)((cnt + f.teams - 1) / f.teams);
    std::vector<int32_t> order(n_chains);
    for (size_t g = 0; g < n_chains; ++g) order[g] = (int32_t)g;
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return cp.pass[(size_t)x] < cp.pass[(size_t)y]; });
    constexpr uint32_t kNoSlot = 0xffffffffu;
    std::vector<uint32_t> slot(n_chains, kNoSlot), free_slots, freed;
    uint32_t n_slots = 0;
    sk.pass_begin.assign((size_t)cp.n_passes + 1, 0);
    sk.table.assign(n_chains * (size_t)f.record_words, 0);
    constexpr uint64_t kIdentityPending = ~0ull >> 1;        // no object, no value's offset, no result mark
    size_t at = 0;
    for (int pass = 0; pass < cp.n_passes; ++pass) {
        sk.pass_begin[(size_t)pass] = (uint32_t)at;
        free_slots.insert(free_slots.end(), freed.begin(), freed.end());
        freed.clear();
        for (size_t i = at; i < n_chains && cp.pass[(size_t)order[i]] == pass; ++i) {
            const size_t g = (size_t)order[i];
            if (g + 1 == n_chains) continue;                   // the result goes to memory
            if (free_slots.empty()) slot[g] = n_slots++;
            else { slot[g] = free_slots.back(); free_slots.pop_back(); }
        }
        for (; at < n_chains && cp.pass[(size_t)order[at]] == pass; ++at) {
            const size_t g = (size_t)order[at];
            const int32_t begin = cp.begin[g], n = cp.begin[g + 1] - begin;
            uint64_t *rec = sk.table.data() + at * (size_t)f.record_words;
            rec[0] = slot[g] == kNoSlot ? (uint64_t)f.result_mark : (uint64_t)slot[g] * f.value_bytes;
            for (int32_t t = 0; t < n; ++t) {
                const int32_t item = cp.items[(size_t)(begin + t)];
                if (item >= 0) {
                    rec[1 + t] = kSkeletonObject | (uint64_t)item;
                } else {
                    rec[1 + t] = (uint64_t)slot[(size_t)(-item - 1)] * f.value_bytes;
                    freed.push_back(slot[(size_t)(-item - 1)]);
                }
            }
            for (int32_t t = n; t < f.record_words - 1; ++t) rec[1 + t] = kIdentityPending;
        }
    }
    sk.pass_begin[(size_t)cp.n_passes] = (uint32_t)at;
    if ((int64_t)n_slots > (int64_t)f.max_values) return false;
    for (uint64_t &word : sk.table)
        if (word == kIdentityPending) word = (uint64_t)n_slots * f.value_bytes;
    sk.n_slots = (int)n_slots;
    sk.n_chains = (int)n_chains;
    sk.n_steps = prog.size();
    return true;
}

// Accumulator levels a tree needs when every position is taken (holes only lower it).
inline int full_tree_depth(int k, int64_t d)
{
    Tree tr;
    tr.shape(k, d);
    std::vector<int32_t> occ(k, 0);
    std::vector<Entry> prog;
    return compile_program(tr, occ, prog);
}

// The subtrees whose partial results are kept for failure repair (section 3.5.2: when a participant
// fails only its ancestors clear their partial results): all subtrees of more than one node that are
// rooted `depth` levels below the root, as ranges [slot_begin, slot_end) of tree positions (in-order
// numbering makes a subtree a contiguous range of arrivals), in arrival order. What lies outside the
// ranges - the nodes above that depth and the childless nodes at it - is re-read by every repair;
// a failure inside a range re-reads that range. More than max_runs ranges: none.
struct SlotRun { int slot_begin, slot_end; };
inline std::vector<SlotRun> subtrees_at_depth(int k, int64_t d, int depth, int max_runs)
{
    std::vector<SlotRun> runs;
    if (d < 2 || k < 3 || depth < 1) return runs;
    auto subtree_size = [&](int64_t j) {
        int64_t size = 0, first = j, last = j;
        while (first < k) {
            size += std::min<int64_t>(last, k - 1) - first + 1;
            if (first > (INT64_MAX - 1) / d) break;
            first = d * first + 1;
            last = (last > (INT64_MAX - d) / d) ? INT64_MAX : d * last + d;
        }
        return size;
    };
    bool too_many = false;
    int64_t slot = 0;
    // in-order walk of the levels above `depth`: first child's subtree, the node, the other children's
    struct Walk {
        const int k; const int64_t d; const int depth, max_runs;
        std::vector<SlotRun> &runs; int64_t &slot; bool &too_many;
        decltype(subtree_size) &size_of;
        void visit(int64_t j, int level) {
            if (too_many) return;
            if (level == depth) {
                const int64_t size = size_of(j);
                if (size >= 2) {
                    if ((int)runs.size() == max_runs) { too_many = true; return; }
                    runs.push_back({(int)slot, (int)(slot + size)});
                }
                slot += size;
                return;
            }
            const int64_t c1 = d * j + 1;
            if (c1 < k) visit(c1, level + 1);
            ++slot;                                      // the node itself
            for (int64_t c = 2; c <= d && !too_many; ++c) {
                const int64_t ch = d * j + c;
                if (ch >= k) break;
                visit(ch, level + 1);
            }
        }
    } w{k, d, depth, max_runs, runs, slot, too_many, subtree_size};
    w.visit(0, 0);
    if (too_many) runs.clear();
    return runs;
}

// The depth at which partial results are kept (1 to 4 levels below the root): the one for which a
// repair reads least, averaged over which participant fails - a failure outside the kept subtrees
// re-reads the other objects outside and every kept value (4 bytes), a failure inside one re-reads
// the rest of that subtree, the objects outside and the other kept values - among the depths that
// have subtrees, at most max_runs of them, and whose kept values stay below a quarter of what a launch
// reads (k elements of elem_bytes). Level 1 - the subtrees below the root - if no depth qualifies.
inline std::vector<SlotRun> kept_subtrees(int k, int64_t d, int elem_bytes, int max_runs)
{
    std::vector<SlotRun> best = subtrees_at_depth(k, d, 1, max_runs);
    auto expected_repair_bytes = [&](const std::vector<SlotRun> &runs) {
        int64_t covered = 0;
        for (const SlotRun &r : runs) covered += r.slot_end - r.slot_begin;
        const int64_t outside = k - covered, n_runs = (int64_t)runs.size();
        double sum = (double)outside * (double)((outside - 1) * elem_bytes + n_runs * 4);
        for (const SlotRun &r : runs) {
            const int64_t size = r.slot_end - r.slot_begin;
            sum += (double)size * (double)((outside + size - 1) * elem_bytes + (n_runs - 1) * 4);
        }
        return sum / k;
    };
    double best_cost = best.empty() ? 0.0 : expected_repair_bytes(best);
    for (int depth = 2; depth <= 4; ++depth) {
        std::vector<SlotRun> runs = subtrees_at_depth(k, d, depth, max_runs);
        if (runs.empty()) break;
        if ((int64_t)runs.size() * 16 > (int64_t)k * elem_bytes) continue;
        const double cost = expected_repair_bytes(runs);
        if (best.empty() || cost < best_cost) {
            best.swap(runs);
            best_cost = cost;
        }
    }
    return best;
}

// Where the scheduler sends work. launch() runs steps [t0, t1) of prog on output
// chunks [c0, c1). If t0 > 0 the accumulators that the previous launch on those
// chunks saved are restored first (live_before levels); if `final` the result
// is stored, otherwise live_after accumulator levels are saved for the next
// segment. Programs are identified by a version that changes whenever the
// occupants change; steps below t0 are the same in the version that ran them.
struct Backend {
    virtual ~Backend() {}
    // Has everything launched so far been executed? Asked only by the adaptive policy, which
    // advances chunks part of the way only while the device would otherwise sit idle.
    virtual bool idle() { return true; }
    // May launches keep up to n_partials partial results (one accumulator-typed array of object length
    // each) beside the result? Asked once, before the first launch that would; a back end without
    // the memory says no and failures are then repaired by producing the chunks again from scratch.
    virtual bool keep_partials(int n_partials) { (void)n_partials; return true; }
    virtual int launch(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1,
                       bool final, int live_before, int live_after) = 0;
};

// Marker for a tree position that nobody has taken yet while arrivals are still
// possible: it shapes the program like an object, but no step can run past it.
constexpr int32_t kPending = -2;

constexpr int kMaxKept = 16;        // most partial results kept per chunk

class Scheduler {
public:
    Scheduler(int n, int k, int64_t n_chunks, int64_t degree, Backend *be)
        : n_(n), k_(k), C_(n_chunks), be_(be),
          ready_(n, 0), state_(n, UNSEEN), slot_of_obj_(n, -1), occupant_(k, -1)
    {
        tree_.shape(k, degree);
        done_.push_back({C_, 0, 0, false});
        kept_.push_back({C_, 0});
        gens_.emplace_back();
    }

    // Retention of partial results across failures (section 3.5.2: when a participant fails, only
    // the partial results that contain its object are cleared). A launch that produces chunks
    // while some participant in the tree is still streaming - and so can still fail - also stores,
    // per element, the partial result of every subtree rooted at one level of the tree (the one
    // kept_subtrees picks; in the accumulation type, exactly the value the parent's fold consumes).
    // If a participant then fails, the chunks already produced are repaired by a launch that reads
    // the kept partials of the untouched subtrees and re-reads only the objects of the subtree that
    // changed and those above the kept level.
    // Launches made when nobody can fail any more (every bulk call) keep nothing and cost nothing.
    //   on          false: never keep anything (failures redo the produced chunks whole)
    //   min_chunks  launches over fewer chunks keep nothing (too small to be worth a second array)
    //   elem_bytes  size of a source element (a kept value takes 4 bytes)
    // Off until this is called. (Where no launch can be long enough, nothing is prepared at all.)
    void set_retention(bool on, int64_t min_chunks, int elem_bytes)
    {
        retain_min_chunks_ = min_chunks < 1 ? 1 : min_chunks;
        elem_bytes_ = elem_bytes;
        const bool want = on && retain_min_chunks_ <= C_;
        if (want == retain_) return;
        retain_ = want;
        // what was kept under another setting is forgotten; the subtrees are found when first needed
        kept_.assign(1, Kept{C_, 0});
        gens_.assign(1, std::vector<uint32_t>());
        runs_.clear();
        run_of_slot_.clear();
        run_ver_.clear();
        if (retain_) find_runs();
        compiled_version_ = 0;              // the next pump compiles again, now with (or without) the runs' step ranges
        dirty_ = true;
    }

    // 0 (default): a chunk is produced in one launch once all its inputs are present.
    // m >= 1: a chunk also advances through the program whenever at least m further steps
    // have become runnable, saving its accumulators in between (work overlaps the wait
    // for late participants, at the price of extra traffic).
    void set_eager(int min_steps)
    {
        eager_ = min_steps < 0 ? 0 : min_steps;
        dirty_ = true;
    }
    // With the eager policy: advance chunks part of the way only when the back end reports that
    // all earlier work has been executed. Arrivals that come in faster than the device works are
    // then folded together into fewer, longer launches (in the limit: the default policy's single
    // launch), arrivals with gaps between them are worked off in the gaps.
    void set_adaptive(bool on) { adaptive_ = on; }

    // Bulk form of on_ready(obj, all chunks) for objects that arrive complete, in this order.
    // Same effect as calling on_ready(objs[i], n_chunks) one by one.
    int on_arrive_complete(const int *objs, int count)
    {
        for (int i = 0; i < count; ++i) {
            const int obj = objs[i];
            if (obj < 0 || obj >= n_) return HOP_ERR_INVALID;
            if (state_[obj] != UNSEEN || !holes_.empty()) {      // not the plain case: take the general path
                int rc = on_ready(obj, C_);
                if (rc < 0) return rc;
                continue;
            }
            state_[obj] = COMPLETE;
            ready_[obj] = C_;
            if (next_free_ < k_) {
                place(obj, next_free_++);
            } else {
                pool_.push_back(obj);
            }
        }
        return HOP_OK;
    }

    // Object obj has chunks [0, c) ready. First call = arrival.
    int on_ready(int obj, int64_t c)
    {
        if (obj < 0 || obj >= n_ || c < 0 || c > C_) return HOP_ERR_INVALID;
        if (state_[obj] == FAILED || c < ready_[obj]) return HOP_ERR_INVALID;
        if (state_[obj] == UNSEEN) {
            state_[obj] = STREAMING;
            if (!holes_.empty()) {
                // a position emptied by a failure goes to the next ready object
                int t = *holes_.begin();
                holes_.erase(holes_.begin());
                place(obj, t);
                info_.n_replaced++;
            } else if (next_free_ < k_) {
                place(obj, next_free_++);
            } else {
                pool_.push_back(obj);
            }
        }
        if (c > ready_[obj] && slot_of_obj_[obj] >= 0) dirty_ = true;      // new chunks of a participant in the tree
        ready_[obj] = c;
        if (c == C_) state_[obj] = COMPLETE;
        return HOP_OK;
    }

    int on_fail(int obj)
    {
        if (obj < 0 || obj >= n_) return HOP_ERR_INVALID;
        if (state_[obj] == FAILED || state_[obj] == COMPLETE) return HOP_OK;   // complete objects are immutable and stay valid
        state_[obj] = FAILED;
        info_.n_failed_seen++;
        int t = slot_of_obj_[obj];
        if (t < 0) return HOP_OK;            // was waiting (or never arrived): skipped when the pool is popped
        slot_of_obj_[obj] = -1;
        occupant_[t] = -1;
        touch_run(t);
        version_++;
        dirty_ = true;
        while (!pool_.empty() && state_[pool_.front()] == FAILED) pool_.pop_front();
        if (!pool_.empty()) {
            int j = pool_.front();
            pool_.pop_front();
            place(j, t);
            info_.n_replaced++;
        } else {
            holes_.insert(t);
        }
        return HOP_OK;
    }

    // Launch whatever the readiness reported so far allows.
    int pump()
    {
        // Nothing that matters has happened since the last pump (e.g. an object beyond the first k
        // reported more chunks), or - default policy - some position has not been taken yet, so no
        // chunk can run the whole program: events stay cheap until there is something to launch.
        if (!dirty_) return HOP_OK;
        if (eager_ == 0 && !closing_ && next_free_ < k_) return HOP_OK;
        dirty_ = false;
        int rc = recompile();
        if (rc < 0) return rc;
        const int n_steps = (int)prog_.size();
        if (n_steps == 0) return HOP_OK;
        // How far can each chunk go? Steps run in order, so chunk c can run t steps iff the
        // objects of steps 0..t-1 all have chunk c. With m[t] = min ready count over steps
        // 0..t (non-increasing in t), chunks [m[t], m[t-1]) can run exactly t steps.
        std::vector<Stair> target;
        {
            std::vector<int64_t> m(n_known_);
            int64_t run = C_;
            for (int t = 0; t < n_known_; ++t) {
                run = std::min(run, ready_[prog_[t].obj]);
                m[t] = run;
            }
            int64_t lo = 0;
            for (int t = n_known_; t >= 0; --t) {
                const int64_t hi = (t == 0) ? C_ : m[t - 1];
                if (hi > lo) { target.push_back({hi, t, 0, false}); lo = hi; }
            }
        }
        // Walk the two staircases together; every piece where progress is allowed is a launch.
        const bool may_partial = eager_ > 0 && (!adaptive_ || be_->idle());
        bool held_back = false;
        // act: what a whole-program launch does with the kept partials of its chunks (see run_actions);
        // empty for launches that have nothing to do with them
        struct Piece { int64_t c0, c1; int t0, t1; int64_t redo, redo_chunks; uint32_t gen; std::vector<int8_t> act; };
        std::vector<Piece> pieces;
        std::vector<Stair> next;
        // runs may be kept or reused only by whole-program launches; everything known about the tree
        const bool retention = retain_ && !keep_refused_ && !runs_.empty() && n_known_ == n_steps;
        const bool exposed = retention && any_streaming();
        std::vector<std::vector<int8_t>> act_of_gen(retention ? gens_.size() : 0);
        std::vector<char> act_known(act_of_gen.size(), 0);
        size_t i = 0, j = 0, m = 0;
        int64_t c = 0;
        while (c < C_) {
            int64_t end = std::min(done_[i].chunk_end, target[j].chunk_end);
            if (retention) end = std::min(end, kept_[m].chunk_end);
            const int t0 = done_[i].t;
            int t1 = std::max(t0, target[j].t);
            const bool complete = (t1 == n_steps);
            if (t1 > t0 && !(complete || (may_partial && t1 - t0 >= eager_))) {
                held_back |= eager_ > 0 && !may_partial && t1 - t0 >= eager_;
                t1 = t0;
            }
            int redo = done_[i].redo;
            bool stored = done_[i].stored;
            // a launch if steps can run, or if every step has run but the result still sits in
            // saved accumulators (the program got shorter after these chunks had run ahead)
            if (t1 > t0 || (t0 == n_steps && !stored)) {
                const int64_t again = std::max(0, std::min(t1, redo) - t0);
                std::vector<int8_t> act;
                uint32_t gen = 0;
                if (retention && t0 == 0 && t1 == n_steps) {
                    gen = kept_[m].gen;
                    if (!act_known[gen]) {
                        act_of_gen[gen] = run_actions(gen, exposed);
                        act_known[gen] = 1;
                    }
                    act = act_of_gen[gen];
                    bool any = false;
                    for (int8_t a : act) any |= a != RUN_PLAIN;
                    if (!any) act.clear();
                }
                if (!pieces.empty() && pieces.back().c1 == c && pieces.back().t0 == t0 && pieces.back().t1 == t1 &&
                    pieces.back().act == act && (act.empty() || pieces.back().gen == gen)) {
                    pieces.back().c1 = end;
                    pieces.back().redo += again * (end - c);
                    pieces.back().redo_chunks += again > 0 ? end - c : 0;
                } else {
                    pieces.push_back({c, end, t0, t1, again * (end - c), again > 0 ? end - c : 0, gen, act});
                }
                if (t1 >= redo || t1 == n_steps) redo = 0;      // (the new program may be shorter than the one redone)
                stored = (t1 == n_steps);
            }
            if (!next.empty() && next.back().t == t1 && next.back().redo == redo && next.back().stored == stored)
                next.back().chunk_end = end;
            else
                next.push_back({end, t1, redo, stored});
            c = end;
            if (done_[i].chunk_end == end) ++i;
            if (target[j].chunk_end == end) ++j;
            if (retention && kept_[m].chunk_end == end) ++m;
        }
        for (Piece &p : pieces) {
            const bool final = (p.t1 == n_steps);
            // launches too short to be worth a kept array store nothing (they may still read)
            if (!p.act.empty() && p.c1 - p.c0 < retain_min_chunks_) {
                bool any = false;
                for (int8_t &a : p.act) {
                    if (a == RUN_SAVE) a = RUN_PLAIN;
                    any |= a != RUN_PLAIN;
                }
                if (!any) p.act.clear();
            }
            if (!p.act.empty() && !keep_asked_) {
                keep_asked_ = true;
                keep_refused_ = !be_->keep_partials((int)runs_.size());
            }
            if (!p.act.empty() && !keep_refused_) {
                std::vector<Entry> rp;
                int n_reuse = 0, n_save = 0;
                retained_program(p.act, rp, &n_reuse, &n_save);
                rc = be_->launch(rp, (uint64_t(1) << 63) | ++aux_version_, p.c0, p.c1, 0, (int)rp.size(), true, 0, 0);
                if (rc < 0) return rc;
                const int64_t chunks = p.c1 - p.c0, n_obj = (int64_t)rp.size() - n_reuse;
                info_.n_launches++;
                info_.chunks_redone += n_reuse > 0 ? p.redo_chunks * n_obj : p.redo;
                info_.chunk_steps += chunks * n_obj;
                info_.chunk_stores += chunks;
                info_.partial_loads += chunks * n_reuse;
                info_.partial_stores += chunks * n_save;
                // what these chunks hold now: the partials just stored, and the older ones still valid
                std::vector<uint32_t> now(runs_.size(), 0);
                const std::vector<uint32_t> had = gens_[p.gen];
                bool any = false;
                for (size_t r = 0; r < runs_.size(); ++r) {
                    now[r] = p.act[r] == RUN_SAVE ? run_ver_[r] : (had[r] == run_ver_[r] ? had[r] : 0);
                    any |= now[r] != 0;
                }
                uint32_t g = 0;
                if (any) {
                    for (g = 1; g < gens_.size() && gens_[g] != now; ++g) {}
                    if (g == gens_.size()) gens_.push_back(now);
                }
                assign_kept(p.c0, p.c1, g);
                continue;
            }
            rc = be_->launch(prog_, version_, p.c0, p.c1, p.t0, p.t1, final, live_levels(p.t0), final ? 0 : live_levels(p.t1));
            if (rc < 0) return rc;
            info_.n_launches++;
            info_.chunks_redone += p.redo;
            info_.chunk_steps += (p.c1 - p.c0) * (int64_t)(p.t1 - p.t0);
            info_.chunk_stores += (p.c1 - p.c0) * (int64_t)(final ? 1 : live_levels(p.t1));
        }
        done_.swap(next);
        if (held_back) dirty_ = true;        // try again at the next event
        return HOP_OK;
    }

    // No more events: incomplete participants count as failed, unfilled
    // positions stay empty, the rest of the output is produced.
    int finish(hop_info_t *info)
    {
        for (int obj : pool_)
            if (state_[obj] == STREAMING) { state_[obj] = FAILED; info_.n_failed_seen++; }
        for (int t = 0; t < k_; ++t) {
            int o = occupant_[t];
            if (o >= 0 && state_[o] == STREAMING) on_fail(o);
            // a replacement pulled from the pool is complete (incomplete ones were just failed)
        }
        if (!closing_) {
            closing_ = true;
            if (next_free_ < k_) version_++;        // positions nobody took are empty for good
        }
        dirty_ = true;
        int rc = pump();
        int live = 0;
        for (int t = 0; t < k_; ++t) live += occupant_[t] >= 0;
        info_.k_eff = live;
        info_.degree_used = (int32_t)std::min<int64_t>(tree_.d, INT32_MAX);
        if (info) *info = info_;
        if (rc < 0) return rc;
        if (live == 0) return HOP_ERR_NO_SURVIVOR;
        return live < k_ ? HOP_PARTIAL : HOP_OK;
    }

    // Output chunks [0, result) are final in the destination (as far as enqueued work goes).
    int64_t chunks_final() const
    {
        if (prog_.empty() || compiled_version_ != version_) return 0;
        return done_.front().stored ? done_.front().chunk_end : 0;
    }

    bool arrived(int obj) const { return state_[obj] != UNSEEN; }
    bool alive(int obj) const { return state_[obj] == STREAMING || state_[obj] == COMPLETE; }
    const Tree &tree() const { return tree_; }
    // who holds each tree position now (-1 = empty)
    const std::vector<int32_t> &occupants() const { return occupant_; }

private:
    enum State : uint8_t { UNSEEN, STREAMING, COMPLETE, FAILED };
    // chunks [previous chunk_end, chunk_end) have run t steps of the program; redo > 0: they had
    // run that many steps of an earlier program whose result was thrown away
    struct Stair { int64_t chunk_end; int t; int redo; bool stored; };

    void place(int obj, int t)
    {
        occupant_[t] = obj;
        slot_of_obj_[obj] = t;
        touch_run(t);
        version_++;
        dirty_ = true;
    }

    // ---- kept partial results -------------------------------------------------------------

    void find_runs()
    {
        runs_ = kept_subtrees(k_, tree_.d, elem_bytes_, kMaxKept);
        if (runs_.empty()) return;
        run_of_slot_.assign((size_t)k_, -1);
        for (size_t r = 0; r < runs_.size(); ++r)
            for (int t = runs_[r].slot_begin; t < runs_[r].slot_end; ++t) run_of_slot_[(size_t)t] = (int16_t)r;
        run_ver_.assign(runs_.size(), 1);
        gens_[0].assign(runs_.size(), 0);
    }

    void touch_run(int t)
    {
        if (run_of_slot_.empty()) return;
        const int r = run_of_slot_[(size_t)t];
        if (r >= 0) run_ver_[(size_t)r]++;
    }

    bool any_streaming() const
    {
        for (int t = 0; t < k_; ++t)
            if (occupant_[t] >= 0 && state_[occupant_[t]] == STREAMING) return true;
        return false;
    }

    // What a whole-program launch over chunks whose kept partials are generation `gen` does with
    // every run: 0 nothing, 1 read its kept partial instead of its objects, 2 store its partial.
    enum : int8_t { RUN_PLAIN = 0, RUN_REUSE = 1, RUN_SAVE = 2 };
    std::vector<int8_t> run_actions(uint32_t gen, bool may_save) const
    {
        std::vector<int8_t> act(runs_.size(), RUN_PLAIN);
        if (runs_.empty() || !retain_ || keep_refused_) return act;
        const std::vector<uint32_t> &have = gens_[gen];
        int n_save = 0;
        for (size_t r = 0; r < runs_.size(); ++r) {
            const int len = run_steps_[r].second - run_steps_[r].first;
            // worth it only if the kept value (4 bytes) is smaller than what it stands for
            if (len < 1 || len * elem_bytes_ <= 4 || !prog_[(size_t)run_steps_[r].first].set) continue;
            if (have[r] != 0 && have[r] == run_ver_[r]) { act[r] = RUN_REUSE; continue; }
            if (may_save) { act[r] = RUN_SAVE; ++n_save; }
        }
        // keeping must stay a side cost: at most a quarter of what the launch reads anyway
        if ((int64_t)n_save * 4 * 4 > (int64_t)prog_.size() * elem_bytes_)
            for (int8_t &a : act) if (a == RUN_SAVE) a = RUN_PLAIN;
        return act;
    }

    // prog_ with the runs treated as act says
    void retained_program(const std::vector<int8_t> &act, std::vector<Entry> &out, int *n_reuse, int *n_save) const
    {
        out.clear();
        out.reserve(prog_.size());
        *n_reuse = *n_save = 0;
        size_t r = 0;
        for (int i = 0; i < (int)prog_.size();) {
            while (r < runs_.size() && run_steps_[r].second <= i) ++r;
            if (r < runs_.size() && run_steps_[r].first == i && run_steps_[r].second > i && act[r] != RUN_PLAIN) {
                const int i0 = run_steps_[r].first, i1 = run_steps_[r].second;
                const Entry &first = prog_[(size_t)i0], &last = prog_[(size_t)i1 - 1];
                const int internal = (int)last.level - (int)first.level;       // folds of the last step that stay inside the run
                if (act[r] == RUN_REUSE) {
                    // the partial starts the run's accumulator; the folds that carried the run's value
                    // further down follow as before
                    Entry e{-(1 + (int32_t)r), first.level, 1, (uint16_t)((int)last.n_fold - internal)};
                    out.push_back(e);
                    ++*n_reuse;
                } else {
                    for (int t = i0; t < i1; ++t) out.push_back(prog_[(size_t)t]);
                    out.back().save = (int16_t)r;
                    out.back().save_level = first.level;
                    ++*n_save;
                }
                i = i1;
                continue;
            }
            out.push_back(prog_[(size_t)i]);
            ++i;
        }
    }

    void assign_kept(int64_t c0, int64_t c1, uint32_t gen)
    {
        std::vector<Kept> next;
        int64_t begin = 0;
        auto put = [&](int64_t end, uint32_t g) {
            if (end <= begin) return;
            if (!next.empty() && next.back().gen == g) next.back().chunk_end = end;
            else next.push_back({end, g});
            begin = end;
        };
        for (const Kept &kp : kept_) {
            const int64_t lo = begin, hi = kp.chunk_end;
            if (hi <= c0 || lo >= c1) { put(hi, kp.gen); continue; }
            if (lo < c0) put(c0, kp.gen);
            put(std::min(hi, c1), gen);
            if (hi > c1) put(hi, kp.gen);
        }
        kept_.swap(next);
    }

    // accumulator levels alive between steps t-1 and t
    int live_levels(int t) const
    {
        if (t <= 0) return 0;
        return (int)prog_[t - 1].level - (int)prog_[t - 1].n_fold + 1;
    }

    // The occupants changed: rebuild the program. Chunks keep what they have computed as long
    // as the steps they ran are unchanged (a common prefix of the old and the new program);
    // chunks that ran past the first difference start over (section 3.5.2: every partial
    // result that contains the failed object is cleared, the others are kept).
    int recompile()
    {
        if (compiled_version_ == version_) return HOP_OK;
        std::vector<int32_t> occ(occupant_);
        if (!closing_)
            for (int t = next_free_; t < k_; ++t) occ[t] = kPending;
        std::vector<Entry> np;
        const int depth = compile_program(tree_, occ, np, runs_.empty() ? nullptr : &slot_of_step_);
        info_.stack_depth = std::max(info_.stack_depth, depth);
        if (depth > HOP_MAX_DEPTH) return HOP_ERR_DEPTH;
        int keep = 0;
        while (keep < (int)prog_.size() && keep < (int)np.size() && np[keep].obj != kPending &&
               prog_[keep].obj == np[keep].obj && prog_[keep].level == np[keep].level &&
               prog_[keep].set == np[keep].set && prog_[keep].n_fold == np[keep].n_fold)
            ++keep;
        // a chunk whose result was stored saved no accumulators: it cannot be continued either,
        // unless nothing changed at all
        const bool unchanged = keep == (int)prog_.size() && keep == (int)np.size();
        std::vector<Stair> next;
        for (Stair st : done_) {
            if (st.t > keep || (st.stored && !unchanged)) {
                st.redo = std::max(st.redo, st.t);
                st.t = 0;
                st.stored = false;
            }
            if (!next.empty() && next.back().t == st.t && next.back().redo == st.redo && next.back().stored == st.stored)
                next.back().chunk_end = st.chunk_end;
            else next.push_back(st);
        }
        done_.swap(next);
        prog_.swap(np);
        // where every run's steps are (positions inside a run are consecutive steps; empty ones emit nothing)
        run_steps_.assign(runs_.size(), std::make_pair(0, 0));
        for (size_t r = 0, i = 0; r < runs_.size(); ++r) {
            while (i < slot_of_step_.size() && slot_of_step_[i] < runs_[r].slot_begin) ++i;
            run_steps_[r].first = (int)i;
            while (i < slot_of_step_.size() && slot_of_step_[i] < runs_[r].slot_end) ++i;
            run_steps_[r].second = (int)i;
        }
        n_known_ = 0;
        while (n_known_ < (int)prog_.size() && prog_[n_known_].obj != kPending) ++n_known_;
        compiled_version_ = version_;
        return HOP_OK;
    }

    int n_, k_;
    int64_t C_;
    Backend *be_;
    Tree tree_;
    std::vector<int64_t> ready_;
    std::vector<State> state_;
    std::vector<int32_t> slot_of_obj_, occupant_;
    std::deque<int32_t> pool_;           // arrived, not in the tree, in arrival order
    std::set<int> holes_;                // positions emptied by a failure with nobody waiting
    int next_free_ = 0;                  // positions [0, next_free_) have been handed out
    bool closing_ = false;
    bool dirty_ = false;                 // something changed that a pump could act on
    int eager_ = 0;
    bool adaptive_ = false;
    struct Kept { int64_t chunk_end; uint32_t gen; };
    std::vector<SlotRun> runs_;                          // the subtrees whose partials are kept, as ranges of positions
    std::vector<int16_t> run_of_slot_;
    std::vector<uint32_t> run_ver_;                  // changes whenever an occupant inside the run changes
    std::vector<std::pair<int, int>> run_steps_;     // the run's steps in prog_: [first, second)
    std::vector<Kept> kept_;                         // chunks [previous end, chunk_end) hold the partials of generation gen
    std::vector<std::vector<uint32_t>> gens_;        // per generation and run: run_ver_ when its partial was stored, 0 = none
    bool retain_ = false, keep_asked_ = false, keep_refused_ = false;
    int64_t retain_min_chunks_ = 1;
    int elem_bytes_ = 4;
    std::vector<int32_t> slot_of_step_;
    uint64_t aux_version_ = 0;                       // names the programs built by retained_program
    std::vector<Stair> done_;            // progress of every chunk through prog_
    uint64_t version_ = 1, compiled_version_ = 0;
    std::vector<Entry> prog_;
    int n_known_ = 0;                    // steps before the first pending position
    hop_info_t info_ = {};
};

// hop_reduce as a replay of session events: every object that ever becomes
// ready announces itself in ready order; then all participants stream their
// chunks side by side, so a participant with fail_mask c is found failed when
// everyone has delivered c chunks, after the scheduler has used them.
inline int replay_reduce(Scheduler &s, int n, int64_t C, const int32_t *ready_order,
                         const int64_t *fail_mask, hop_info_t *info)
{
    std::vector<int> arrival;
    arrival.reserve(n);
    std::vector<int64_t> limit(n, C);
    std::vector<int64_t> steps;
    for (int t = 0; t < n; ++t) {
        int i = ready_order ? ready_order[t] : t;
        if (fail_mask && fail_mask[i] >= 0 && fail_mask[i] < C) limit[i] = fail_mask[i];
        if (limit[i] == 0) continue;                 // never becomes ready
        arrival.push_back(i);
        if (limit[i] < C) steps.push_back(limit[i]);
    }
    int rc;
    if (steps.empty()) {
        // nobody fails part-way: everyone announces itself and delivers everything, one launch
        if ((rc = s.on_arrive_complete(arrival.data(), (int)arrival.size())) < 0) return rc;
        return s.finish(info);
    }
    std::sort(steps.begin(), steps.end());
    steps.erase(std::unique(steps.begin(), steps.end()), steps.end());
    for (int i : arrival)
        if ((rc = s.on_ready(i, 0)) < 0) return rc;
    for (int64_t step : steps) {
        for (int i : arrival)
            if (s.alive(i) && (rc = s.on_ready(i, std::min(step, limit[i]))) < 0) return rc;
        if ((rc = s.pump()) < 0) return rc;
        for (int i : arrival)
            if (limit[i] == step && (rc = s.on_fail(i)) < 0) return rc;
    }
    for (int i : arrival)
        if (s.alive(i) && (rc = s.on_ready(i, C)) < 0) return rc;
    return s.finish(info);
}

// Eq. 1 of section 3.4.2: T(1) = n L + S/B, T(d) = L log_d n + d S/B. The
// paper's runtime restricts the choice to d in {1, 2, n} (section 4).
inline double tree_cost(int n, double d, double S, double L, double B)
{
    if (d <= 1.0) return n * L + S / B;
    return L * (std::log((double)n) / std::log(d)) + d * S / B;
}

}  // namespace hop
