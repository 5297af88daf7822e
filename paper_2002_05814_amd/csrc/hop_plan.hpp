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
struct Entry {
    int32_t obj;
    uint8_t level;
    uint8_t set;
    uint16_t n_fold;
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
inline int compile_program(const Tree &tr, const std::vector<int32_t> &occupant, std::vector<Entry> &out)
{
    out.clear();
    const int k = tr.k;
    const int64_t d = tr.d;
    if (d == 1 || k == 1) {
        // chain: plain left fold in arrival order
        for (int t = 0; t < k; ++t) {
            if (occupant[t] == -1) continue;
            out.push_back({occupant[t], 0, (uint8_t)out.empty(), 0});
        }
        return out.empty() ? 0 : 1;
    }
    // d >= 2: height <= log2(k), recursion is shallow. The walk is the in-order traversal
    // itself, so the next position in arrival order is simply a running counter. Most nodes
    // of a wide tree are leaves: they are emitted without a call.
    out.resize((size_t)k);
    struct Walk {
        const int k; const int64_t d; const int32_t *occ; Entry *out; int n_out; int depth; int slot;
        bool leaf(int level) {
            const int32_t o = occ[slot++];
            if (o == -1) return false;
            out[n_out++] = Entry{o, (uint8_t)level, 1, 0};
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
                out[n_out++] = Entry{o, (uint8_t)level, (uint8_t)!started, 0};
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
                    if (o != -1) out[n_out++] = Entry{o, (uint8_t)level, 0, 0};
                } else if (node(ch, level + 1)) {     // at most log2(k) < 32 levels
                    out[n_out - 1].n_fold++;
                }
            }
            return started;
        }
    } w{k, d, occupant.data(), out.data(), 0, 0, 0};
    w.node(0, 0);
    out.resize((size_t)w.n_out);
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

// Accumulator levels a tree needs when every position is taken (holes only lower it).
inline int full_tree_depth(int k, int64_t d)
{
    Tree tr;
    tr.shape(k, d);
    std::vector<int32_t> occ(k, 0);
    std::vector<Entry> prog;
    return compile_program(tr, occ, prog);
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
    virtual int launch(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1,
                       bool final, int live_before, int live_after) = 0;
};

// Marker for a tree position that nobody has taken yet while arrivals are still
// possible: it shapes the program like an object, but no step can run past it.
constexpr int32_t kPending = -2;

class Scheduler {
public:
    Scheduler(int n, int k, int64_t n_chunks, int64_t degree, Backend *be)
        : n_(n), k_(k), C_(n_chunks), be_(be),
          ready_(n, 0), state_(n, UNSEEN), slot_of_obj_(n, -1), occupant_(k, -1)
    {
        tree_.shape(k, degree);
        done_.push_back({C_, 0, 0, false});
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
                occupant_[next_free_] = obj;
                slot_of_obj_[obj] = next_free_++;
                version_++;
                dirty_ = true;
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
        struct Piece { int64_t c0, c1; int t0, t1; int64_t redo; };
        std::vector<Piece> pieces;
        std::vector<Stair> next;
        size_t i = 0, j = 0;
        int64_t c = 0;
        while (c < C_) {
            const int64_t end = std::min(done_[i].chunk_end, target[j].chunk_end);
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
                if (!pieces.empty() && pieces.back().c1 == c && pieces.back().t0 == t0 && pieces.back().t1 == t1) {
                    pieces.back().c1 = end;
                    pieces.back().redo += again * (end - c);
                } else {
                    pieces.push_back({c, end, t0, t1, again * (end - c)});
                }
                if (t1 >= redo) redo = 0;
                stored = (t1 == n_steps);
            }
            if (!next.empty() && next.back().t == t1 && next.back().redo == redo && next.back().stored == stored)
                next.back().chunk_end = end;
            else
                next.push_back({end, t1, redo, stored});
            c = end;
            if (done_[i].chunk_end == end) ++i;
            if (target[j].chunk_end == end) ++j;
        }
        for (const Piece &p : pieces) {
            const bool final = (p.t1 == n_steps);
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

private:
    enum State : uint8_t { UNSEEN, STREAMING, COMPLETE, FAILED };
    // chunks [previous chunk_end, chunk_end) have run t steps of the program; redo > 0: they had
    // run that many steps of an earlier program whose result was thrown away
    struct Stair { int64_t chunk_end; int t; int redo; bool stored; };

    void place(int obj, int t)
    {
        occupant_[t] = obj;
        slot_of_obj_[obj] = t;
        version_++;
        dirty_ = true;
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
        const int depth = compile_program(tree_, occ, np);
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
