// Host-side coordination of the receiver-driven broadcast (paper section 3.4.1)
// and its failure handling (section 3.5.1). No HIP in this file.
//
// The "directory" lists, for one object, the copies that are not busy sending:
// complete copies and partial ones (still being received). A receiver that
// joins asks for ONE location, complete preferred over partial; that sender
// leaves the directory while it serves the receiver, the receiver enters it at
// once as a partial copy (so later receivers can chain off it chunk by chunk),
// and when the transfer ends the sender is listed again and the receiver is
// complete. Hence every copy sends to at most one receiver at a time and the
// broadcast tree forms from the arrival order. When a sender fails, its
// receiver asks again and resumes from the chunk it already has, never from a
// copy that (transitively) fetches from the receiver itself.
#pragma once

#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/hop.h"

namespace hop {

struct BcastBackend {
    virtual ~BcastBackend() {}
    // copy chunks [c0, c1) of copy `from` into copy `to`
    virtual int copy(int from, int to, int64_t c0, int64_t c1) = 0;
};

class BcastScheduler {
public:
    BcastScheduler(int64_t n_chunks, BcastBackend *be) : C_(n_chunks), be_(be)
    {
        copies_.push_back(Copy());          // copy 0 is the original (the creator's Put)
    }

    // the original copy has chunks [0, c) (its Put may still be in progress)
    int source_ready(int64_t c)
    {
        if (c < copies_[0].have || c > C_ || copies_[0].failed) return HOP_ERR_INVALID;
        copies_[0].have = c;
        return HOP_OK;
    }

    // A receiver arrives. Returns its copy id (>= 1); *sender is the copy it fetches from, or -1
    // if every copy is busy (it is served as soon as one is listed again).
    int join(int *sender)
    {
        Copy r;
        copies_.push_back(r);
        const int id = (int)copies_.size() - 1;
        const int s = pick_sender(id);
        if (s >= 0) attach(id, s);
        if (sender) *sender = s;
        return id;
    }

    // Copy `id` is lost (its node failed). Its receiver asks the directory again; the copy it was
    // fetching from is listed again.
    int fail(int id)
    {
        if (id < 0 || id >= (int)copies_.size()) return HOP_ERR_INVALID;
        Copy &x = copies_[(size_t)id];
        if (x.failed) return HOP_OK;
        x.failed = true;
        info_failed_++;
        if (x.from >= 0) {
            copies_[(size_t)x.from].serving = -1;
            x.from = -1;
        }
        if (x.serving >= 0) {
            const int r = x.serving;
            x.serving = -1;
            copies_[(size_t)r].from = -1;
            const int s = pick_sender(r);
            if (s >= 0) attach(r, s);
        }
        return HOP_OK;
    }

    // One time step: every transfer moves up to max_chunks chunks (0 = as many as its sender has),
    // senders before their receivers; finished transfers list their sender again, and receivers
    // that found every copy busy ask again.
    int step(int64_t max_chunks)
    {
        int rc = move(max_chunks);
        return rc < 0 ? rc : requery();
    }

    // Run to the end: repeat unlimited steps until nothing changes.
    int drain()
    {
        for (;;) {
            const int64_t before = chunks_copied_;
            const int attached_before = n_attached_;
            int rc = step(0);
            if (rc < 0) return rc;
            if (chunks_copied_ == before && n_attached_ == attached_before) return HOP_OK;
        }
    }

private:
    int move(int64_t max_chunks)
    {
        {
            // senders before their receivers: walk copies in an order where a copy's source comes first
            std::vector<int> order = topo_order();
            for (int id : order) {
                Copy &r = copies_[(size_t)id];
                if (r.failed || r.from < 0) continue;
                Copy &s = copies_[(size_t)r.from];
                int64_t upto = s.have;
                if (max_chunks > 0) upto = std::min(upto, r.have + max_chunks);
                if (upto > r.have) {
                    int rc = be_->copy(r.from, id, r.have, upto);
                    if (rc < 0) return rc;
                    chunks_copied_ += upto - r.have;
                    r.have = upto;
                }
                if (r.have == C_) {              // transfer complete: sender listed again, receiver complete
                    s.serving = -1;
                    r.from = -1;
                }
            }
        }
        return HOP_OK;
    }

    int requery()
    {
        for (size_t id = 1; id < copies_.size(); ++id) {
            Copy &r = copies_[id];
            if (r.failed || r.from >= 0 || r.have == C_) continue;
            const int s = pick_sender((int)id);
            if (s >= 0) attach((int)id, s);
        }
        return HOP_OK;
    }

public:
    int n_copies() const { return (int)copies_.size(); }
    int64_t have(int id) const { return copies_[(size_t)id].have; }
    bool complete(int id) const { return copies_[(size_t)id].have == C_; }
    int sender_of(int id) const { return copies_[(size_t)id].from; }
    bool failed(int id) const { return copies_[(size_t)id].failed; }
    int64_t chunks_copied() const { return chunks_copied_; }
    int n_failed() const { return info_failed_; }
    int n_resumed() const { return info_resumed_; }
    bool all_complete() const
    {
        for (size_t id = 1; id < copies_.size(); ++id)
            if (!copies_[id].failed && copies_[id].have != C_) return false;
        return true;
    }

private:
    struct Copy {
        int64_t have = 0;       // chunks [0, have) present
        int from = -1;          // copy it is fetching from
        int serving = -1;       // copy it is sending to (at most one)
        bool failed = false;
        bool attached_before = false;
    };

    bool depends_on(int id, int target) const      // does `id` (transitively) fetch from `target`?
    {
        for (int x = id; x >= 0; x = copies_[(size_t)x].from)
            if (x == target) return true;
        return false;
    }

    // the directory's answer: an idle complete copy if there is one, else an idle partial one
    int pick_sender(int receiver) const
    {
        int partial = -1;
        for (int id = 0; id < (int)copies_.size(); ++id) {
            const Copy &c = copies_[(size_t)id];
            if (id == receiver || c.failed || c.serving >= 0) continue;
            if (id != 0 && c.from < 0 && c.have < C_) continue;      // a receiver that is itself waiting has nothing to offer yet
            if (depends_on(id, receiver)) continue;
            if (c.have == C_ && c.from < 0) return id;               // complete
            if (partial < 0) partial = id;
        }
        return partial;
    }

    void attach(int receiver, int sender)
    {
        n_attached_++;
        if (copies_[(size_t)receiver].attached_before) info_resumed_++;      // a transfer taken up again elsewhere
        copies_[(size_t)receiver].attached_before = true;
        copies_[(size_t)receiver].from = sender;
        copies_[(size_t)sender].serving = receiver;
    }

    std::vector<int> topo_order() const
    {
        std::vector<int> depth(copies_.size(), 0), order;
        for (size_t id = 0; id < copies_.size(); ++id) {
            int d = 0;
            for (int x = copies_[id].from; x >= 0; x = copies_[(size_t)x].from) ++d;
            depth[id] = d;
            order.push_back((int)id);
        }
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return depth[(size_t)a] < depth[(size_t)b]; });
        return order;
    }

    int64_t C_;
    BcastBackend *be_;
    std::vector<Copy> copies_;
    int64_t chunks_copied_ = 0;
    int info_failed_ = 0, info_resumed_ = 0, n_attached_ = 0;
};

}  // namespace hop
