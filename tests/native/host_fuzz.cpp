// Host-only stress of the chunk scheduler (hop_plan.hpp) under AddressSanitizer and
// UBSan: random sessions (arrivals, chunk deliveries, failures, eager policies) against a
// back end that checks every launch it is given. No GPU, no HIP.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <string>
#include <vector>

#include "../../paper_2002_05814_amd/csrc/hop_bcast.hpp"
#include "../../paper_2002_05814_amd/csrc/hop_plan.hpp"
#include "../../paper_2002_05814_amd/csrc/hop_program.h"

using namespace hop;

// Evaluates every launch symbolically, chunk by chunk: accumulators, saved accumulators and kept
// partial results are expressions written out as strings, so that at the end every chunk's stored
// result can be compared, parenthesis for parenthesis, with the expression of the final tree.
static std::string sym_eval(const std::vector<Entry> &prog, int t0, int t1, std::vector<std::string> acc,
                            const std::vector<std::string> *kept_of_chunk, std::vector<std::string> *kept_out,
                            std::vector<std::string> *acc_out)
{
    acc.resize(HOP_MAX_DEPTH + 1);
    for (int t = t0; t < t1; ++t) {
        const Entry &e = prog[(size_t)t];
        std::string x;
        if (e.obj >= 0) x = "o" + std::to_string(e.obj);
        else {
            const size_t q = (size_t)(-e.obj - 1);
            if (!kept_of_chunk || q >= kept_of_chunk->size() || (*kept_of_chunk)[q].empty()) { std::printf("reads a partial that was never kept\n"); std::abort(); }
            x = (*kept_of_chunk)[q];
        }
        int level = e.level, n_fold = e.n_fold;
        acc[(size_t)level] = e.set ? x : "(" + acc[(size_t)level] + "+" + x + ")";
        auto fold = [&]() { acc[(size_t)level - 1] = "(" + acc[(size_t)level - 1] + "+" + acc[(size_t)level] + ")"; acc[(size_t)level].clear(); --level; --n_fold; };
        if (e.save >= 0) {
            if (e.save_level > e.level || (int)e.level - (int)e.save_level > n_fold) { std::printf("save level\n"); std::abort(); }
            while (level > (int)e.save_level) fold();
            if (!kept_out || (size_t)e.save >= kept_out->size()) { std::printf("keeps where nothing can be kept\n"); std::abort(); }
            (*kept_out)[(size_t)e.save] = acc[(size_t)level];
        }
        while (n_fold > 0) fold();
    }
    if (acc_out) *acc_out = acc;
    return acc[0];
}

struct CheckingBackend : Backend {
    int64_t C = 0;
    std::mt19937_64 *rng = nullptr;      // when set: the device is "busy" at random
    bool idle() override { return !rng || ((*rng)() & 1u); }
    bool refuse_keeping = false;
    int n_partials = 0;
    bool keep_partials(int n) override
    {
        if (n < 1 || n > 16) { std::printf("asks to keep %d partials\n", n); std::abort(); }
        n_partials = n;
        return !refuse_keeping;
    }
    std::vector<int> steps_done;        // per chunk: steps whose accumulators are saved, or -1 if the result is stored
    std::vector<std::vector<std::string>> saved;      // per chunk: accumulators saved by the last segment
    std::vector<std::vector<std::string>> kept;       // per chunk: kept partial results
    std::vector<std::string> result;                  // per chunk: what was stored
    uint64_t last_version = 0;
    long launches = 0, kept_reads = 0, kept_writes = 0;
    int launch(const std::vector<Entry> &prog, uint64_t version, int64_t c0, int64_t c1, int t0, int t1, bool final,
               int live_before, int live_after) override
    {
        if (!(0 <= c0 && c0 < c1 && c1 <= C)) { std::printf("bad chunk range\n"); std::abort(); }
        if (!(0 <= t0 && t0 <= t1 && t1 <= (int)prog.size())) { std::printf("bad step range\n"); std::abort(); }
        if (final != (t1 == (int)prog.size())) { std::printf("final flag\n"); std::abort(); }
        if (t0 == t1 && !(final && t0 > 0)) { std::printf("empty launch\n"); std::abort(); }
        const bool aux = (version >> 63) != 0;       // a program built for keeping / reusing partials
        if (!aux) {
            if (version < last_version) { std::printf("version went back\n"); std::abort(); }
            last_version = version;
        }
        for (int t = t0; t < t1; ++t) {
            const Entry &e = prog[(size_t)t];
            if ((e.obj < 0 || e.save >= 0) && !(aux && t0 == 0 && final && n_partials > 0 && !refuse_keeping)) { std::printf("partial in a plain launch\n"); std::abort(); }
            kept_reads += e.obj < 0;
            kept_writes += e.save >= 0;
        }
        // accumulator bookkeeping: what is restored must be what was saved
        int level = t0 > 0 ? (int)prog[(size_t)t0 - 1].level - (int)prog[(size_t)t0 - 1].n_fold : -1;
        if (live_before != level + 1) { std::printf("live_before\n"); std::abort(); }
        for (int t = t0; t < t1; ++t) {
            const Entry &e = prog[(size_t)t];
            if (e.set ? (int)e.level != level + 1 : (int)e.level != level) { std::printf("level discipline\n"); std::abort(); }
            level = (int)e.level - (int)e.n_fold;
            if (level < 0) { std::printf("fold below zero\n"); std::abort(); }
        }
        if (final ? (level != 0 || live_after != 0) : live_after != level + 1) { std::printf("live_after\n"); std::abort(); }
        for (int64_t c = c0; c < c1; ++c) {
            const int have = steps_done[(size_t)c];
            if (t0 == 0 ? false : have != t0) { std::printf("resume from %d but chunk has %d\n", t0, have); std::abort(); }
            steps_done[(size_t)c] = final ? -1 : t1;
            std::vector<std::string> acc(t0 > 0 ? saved[(size_t)c] : std::vector<std::string>()), after;
            kept[(size_t)c].resize(16);
            const std::vector<std::string> before(kept[(size_t)c]);
            const std::string r = sym_eval(prog, t0, t1, acc, &before, &kept[(size_t)c], &after);
            if (final) result[(size_t)c] = r;
            else saved[(size_t)c] = after;
        }
        ++launches;
        return HOP_OK;
    }
};

struct CheckingBcast : BcastBackend {
    int64_t C = 0;
    std::map<int, int64_t> have;
    int copy(int from, int to, int64_t c0, int64_t c1) override
    {
        if (from == to || to < 1 || c0 >= c1 || c1 > C) { std::printf("bad copy\n"); std::abort(); }
        if (have[to] != c0) { std::printf("receiver %d has %ld, copy starts at %ld\n", to, (long)have[to], (long)c0); std::abort(); }
        if (from != 0 && have[from] < c1) { std::printf("sender lacks the chunks\n"); std::abort(); }
        have[to] = c1;
        return HOP_OK;
    }
};

static void fuzz_bcast(std::mt19937_64 &rng)
{
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (uint64_t)(hi - lo + 1)); };
    CheckingBcast be;
    be.C = rnd(1, 8);
    BcastScheduler s(be.C, &be);
    int64_t src = 0;
    const int ops = rnd(1, 60);
    for (int i = 0; i < ops; ++i) {
        const int what = rnd(0, 9);
        if (what < 3) { src = std::min<int64_t>(be.C, src + rnd(0, 2)); if (s.source_ready(src) != HOP_OK) std::abort(); }
        else if (what < 6) { int sender; s.join(&sender); }
        else if (what == 6 && s.n_copies() > 1) s.fail(rnd(1, s.n_copies() - 1));
        else if (s.step(rnd(0, 2)) < 0) std::abort();
        for (int a = 1; a < s.n_copies(); ++a)
            for (int b2 = a + 1; b2 < s.n_copies(); ++b2)
                if (s.sender_of(a) >= 0 && s.sender_of(a) == s.sender_of(b2)) { std::printf("two receivers on one sender\n"); std::abort(); }
    }
    s.source_ready(be.C);
    if (s.drain() < 0 || !s.all_complete()) { std::printf("broadcast did not complete\n"); std::abort(); }
}

// The marking of step groups (hop_program.h): a marked group must be eight plain combines into one
// level and start a multiple of eight steps from the program's start, every such group must be
// marked, and a walk that takes marked groups in one go (as the small-tile kernel does) must build
// the same expression, parenthesis for parenthesis, as the walk that looks at every control word.
static std::string walk(const std::vector<DevEntry> &p, bool use_marks)
{
    std::vector<std::string> acc(HOP_MAX_DEPTH + 1);
    auto term = [&](size_t t) { return "x" + std::to_string((size_t)(uintptr_t)p[t].src); };
    auto one = [&](size_t t) {
        uint32_t level = p[t].ctl & 0xffu, n_fold = p[t].ctl >> 16;
        const bool set = (p[t].ctl >> 8) & 1u;
        acc[level] = set ? term(t) : "(" + acc[level] + "+" + term(t) + ")";
        for (; n_fold; --n_fold, --level) acc[level - 1] = "(" + acc[level - 1] + "+" + acc[level] + ")";
    };
    size_t t = 0;
    for (; t + kRunSteps <= p.size(); t += kRunSteps) {
        if (use_marks && (p[t].ctl & kRunBit)) {
            const uint32_t level = p[t].ctl & 0xffu;
            for (int u = 0; u < kRunSteps; ++u) acc[level] = "(" + acc[level] + "+" + term(t + (size_t)u) + ")";
        } else {
            for (int u = 0; u < kRunSteps; ++u) one(t + (size_t)u);
        }
    }
    for (; t < p.size(); ++t) one(t);
    return acc[0];
}
static void check_marks(const std::vector<Entry> &prog)
{
    std::vector<DevEntry> p(prog.size());
    for (size_t t = 0; t < prog.size(); ++t) {
        p[t].src = (const void *)(uintptr_t)(t + 1);
        p[t].ctl = (uint32_t)prog[t].level | ((uint32_t)prog[t].set << 8) | ((uint32_t)prog[t].n_fold << 16);
        p[t].aux = 0;
    }
    const std::string plain = walk(p, false);
    mark_runs(p.data(), p.size());
    for (size_t t = 0; t < p.size(); ++t) {
        bool all_plain = t % kRunSteps == 0 && t + kRunSteps <= p.size();
        for (int u = 0; all_plain && u < kRunSteps; ++u)
            all_plain = prog[t + (size_t)u].set == 0 && prog[t + (size_t)u].n_fold == 0 && prog[t + (size_t)u].level == prog[t].level;
        if (((p[t].ctl & kRunBit) != 0) != all_plain) { std::printf("run mark wrong at step %zu\n", t); std::abort(); }
        if ((p[t].ctl & ~kRunBit) != ((uint32_t)prog[t].level | ((uint32_t)prog[t].set << 8) | ((uint32_t)prog[t].n_fold << 16))) std::abort();
    }
    if (walk(p, true) != plain) { std::printf("marked walk builds another expression\n"); std::abort(); }
}

// The one-launch table of a program, run as the kernel runs it: pass by pass, values in numbered places; no
// place is written while its value is still unread or is read in the same pass, every read finds a value of
// an earlier pass, the padding is the identity's place, and the result is the program's. Returns 1 if the
// program has such a table.
static long check_skeleton(const std::vector<Entry> &prog)
{

            ChainFormat f;
            f.min_cut = 1 + (int)(prog.size() % 6);
            f.max_items = 2 + (int)(prog.size() % 23);
            f.record_words = f.max_items + 1 + (int)(prog.size() % 3);
            f.teams = 1 + (int)(prog.size() % 7);
            f.value_bytes = 16u << (prog.size() % 3);
            f.max_values = 1 << 20;
            f.max_passes = 1 << 20;
            ChainSkeleton sk;
            if (build_chain_skeleton(prog, f, sk)) {
                const std::string want = sym_eval(prog, 0, (int)prog.size(), {}, nullptr, nullptr, nullptr);
                std::vector<std::string> place((size_t)sk.n_slots);
                std::vector<int> written_in((size_t)sk.n_slots, -1);
                std::string result;
                bool has_result = false;
                if (sk.table.size() != (size_t)sk.n_chains * (size_t)f.record_words || sk.pass_begin.back() != (uint32_t)sk.n_chains) { std::printf("table size\n"); std::abort(); }
                for (size_t pass = 0; pass + 1 < sk.pass_begin.size(); ++pass) {
                    std::vector<std::pair<size_t, std::string>> writes;
                    std::vector<size_t> reads;
                    for (uint32_t c = sk.pass_begin[pass]; c < sk.pass_begin[pass + 1]; ++c) {
                        const uint64_t *rec = sk.table.data() + (size_t)c * (size_t)f.record_words;
                        std::string acc;
                        bool padding = false;
                        for (int t = 1; t < f.record_words; ++t) {
                            const uint64_t w = rec[t];
                            std::string x;
                            if (w & kSkeletonObject) x = "o" + std::to_string(w & ~kSkeletonObject);
                            else {
                                if (w % f.value_bytes) { std::printf("offset\n"); std::abort(); }
                                const size_t sl = (size_t)(w / f.value_bytes);
                                if (sl == (size_t)sk.n_slots) { padding = true; continue; }       // the identity
                                if (sl > (size_t)sk.n_slots || written_in[sl] < 0 || written_in[sl] >= (int)pass || place[sl].empty()) { std::printf("reads a place nothing was put in\n"); std::abort(); }
                                x = place[sl];
                                reads.push_back(sl);
                            }
                            if (padding) { std::printf("an item behind the padding\n"); std::abort(); }
                            acc = t == 1 ? x : "(" + acc + "+" + x + ")";
                        }
                        if (rec[0] == f.result_mark) { result = acc; has_result = true; if (c + 1 != (uint32_t)sk.n_chains) { std::printf("result is not last\n"); std::abort(); } }
                        else writes.emplace_back((size_t)(rec[0] / f.value_bytes), acc);
                    }
                    for (size_t sl : reads) place[sl].clear();                                // read exactly once
                    for (auto &wv : writes) {
                        if (wv.first >= (size_t)sk.n_slots || !place[wv.first].empty()) { std::printf("writes over a live value\n"); std::abort(); }
                        for (size_t sl : reads) if (sl == wv.first) { std::printf("writes a place read in the same pass\n"); std::abort(); }
                        place[wv.first] = wv.second;
                        written_in[wv.first] = (int)pass;
                    }
                }
                if (!has_result || result != want) { std::printf("the table gives %s, the program %s\n", result.c_str(), want.c_str()); std::abort(); }
                return 1;
            }
            return 0;
}

int main(int argc, char **argv)
{
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 3000;
    std::mt19937_64 rng(12345);
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (uint64_t)(hi - lo + 1)); };
    long total_launches = 0, total_kept_reads = 0, total_kept_writes = 0, total_chains = 0, total_tables = 0;
    for (int r = 0; r < rounds; ++r) {
        const int n = rnd(1, 40), k = rnd(1, n);
        const int degs[] = {1, 2, 3, 4, 8, 16, n + 1};
        const int64_t d = degs[rnd(0, 6)];
        const int64_t C = rnd(1, 9);
        CheckingBackend be;
        be.C = C;
        be.steps_done.assign((size_t)C, 0);
        be.saved.assign((size_t)C, {});
        be.kept.assign((size_t)C, {});
        be.result.assign((size_t)C, "");
        be.refuse_keeping = rnd(0, 9) == 0;
        Scheduler s(n, k, C, d, &be);
        s.set_retention(rnd(0, 4) != 0, rnd(1, 3), rnd(0, 1) ? 4 : 2);
        s.set_eager(rnd(0, 3) ? 0 : rnd(1, 3));
        if (rnd(0, 2) == 0) { be.rng = &rng; s.set_adaptive(true); }
        std::vector<int> order((size_t)n);
        for (int i = 0; i < n; ++i) order[(size_t)i] = i;
        std::shuffle(order.begin(), order.end(), rng);
        std::vector<int64_t> progress((size_t)n, -1);
        std::vector<int> active;
        size_t next = 0;
        int guard = 0;
        while ((next < order.size() || !active.empty()) && ++guard < 100000) {
            if (next < order.size() && (active.empty() || rnd(0, 9) < 4)) {
                const int a = order[next++];
                if (rnd(0, 19) == 0) continue;                       // never shows up
                progress[(size_t)a] = 0;
                active.push_back(a);
                if (s.on_ready(a, 0) != HOP_OK) std::abort();
            } else {
                const size_t pick = (size_t)rnd(0, (int)active.size() - 1);
                const int a = active[pick];
                const int what = rnd(0, 19);
                if (what == 0) {                                     // fails
                    if (s.on_fail(a) != HOP_OK) std::abort();
                    active.erase(active.begin() + (long)pick);
                } else if (what == 1) {                              // stalls for good
                    active.erase(active.begin() + (long)pick);
                } else {
                    progress[(size_t)a] = std::min<int64_t>(C, progress[(size_t)a] + rnd(1, 3));
                    if (s.on_ready(a, progress[(size_t)a]) != HOP_OK) std::abort();
                    if (progress[(size_t)a] == C) active.erase(active.begin() + (long)pick);
                }
            }
            if (s.pump() < 0) std::abort();
            // invalid calls must be refused without damage
            if (s.on_ready(-1, 0) != HOP_ERR_INVALID || s.on_ready(n, 0) != HOP_ERR_INVALID || s.on_fail(n) != HOP_ERR_INVALID)
                std::abort();
        }
        hop_info_t info;
        const int rc = s.finish(&info);
        if (rc == HOP_OK || rc == HOP_PARTIAL) {
            for (int64_t c = 0; c < C; ++c)
                if (be.steps_done[(size_t)c] != -1) { std::printf("chunk %ld not stored (round %d)\n", (long)c, r); std::abort(); }
            if (info.k_eff < 1 || info.k_eff > k || (rc == HOP_OK) != (info.k_eff == k)) std::abort();
            // every chunk holds the expression of the final tree, whatever was kept and reused on the way
            Tree ft;
            ft.shape(k, d);
            std::vector<Entry> fp;
            compile_program(ft, s.occupants(), fp);
            const std::string want = sym_eval(fp, 0, (int)fp.size(), {}, nullptr, nullptr, nullptr);
            for (int64_t c = 0; c < C; ++c)
                if (be.result[(size_t)c] != want) {
                    std::printf("round %d chunk %ld holds %s, the tree says %s\n", r, (long)c, be.result[(size_t)c].c_str(), want.c_str());
                    std::abort();
                }
            if (info.partial_loads < 0 || (info.partial_loads > 0) != (be.kept_reads > 0) || (info.partial_stores > 0) != (be.kept_writes > 0)) std::abort();
            total_kept_reads += be.kept_reads;
            total_kept_writes += be.kept_writes;
        } else if (rc != HOP_ERR_NO_SURVIVOR) {
            std::printf("unexpected status %d\n", rc);
            std::abort();
        }
        total_launches += be.launches;
        // the program cutter on whatever tree this was
        Tree tr;
        tr.build(k, d);
        std::vector<int32_t> occ((size_t)k);
        for (int t = 0; t < k; ++t) occ[(size_t)t] = rnd(0, 9) ? t : -1;
        std::vector<Entry> prog;
        compile_program(tr, occ, prog);
        check_marks(prog);
        MultiPlan mp;
        { const int lo = rnd(1, 6); plan_passes(prog, (size_t)rnd(1, 40), lo, lo + rnd(0, 30), mp); }
        // the same program as chains: the last chain's expression, with every chain's value written out, is
        // the program's, parenthesis for parenthesis; chains read only values of earlier passes
        {
            ChainPlan cp;
            const int max_items = 2 + (int)(prog.size() % 29);
            const bool ok = plan_chains(prog, 1 + (int)(prog.size() % 8), max_items, cp);
            if (ok != (prog.size() >= 2)) { std::printf("plan_chains: %d for %zu steps\n", (int)ok, prog.size()); std::abort(); }
            if (ok) {
                std::vector<std::string> value(cp.n_chains());
                for (size_t g = 0; g < cp.n_chains(); ++g) {
                    std::string acc;
                    for (int32_t t = cp.begin[g]; t < cp.begin[g + 1]; ++t) {
                        const int32_t item = cp.items[(size_t)t];
                        if (item < 0 && ((size_t)(-item - 1) >= g || cp.pass[(size_t)(-item - 1)] >= cp.pass[g])) { std::printf("chain reads ahead\n"); std::abort(); }
                        const std::string x = item >= 0 ? "o" + std::to_string(item) : value[(size_t)(-item - 1)];
                        acc = t == cp.begin[g] ? x : "(" + acc + "+" + x + ")";
                    }
                    if (cp.begin[g + 1] - cp.begin[g] > max_items || cp.begin[g + 1] - cp.begin[g] < 2) { std::printf("chain length\n"); std::abort(); }
                    value[g] = acc;
                }
                const std::string want = sym_eval(prog, 0, (int)prog.size(), {}, nullptr, nullptr, nullptr);
                if (value.back() != want) { std::printf("chains give %s, the program %s\n", value.back().c_str(), want.c_str()); std::abort(); }
                total_chains += (long)cp.n_chains();
            }
        }
        total_tables += check_skeleton(prog);
        if (r % 8 == 0) {
            // larger trees, where the form pays
            std::mt19937_64 own((uint64_t)r * 7919 + 1);           // a generator of its own: the sessions' stream stays as it is
            Tree big;
            const int bk = 40 + (int)(own() % 660);
            big.build(bk, 2 + (int64_t)(own() % 23));
            std::vector<int32_t> bocc((size_t)bk);
            for (int t = 0; t < bk; ++t) bocc[(size_t)t] = own() % 20 ? t : -1;
            std::vector<Entry> bprog;
            compile_program(big, bocc, bprog);
            total_tables += check_skeleton(bprog);
        }
        fuzz_bcast(rng);
    }
    if (rounds >= 1000 && (total_kept_reads < 50 || total_kept_writes < 200)) { std::printf("keeping was hardly exercised: %ld reads, %ld writes\n", total_kept_reads, total_kept_writes); return 1; }
    std::printf("ok %d sessions, %ld launches, %ld partials kept, %ld reused, %ld chains, %ld tables\n", rounds, total_launches, total_kept_writes, total_kept_reads, total_chains, total_tables);
    return 0;
}
