// Host-side preparation of a character automaton for the compile stage: range check, the order in
// which the kernel's lanes take the states, and the default-chain jump tables.  Plain C++, run
// once per constraint by tdfa_dfa_create.  The jump tables are values of delta* themselves (the
// state after m clean bytes), which the kernel copies into the table for tokens made of clean
// bytes only: that part of the method's arithmetic is done here, per constraint, and not per
// table entry.  The passes that read the whole automaton run on a few host threads.
//
// Default chains.  For a state q let dflt(q) be the target that most of its live bytes lead to and
// C(q) the set of bytes that lead there ("clean" bytes).  States with the same clean set C form a
// class.  For a state s call c_C(s) the common target of s on all bytes of C, if there is one.  By
// induction over the bytes, a token whose first m bytes all lie in C takes a state q of class C to
// c_C^m(q), whatever those bytes are: delta*(q, d(t)) of Section 2.4 restricted to such a prefix
// depends on its length only.  Counter-like subautomata (a bounded string body, an identifier
// loop) are exactly of this kind.  The plan lists, for the largest classes, J[m][q] = c_C^m(q)
// for m = 1 .. kJumpDepth, and keeps only the states for which every J[m][q] exists.
#include <algorithm>
#include <array>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <new>
#include <thread>

#include "tdfa_internal.h"

namespace tdfa {

namespace {

constexpr int32_t kUnset = -3, kNone = -2;   // memo marks; -1 is DEAD
constexpr unsigned kMaxHostThreads = 16;

struct Candidate {
    std::array<uint32_t, 8> clean;
    std::vector<int32_t> states;
};

// What the first pass keeps of a state.
struct StateFacts {
    std::array<uint32_t, 8> live;      // bit b set = a transition on byte b
    std::array<uint32_t, 8> clean;     // bit b set = byte b leads to the most frequent target (if it has two bytes or more)
    uint64_t clean_hash;
    int32_t n_live;
    int32_t has_clean;
};

// A few host threads (at most 16 with the caller's) that stay around between calls (starting them costs about as much as
// the whole plan of a 5,000-state automaton).  run(n, task) calls task(0) .. task(n - 1), the caller
// taking its share, and returns when all are done; calls from several threads take turns.  The
// workers are never joined: they sleep on a condition variable for the life of the process.
class Workers {
public:
    static Workers& get()
    {
        static Workers* w = new Workers;
        return *w;
    }
    unsigned size() const { return n_workers_ + 1; }
    void run(unsigned n_tasks, const std::function<void(unsigned)>& task)
    {
        if (n_tasks == 0) return;
        if (n_tasks == 1 || n_workers_ == 0) {
            for (unsigned i = 0; i < n_tasks; ++i) task(i);
            return;
        }
        std::lock_guard<std::mutex> turn(turn_);
        {
            std::lock_guard<std::mutex> lock(m_);
            task_ = &task;
            n_tasks_ = n_tasks;
            next_ = 0;
            pending_ = n_tasks;
            ++epoch_;
        }
        work_.notify_all();
        take_tasks();
        std::unique_lock<std::mutex> lock(m_);
        done_.wait(lock, [&] { return pending_ == 0; });
        task_ = nullptr;
    }

private:
    Workers()
    {
        const unsigned hw = std::max(1u, std::thread::hardware_concurrency());
        n_workers_ = std::min(kMaxHostThreads, hw) - 1;
        for (unsigned i = 0; i < n_workers_; ++i) std::thread([this] { loop(); }).detach();
    }
    void take_tasks()
    {
        for (;;) {
            unsigned i;
            const std::function<void(unsigned)>* task;
            {
                std::lock_guard<std::mutex> lock(m_);
                if (!task_ || next_ >= n_tasks_) return;
                i = next_++;
                task = task_;
            }
            (*task)(i);
            std::lock_guard<std::mutex> lock(m_);
            if (--pending_ == 0) done_.notify_all();
        }
    }
    void loop()
    {
        uint64_t seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> lock(m_);
                work_.wait(lock, [&] { return epoch_ != seen; });
                seen = epoch_;
            }
            take_tasks();
        }
    }
    std::mutex turn_, m_;
    std::condition_variable work_, done_;
    const std::function<void(unsigned)>* task_ = nullptr;
    unsigned n_tasks_ = 0, next_ = 0, pending_ = 0, n_workers_ = 0;
    uint64_t epoch_ = 0;
};

// Runs fn(first, last, part) over [0, n) in at most kMaxHostThreads parts on the host threads; small inputs
// stay on the caller's.
template <class Fn>
void over_states(int32_t n, Fn fn)
{
    unsigned n_parts = n < 2048 ? 1u : Workers::get().size();
    if (n_parts == 1) {
        fn(0, n, 0u);
        return;
    }
    const int32_t per = (n + (int32_t)n_parts - 1) / (int32_t)n_parts;
    Workers::get().run(n_parts, [&](unsigned t) {
        const int32_t first = std::min(n, (int32_t)t * per), last = std::min(n, first + per);
        fn(first, last, t);
    });
}

int build_plan(const int32_t* trans, int32_t n_states, StatePlan* plan)
{
    // First pass, one read of the automaton: range check, live bytes, the most frequent target
    // (lowest id on ties) and the bytes that lead to it.
    std::vector<StateFacts> facts((size_t)n_states);
    std::vector<int32_t> n_live((size_t)n_states);
    struct Bad { int32_t q = -1, b = 0, v = 0; };
    std::array<Bad, kMaxHostThreads> bad{};
    over_states(n_states, [&](int32_t first, int32_t last, unsigned t) {
        std::vector<int32_t> count((size_t)n_states, 0);
        for (int32_t q = first; q < last; ++q) {
            const int32_t* row = trans + (int64_t)q * 256;
            StateFacts& f = facts[(size_t)q];
            f.clean.fill(0u);
            // which bytes have a transition, and the range check, without a branch per byte
            int32_t lo = 0, hi = -1;
            for (int w = 0; w < 8; ++w) {
                uint32_t bits = 0;
                for (int k = 0; k < 32; ++k) {
                    const int32_t to = row[w * 32 + k];
                    bits |= (uint32_t)(to >= 0) << k;
                    lo = std::min(lo, to);
                    hi = std::max(hi, to);
                }
                f.live[(size_t)w] = bits;
            }
            if (lo < TDFA_DEAD || hi >= n_states) {
                for (int b = 0; b < 256; ++b)
                    if (row[b] < TDFA_DEAD || row[b] >= n_states) {
                        bad[t] = Bad{q, b, row[b]};
                        return;
                    }
            }
            // most frequent live target, lowest id on ties: over the live bytes only
            int live = 0;
            int32_t dflt = TDFA_DEAD, best = 0;
            for (int w = 0; w < 8; ++w)
                for (uint32_t m = f.live[(size_t)w]; m; m &= m - 1) {
                    const int32_t to = row[w * 32 + __builtin_ctz(m)];
                    ++live;
                    const int32_t c = ++count[(size_t)to];
                    if (c > best || (c == best && to < dflt)) {      // whoever ends with the highest count passes here last
                        best = c;
                        dflt = to;
                    }
                }
            f.n_live = live;
            n_live[(size_t)q] = live;
            f.has_clean = best >= 2;                         // a clean set of one byte gains nothing
            for (int w = 0; w < 8; ++w)
                for (uint32_t m = f.live[(size_t)w]; m; m &= m - 1) {
                    const int k = __builtin_ctz(m);
                    const int32_t to = row[w * 32 + k];
                    count[(size_t)to] = 0;
                    if (f.has_clean && to == dflt) f.clean[(size_t)w] |= 1u << k;
                }
            uint64_t h = 0x9E3779B97F4A7C15ull;
            if (f.has_clean)
                for (uint32_t w : f.clean) h = (h ^ w) * 0xFF51AFD7ED558CCDull, h ^= h >> 29;
            f.clean_hash = h;
        }
    });
    for (const Bad& e : bad)                                  // (thread ranges ascend, so this is the lowest bad state)
        if (e.q >= 0) return fail(TDFA_E_INVALID_ARG, "trans[%d][%d] = %d outside [-1, %d)", e.q, e.b, e.v, n_states);

    // Classes: states with the same clean set.  An open-addressed table of the distinct sets counts their
    // states; the states of the sets that are large enough are then collected, in ascending order.
    std::vector<Candidate> cand;
    {
        size_t n_slots = 64;
        while (n_slots < 2 * (size_t)n_states) n_slots <<= 1;
        std::vector<int32_t> slot_set(n_slots, -1), set_of((size_t)n_states, -1), set_first, set_count;
        for (int32_t q = 0; q < n_states; ++q) {
            const StateFacts& f = facts[(size_t)q];
            if (!f.has_clean) continue;
            size_t slot = (size_t)(f.clean_hash >> 20) & (n_slots - 1);
            while (slot_set[slot] >= 0 && facts[(size_t)set_first[(size_t)slot_set[slot]]].clean != f.clean) slot = (slot + 1) & (n_slots - 1);
            if (slot_set[slot] < 0) {
                slot_set[slot] = (int32_t)set_first.size();
                set_first.push_back(q);
                set_count.push_back(0);
            }
            set_of[(size_t)q] = slot_set[slot];
            ++set_count[(size_t)slot_set[slot]];
        }
        std::vector<int32_t> cand_of(set_first.size(), -1);
        for (size_t k = 0; k < set_first.size(); ++k)
            if (set_count[k] >= kMinJumpClass) {
                cand_of[k] = (int32_t)cand.size();
                cand.push_back(Candidate{facts[(size_t)set_first[k]].clean, {}});
                cand.back().states.reserve((size_t)set_count[k]);
            }
        if (!cand.empty())
            for (int32_t q = 0; q < n_states; ++q)
                if (set_of[(size_t)q] >= 0 && cand_of[(size_t)set_of[(size_t)q]] >= 0) cand[(size_t)cand_of[(size_t)set_of[(size_t)q]]].states.push_back(q);
    }
    // the largest classes, at most kMaxJumpClasses of them (ties: the class of the lowest state first)
    std::sort(cand.begin(), cand.end(), [](const Candidate& x, const Candidate& y) {
        return x.states.size() != y.states.size() ? x.states.size() > y.states.size() : x.states[0] < y.states[0];
    });
    if ((int)cand.size() > kMaxJumpClasses) cand.resize((size_t)kMaxJumpClasses);

    // Per candidate class, each on one of the host threads: the states whose chain of common targets exists
    // for kJumpDepth steps, and those targets.
    struct ClassJumps {
        std::vector<int32_t> ok;       // states that jump
        std::vector<int32_t> to;       // [ok.size()][kJumpDepth]
    };
    std::vector<ClassJumps> found(cand.size());
    auto follow_class = [&](size_t ci) {
        const Candidate& c = cand[ci];
        std::vector<int32_t> memo((size_t)n_states, kUnset);
        int first_clean = 0;
        while (!(c.clean[(size_t)(first_clean >> 5)] >> (first_clean & 31) & 1u)) ++first_clean;     // (a class has two clean bytes or more)
        auto common_target = [&](int32_t s) -> int32_t {     // c_C(s), kNone if the clean bytes disagree
            if (s < 0) return s;
            int32_t& known = memo[(size_t)s];
            if (known != kUnset) return known;
            // the target on the first clean byte, then: do all clean bytes agree with it?  (compared over
            // the whole row without a branch, which the compiler turns into vector compares)
            const int32_t* row = trans + (int64_t)s * 256;
            const int32_t t0 = row[first_clean];
            bool all = true;
            for (int w = 0; w < 8; ++w) {
                uint32_t agree = 0;
                for (int k = 0; k < 32; ++k) agree |= (uint32_t)(row[w * 32 + k] == t0) << k;
                all = all && (agree & c.clean[(size_t)w]) == c.clean[(size_t)w];
            }
            return known = all ? t0 : kNone;
        };
        ClassJumps& out = found[ci];
        for (int32_t q : c.states) {
            int32_t chain[kJumpDepth];
            int32_t s = q;
            for (int m = 0; m < kJumpDepth && s != kNone; ++m) chain[m] = s = common_target(s);
            if (s == kNone) continue;
            out.ok.push_back(q);
            out.to.insert(out.to.end(), chain, chain + kJumpDepth);
        }
    };
    if (cand.size() > 1 && n_states >= 1024) {
        Workers::get().run((unsigned)cand.size(), [&](unsigned ci) { follow_class(ci); });
    } else {
        for (size_t ci = 0; ci < cand.size(); ++ci) follow_class(ci);
    }
    std::vector<int32_t> jump_class((size_t)n_states, -1);   // class of the states that jump
    plan->n_classes = 0;
    plan->clean_set.clear();
    plan->jump.clear();
    std::vector<std::vector<int32_t>> members;
    for (size_t k = 0; k < cand.size(); ++k) {
        ClassJumps& f = found[k];
        if ((int)f.ok.size() < kMinJumpClass) continue;
        if (plan->jump.empty()) plan->jump.assign((size_t)kJumpDepth * (size_t)n_states, TDFA_DEAD);
        const int ci = plan->n_classes++;
        plan->clean_set.insert(plan->clean_set.end(), cand[k].clean.begin(), cand[k].clean.end());
        for (size_t i = 0; i < f.ok.size(); ++i) {
            const int32_t q = f.ok[i];
            jump_class[(size_t)q] = ci;
            for (int m = 0; m < kJumpDepth; ++m)
                plan->jump[(size_t)m * (size_t)n_states + (size_t)q] = f.to[i * (size_t)kJumpDepth + (size_t)m];
        }
        members.push_back(std::move(f.ok));
    }

    // How many (state, b1, b2) survive two bytes: sizes the lists of the sweep over prefixes.
    {
        std::array<int64_t, kMaxHostThreads> part{};
        over_states(n_states, [&](int32_t first, int32_t last, unsigned t) {
            int64_t total = 0;
            for (int32_t q = first; q < last; ++q) {
                const int32_t* row = trans + (int64_t)q * 256;
                for (int w = 0; w < 8; ++w)
                    for (uint32_t m = facts[(size_t)q].live[(size_t)w]; m; m &= m - 1) total += n_live[(size_t)row[w * 32 + __builtin_ctz(m)]];
            }
            part[t] = total;
        });
        plan->n_pairs = 0;
        for (int64_t v : part) plan->n_pairs += v;
    }

    // Order: the jump classes first, each padded to whole groups of 64 lanes (-1 = idle lane); then
    // the other states, those that accept many bytes first (wildcard-like states keep most tokens
    // alive, states that expect one literal kill most at once), each bucket in state order, which
    // keeps neighbours close in memory.  The lanes of a 64-state group then tend to stay alive, or
    // die, together.
    plan->order.clear();
    plan->group_class.clear();
    for (int ci = 0; ci < plan->n_classes; ++ci) {
        for (int32_t q : members[(size_t)ci]) plan->order.push_back(q);
        while (plan->order.size() % 64) plan->order.push_back(-1);
        plan->group_class.resize(plan->order.size() / 64, (int8_t)ci);
    }
    std::array<std::vector<int32_t>, 9> by_bucket;            // floor(log2(live + 1)): 0 .. 8
    for (int32_t q = 0; q < n_states; ++q) {
        if (jump_class[(size_t)q] >= 0) continue;
        const int live = facts[(size_t)q].n_live;
        int bk = 0;
        while ((live + 1) >> (bk + 1)) ++bk;
        by_bucket[(size_t)bk].push_back(q);
    }
    for (int bk = 8; bk >= 0; --bk)
        plan->order.insert(plan->order.end(), by_bucket[(size_t)bk].begin(), by_bucket[(size_t)bk].end());
    plan->group_class.resize((plan->order.size() + 63) / 64, (int8_t)-1);
    // per group: the bytes on which at least one of its states moves on
    plan->group_live.assign(plan->group_class.size() * 8, 0u);
    for (size_t i = 0; i < plan->order.size(); ++i) {
        const int32_t q = plan->order[i];
        if (q < 0) continue;
        uint32_t* live = plan->group_live.data() + i / 64 * 8;
        for (int w = 0; w < 8; ++w) live[w] |= facts[(size_t)q].live[(size_t)w];
    }
    return TDFA_OK;
}

}  // namespace

void host_tasks(unsigned n_tasks, const std::function<void(unsigned)>& task) { Workers::get().run(n_tasks, task); }

int make_state_plan(const int32_t* trans, int32_t n_states, StatePlan* plan)
{
    try {
        return build_plan(trans, n_states, plan);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
}

}  // namespace tdfa
