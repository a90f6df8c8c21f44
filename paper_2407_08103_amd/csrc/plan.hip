// Host-side preparation of a character automaton for the compile stage: range check, the order in
// which the kernel's lanes take the states, and the default-chain jump tables.  Plain C++, run
// once per constraint by tdfa_dfa_create.  The jump tables are values of delta* themselves (the
// state after m clean bytes), which the kernel copies into the table for tokens made of clean
// bytes only: that part of the method's arithmetic is done here, per constraint, and not per
// table entry.
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
#include <map>
#include <new>

#include "tdfa_internal.h"

namespace tdfa {

namespace {

constexpr int32_t kUnset = -3, kNone = -2;   // memo marks; -1 is DEAD

struct Candidate {
    std::array<uint32_t, 8> clean;
    std::vector<int32_t> states;
};

int build_plan(const int32_t* trans, int32_t n_states, StatePlan* plan)
{
    std::vector<int32_t> bucket((size_t)n_states);
    std::vector<int32_t> count((size_t)n_states, 0);
    std::map<std::array<uint32_t, 8>, std::vector<int32_t>> classes;
    for (int32_t q = 0; q < n_states; ++q) {
        const int32_t* row = trans + (int64_t)q * 256;
        int live = 0;
        for (int b = 0; b < 256; ++b) {
            if (row[b] < TDFA_DEAD || row[b] >= n_states)
                return fail(TDFA_E_INVALID_ARG, "trans[%d][%d] = %d outside [-1, %d)", q, b, row[b], n_states);
            if (row[b] >= 0) {
                ++live;
                ++count[(size_t)row[b]];
            }
        }
        int bk = 0;                                      // floor(log2(live + 1)): 0 .. 8
        while ((live + 1) >> (bk + 1)) ++bk;
        bucket[(size_t)q] = bk;
        int32_t dflt = TDFA_DEAD, best = 0;              // most frequent live target, lowest id on ties
        for (int b = 0; b < 256; ++b) {
            const int32_t t = row[b];
            if (t >= 0 && (count[(size_t)t] > best || (count[(size_t)t] == best && t < dflt))) {
                best = count[(size_t)t];
                dflt = t;
            }
        }
        for (int b = 0; b < 256; ++b)
            if (row[b] >= 0) count[(size_t)row[b]] = 0;
        if (best >= 2) {                                 // a clean set of one byte gains nothing
            std::array<uint32_t, 8> clean{};
            for (int b = 0; b < 256; ++b)
                if (row[b] == dflt) clean[(size_t)(b >> 5)] |= 1u << (b & 31);
            classes[clean].push_back(q);
        }
    }

    // the largest classes, at most kMaxJumpClasses of them
    std::vector<Candidate> cand;
    for (auto& kv : classes)
        if ((int)kv.second.size() >= kMinJumpClass) cand.push_back(Candidate{kv.first, std::move(kv.second)});
    classes.clear();
    std::stable_sort(cand.begin(), cand.end(),
                     [](const Candidate& x, const Candidate& y) { return x.states.size() > y.states.size(); });
    if ((int)cand.size() > kMaxJumpClasses) cand.resize((size_t)kMaxJumpClasses);

    std::vector<int32_t> jump_class((size_t)n_states, -1);   // class of the states that jump
    std::vector<int32_t> memo;
    plan->n_classes = 0;
    plan->clean_set.clear();
    plan->jump.clear();
    std::vector<std::vector<int32_t>> members;
    for (const Candidate& c : cand) {
        memo.assign((size_t)n_states, kUnset);
        auto common_target = [&](int32_t s) -> int32_t {     // c_C(s), kNone if the clean bytes disagree
            if (s < 0) return s;
            int32_t& m = memo[(size_t)s];
            if (m != kUnset) return m;
            const int32_t* row = trans + (int64_t)s * 256;
            int32_t t = kUnset;
            for (int b = 0; b < 256 && t != kNone; ++b)
                if (c.clean[(size_t)(b >> 5)] >> (b & 31) & 1u) t = (t == kUnset || t == row[b]) ? row[b] : kNone;
            return m = t;
        };
        std::vector<int32_t> ok;
        for (int32_t q : c.states) {
            int32_t s = q;
            for (int m = 0; m < kJumpDepth && s != kNone; ++m) s = common_target(s);
            if (s != kNone) ok.push_back(q);
        }
        if ((int)ok.size() < kMinJumpClass) continue;
        if (plan->jump.empty()) plan->jump.assign((size_t)kJumpDepth * (size_t)n_states, TDFA_DEAD);
        const int ci = plan->n_classes++;
        plan->clean_set.insert(plan->clean_set.end(), c.clean.begin(), c.clean.end());
        for (int32_t q : ok) {
            jump_class[(size_t)q] = ci;
            int32_t s = q;
            for (int m = 0; m < kJumpDepth; ++m) {
                s = common_target(s);
                plan->jump[(size_t)m * (size_t)n_states + (size_t)q] = s;
            }
        }
        members.push_back(std::move(ok));
    }

    // How many (state, b1, b2) survive two bytes: sizes the pair lists of pairs.hip.
    {
        std::vector<int32_t> n_live((size_t)n_states, 0);
        for (int32_t q = 0; q < n_states; ++q) {
            const int32_t* row = trans + (int64_t)q * 256;
            int c = 0;
            for (int b = 0; b < 256; ++b) c += row[b] >= 0;
            n_live[(size_t)q] = c;
        }
        int64_t total = 0;
        for (int32_t q = 0; q < n_states; ++q) {
            const int32_t* row = trans + (int64_t)q * 256;
            for (int b = 0; b < 256; ++b)
                if (row[b] >= 0) total += n_live[(size_t)row[b]];
        }
        plan->n_pairs = total;
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
    std::vector<int32_t> rest;
    for (int32_t q = 0; q < n_states; ++q)
        if (jump_class[(size_t)q] < 0) rest.push_back(q);
    std::stable_sort(rest.begin(), rest.end(),
                     [&](int32_t x, int32_t y) { return bucket[(size_t)x] > bucket[(size_t)y]; });
    plan->order.insert(plan->order.end(), rest.begin(), rest.end());
    plan->group_class.resize((plan->order.size() + 63) / 64, (int8_t)-1);
    // per group: the bytes on which at least one of its states moves on
    plan->group_live.assign(plan->group_class.size() * 8, 0u);
    for (size_t i = 0; i < plan->order.size(); ++i) {
        const int32_t q = plan->order[i];
        if (q < 0) continue;
        const int32_t* row = trans + (int64_t)q * 256;
        uint32_t* live = plan->group_live.data() + i / 64 * 8;
        for (int b = 0; b < 256; ++b)
            if (row[b] >= 0) live[b >> 5] |= 1u << (b & 31);
    }
    return TDFA_OK;
}

}  // namespace

int make_state_plan(const int32_t* trans, int32_t n_states, StatePlan* plan)
{
    try {
        return build_plan(trans, n_states, plan);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
}

}  // namespace tdfa
