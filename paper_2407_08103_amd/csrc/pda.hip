// Push-down constraints (Section 3; Algorithm 3) for gfx950: the token-accepting automaton
// P_{G o V} = P_G o T_V as a list of token edges, and the decode step that conditions the
// allowed set on each sequence's stack.
//
// compile   With a deterministic P_G, the token edges that leave state q on token t are the runs
//           of P_G over the bytes of t that start in q: epsilon edges before a byte belong to
//           that byte's step, the edge ends with the token's last byte (in T_V the closing edge
//           of the token's cycle carries the token label).  A run starts knowing nothing of the
//           stack, so its stack edit is symbolic: `need` = what the stack must end with (and
//           loses), `top` = what is then on top of it.  An edge of P_G whose pops reach below
//           `top` extends `need`; two such edges that differ in what they want below split the
//           run into two token edges.  One thread per (state, token) follows its runs, twice:
//           once to count its token edges, once (after a prefix sum) to write them, so the list
//           is sorted by state and token.
// step      The allowed set of Algorithm 3 depends on the state and on what the stack ends with.
//           The token edges of a state are sorted into classes by their pops (a state has a
//           handful: nothing, one bracket, the other bracket, ...), each class with a row of
//           allowed bits like a state of the regular case.  The allowed set of a sequence is
//           the OR of the rows of the classes whose pops its stack ends with.  On 16-bit logits
//           the ordinary decode step kernel (penalty, best allowed logit; it reads only the
//           logits that can matter where few tokens are allowed) finds those classes and ORs
//           their rows as it reads them; with fp32 logits or a penalised row to write, a launch
//           before it ORs them into one row per sequence.  Then the one edge of the chosen
//           token that matches the stack is traversed: state, pops off, pushes on.
//           A table with more than kMaxClasses classes in a state keeps no rows; its step scans
//           the edges of the state instead (one workgroup per sequence).
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "tdfa_internal.h"

struct tdfa_pda {
    int32_t n_states = 0, start = 0, n_edges = 0;
    int32_t* first = nullptr;       // device [n_states + 1]: edges of a state (sorted by source)
    int32_t* input = nullptr;       // device [n_edges]: byte or -1
    int32_t* dst = nullptr;
    int32_t* pop_begin = nullptr;   // device [n_edges + 1]
    int32_t* pop_syms = nullptr;
    int32_t* push_begin = nullptr;
    int32_t* push_syms = nullptr;
    uint8_t* accept = nullptr;      // device [n_states]
};

struct tdfa_ptable {
    int32_t n_states = 0, n_tokens = 0;
    int64_t n_edges = 0;
    int64_t* edge_first = nullptr;  // device [n_states + 1]
    int32_t* token = nullptr;       // device [n_edges], ascending inside a state
    int32_t* dst = nullptr;
    int32_t* n_pops = nullptr;
    int32_t* pops = nullptr;        // device [n_edges][TDFA_PDA_STRING], bottom to top, unused places -1
    int32_t* n_push = nullptr;
    int32_t* pushes = nullptr;
    // classes of edges by their pops, per state; n_class_rows == 0: none kept
    int32_t n_class_rows = 0;
    int64_t row_words = 0;          // 32-bit words per row of allowed bits
    int32_t* class_first = nullptr; // device [n_states + 1]
    int32_t* class_n_pops = nullptr;// device [n_class_rows]
    int32_t* class_pops = nullptr;  // device [n_class_rows][TDFA_PDA_STRING], top of the stack first
    uint32_t* class_bits = nullptr; // device [n_class_rows][row_words]
    // per-step rows (one per sequence) and the identity map onto them, grown outside stream capture
    mutable uint32_t* step_allow = nullptr;
    mutable int32_t* step_rows = nullptr;       // [cap]: 0, 1, 2, ...
    mutable int32_t* step_unused = nullptr;     // [cap]: receives the step kernel's state output
    mutable int32_t step_cap = 0;
    mutable std::vector<void*> retired;         // earlier, smaller buffers: a captured graph may still name them
};

namespace tdfa {
namespace {

constexpr int kStr = TDFA_PDA_STRING;
static_assert(kStr == tdfa::kPdaPops, "the step kernel reads a class's pops whole");
constexpr int kEpsRun = 64;          // longest run of epsilon edges before one byte
constexpr int kPending = 8;          // runs of one (state, token) that wait to be followed
enum { kErrString = 1, kErrEpsRun = 2, kErrPending = 4 };

struct PdaDev {
    const int32_t* first;
    const int32_t* input;
    const int32_t* dst;
    const int32_t* pop_begin;
    const int32_t* pop_syms;
    const int32_t* push_begin;
    const int32_t* push_syms;
    int32_t n_states;
};

// A run in progress: in state p before byte i of the token, after n_eps epsilon edges since the last byte.
struct Run {
    int32_t p, i, n_eps;
    int32_t n_need, n_top;
    int32_t need[kStr], top[kStr];
};

// The run after edge e: 1 = the edge can be taken (r updated), 0 = it cannot, -1 = a string outgrew kStr.
__device__ int take_edge(const PdaDev& a, int32_t e, Run& r)
{
    const int32_t* pops = a.pop_syms + a.pop_begin[e];
    const int n_pops = a.pop_begin[e + 1] - a.pop_begin[e];
    const int32_t* pushes = a.push_syms + a.push_begin[e];
    const int n_push = a.push_begin[e + 1] - a.push_begin[e];
    const int shared = min(n_pops, r.n_top);                  // symbols that come off `top`
    for (int j = 0; j < shared; ++j)
        if (pops[n_pops - 1 - j] != r.top[r.n_top - 1 - j]) return 0;
    const int below = n_pops - shared;                        // symbols wanted from under everything known
    if (below > 0) {
        if (r.n_need + below > kStr) return -1;
        for (int j = r.n_need - 1; j >= 0; --j) r.need[j + below] = r.need[j];
        for (int j = 0; j < below; ++j) r.need[j] = pops[j];
        r.n_need += below;
    }
    r.n_top -= shared;
    if (r.n_top + n_push > kStr) return -1;
    for (int j = 0; j < n_push; ++j) r.top[r.n_top + j] = pushes[j];
    r.n_top += n_push;
    return 1;
}

struct EdgeOut {
    int32_t* token;
    int32_t* dst;
    int32_t* n_pops;
    int32_t* pops;
    int32_t* n_push;
    int32_t* pushes;
};

// All runs of P_G from state q over the bytes of one token.  Returns the number of token edges; if
// `out` is given they are written from edge index `at` on.  Sets bits of *err on a limit.
__device__ int follow_token(const PdaDev& a, int32_t q, const uint8_t* bytes, int32_t len, int32_t token, const EdgeOut* out,
                            int64_t at, uint32_t* err)
{
    if (len <= 0) return 0;                                   // no cycle in T_V for an empty token
    Run pending[kPending];
    int n_pending = 1, found = 0;
    pending[0].p = q;
    pending[0].i = 0;
    pending[0].n_eps = 0;
    pending[0].n_need = 0;
    pending[0].n_top = 0;
    while (n_pending > 0) {
        Run r = pending[--n_pending];
        bool alive = true;
        while (alive && r.i < len) {
            const int32_t byte = bytes[r.i];
            // the edges of r.p that can be taken now: epsilon, or this byte; the first continues this
            // run, any other starts a run of its own (they differ in what they want below `need`)
            bool moved = false;
            Run next;
            for (int32_t e = a.first[r.p]; e < a.first[r.p + 1]; ++e) {
                const int32_t in = a.input[e];
                if (in != -1 && in != byte) continue;
                Run cand = r;
                const int ok = take_edge(a, e, cand);
                if (ok < 0) { atomicOr(err, (uint32_t)kErrString); return found; }
                if (!ok) continue;
                cand.p = a.dst[e];
                if (in == -1) {
                    if (++cand.n_eps > kEpsRun) { atomicOr(err, (uint32_t)kErrEpsRun); return found; }
                } else {
                    cand.n_eps = 0;
                    ++cand.i;
                }
                if (!moved) {
                    next = cand;
                    moved = true;
                } else {
                    if (n_pending >= kPending) { atomicOr(err, (uint32_t)kErrPending); return found; }
                    pending[n_pending++] = cand;
                }
            }
            if (moved) r = next;
            else alive = false;
        }
        if (!alive) continue;
        if (out) {
            const int64_t k = at + found;
            out->token[k] = token;
            out->dst[k] = r.p;
            out->n_pops[k] = r.n_need;
            out->n_push[k] = r.n_top;
            for (int j = 0; j < kStr; ++j) {
                out->pops[k * kStr + j] = j < r.n_need ? r.need[j] : -1;
                out->pushes[k * kStr + j] = j < r.n_top ? r.top[j] : -1;
            }
        }
        ++found;
    }
    return found;
}

// counts[q][t] = token edges of (q, t)
__global__ void __launch_bounds__(256)
pda_count_kernel(PdaDev a, const uint32_t* __restrict__ vwords, const uint32_t* __restrict__ voff, const uint32_t* __restrict__ vlen,
                 int32_t n_tokens, uint32_t* __restrict__ counts, uint32_t* err)
{
    const int32_t t = (int32_t)(blockIdx.x * 256 + threadIdx.x), q = (int32_t)blockIdx.y;
    if (t >= n_tokens) return;
    const uint8_t* bytes = reinterpret_cast<const uint8_t*>(vwords) + (size_t)voff[t] * 4;
    counts[(size_t)q * n_tokens + t] = (uint32_t)follow_token(a, q, bytes, (int32_t)vlen[t], t, nullptr, 0, err);
}

// One workgroup per state: counts[q][.] <- its exclusive prefix sums, row_total[q] <- the sum.
__global__ void __launch_bounds__(1024)
pda_row_scan_kernel(uint32_t* __restrict__ counts, int32_t n_tokens, unsigned long long* __restrict__ row_total)
{
    __shared__ uint32_t s_wave[16];
    __shared__ uint32_t s_carry;
    uint32_t* row = counts + (size_t)blockIdx.x * n_tokens;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < n_tokens; base += 1024) {
        const int i = base + (int)threadIdx.x;
        const uint32_t v = i < n_tokens ? row[i] : 0u;
        uint32_t incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const uint32_t o = __shfl_up(incl, s, 64);
            if (lane >= s) incl += o;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        uint32_t before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        if (i < n_tokens) row[i] = before + incl - v;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) row_total[blockIdx.x] = s_carry;
}

// edge_first <- exclusive prefix sums of row_total (one thread: there are few states)
__global__ void pda_state_scan_kernel(const unsigned long long* __restrict__ row_total, int32_t n_states, int64_t* __restrict__ edge_first)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int64_t acc = 0;
    for (int32_t q = 0; q < n_states; ++q) {
        edge_first[q] = acc;
        acc += (int64_t)row_total[q];
    }
    edge_first[n_states] = acc;
}

__global__ void __launch_bounds__(256)
pda_fill_kernel(PdaDev a, const uint32_t* __restrict__ vwords, const uint32_t* __restrict__ voff, const uint32_t* __restrict__ vlen,
                int32_t n_tokens, const uint32_t* __restrict__ offsets, const int64_t* __restrict__ edge_first, EdgeOut out,
                uint32_t* err)
{
    const int32_t t = (int32_t)(blockIdx.x * 256 + threadIdx.x), q = (int32_t)blockIdx.y;
    if (t >= n_tokens) return;
    const uint8_t* bytes = reinterpret_cast<const uint8_t*>(vwords) + (size_t)voff[t] * 4;
    follow_token(a, q, bytes, (int32_t)vlen[t], t, &out, edge_first[q] + (int64_t)offsets[(size_t)q * n_tokens + t], err);
}

// ---- decode step

__device__ __forceinline__ uint32_t order_key(uint32_t u)      // float bits -> unsigned key of the same order
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) u = 0xFF800000u;     // NaN ranks as -inf
    if ((u & 0x7FFFFFFFu) == 0) u = 0;                        // -0 equals +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct PdaStepArgs {
    const int64_t* edge_first;
    const int32_t* token;
    const int32_t* dst;
    const int32_t* n_pops;
    const int32_t* pops;
    const int32_t* n_push;
    const int32_t* pushes;
    int32_t n_states, n_tokens;
    const void* logits;
    int64_t row_stride;
    const int32_t* states;
    int32_t* stacks;
    int32_t* depths;
    int32_t stack_cap;
    int32_t* tokens;
    int32_t* new_states;
    void* masked_out;
};

template <bool BF16>
__global__ void __launch_bounds__(256)
pda_step_kernel(PdaStepArgs a)
{
    __shared__ unsigned long long s_best[4];
    __shared__ unsigned long long s_win;
    __shared__ long long s_edge;
    const int b = (int)blockIdx.x;
    const int32_t q = a.states[b];
    const int32_t depth = a.depths[b];
    int32_t* stack = a.stacks + (int64_t)b * a.stack_cap;
    const bool valid = q >= 0 && q < a.n_states && depth >= 0 && depth <= a.stack_cap;
    const int64_t e_lo = valid ? a.edge_first[q] : 0, e_hi = valid ? a.edge_first[q + 1] : 0;
    const uint16_t* row16 = static_cast<const uint16_t*>(a.logits) + (int64_t)b * a.row_stride;
    const uint32_t* row32 = static_cast<const uint32_t*>(a.logits) + (int64_t)b * a.row_stride;
    // the penalised row: everything -inf first, the allowed logits are put in by the scan (after the
    // barrier below); the row must not be the logits themselves
    if (a.masked_out) {
        if (BF16) {
            uint16_t* o = static_cast<uint16_t*>(a.masked_out) + (int64_t)b * a.row_stride;
            for (int t = threadIdx.x; t < a.n_tokens; t += 256) o[t] = 0xFF80u;
        } else {
            uint32_t* o = static_cast<uint32_t*>(a.masked_out) + (int64_t)b * a.row_stride;
            for (int t = threadIdx.x; t < a.n_tokens; t += 256) o[t] = 0xFF800000u;
        }
    }
    if (threadIdx.x == 0) s_edge = -1;
    __syncthreads();
    unsigned long long best = 0;
    long long best_edge = -1;
    // four edges per thread at a time: their lengths and tokens are requested together, then the pops of
    // those that have any, then the logits of those that match
    constexpr int kU = 4;
    for (int64_t e0 = e_lo + threadIdx.x; e0 < e_hi; e0 += 256 * kU) {
        int np[kU];
        int32_t tk[kU];
        bool ok[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int64_t e = e0 + 256 * u;
            ok[u] = e < e_hi;
            np[u] = ok[u] ? a.n_pops[e] : 0;
            tk[u] = ok[u] ? a.token[e] : 0;
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int64_t e = e0 + 256 * u;
            ok[u] = ok[u] && np[u] <= depth;
            for (int j = 0; ok[u] && j < np[u]; ++j) ok[u] = a.pops[e * kStr + j] == stack[depth - np[u] + j];
        }
        uint32_t bits[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) bits[u] = !ok[u] ? 0u : (BF16 ? (uint32_t)row16[tk[u]] << 16 : row32[tk[u]]);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!ok[u]) continue;
            if (a.masked_out) {
                if (BF16) static_cast<uint16_t*>(a.masked_out)[(int64_t)b * a.row_stride + tk[u]] = (uint16_t)(bits[u] >> 16);
                else static_cast<uint32_t*>(a.masked_out)[(int64_t)b * a.row_stride + tk[u]] = bits[u];
            }
            const unsigned long long cand = ((unsigned long long)order_key(bits[u]) << 32) | (0xFFFFFFFFu - (uint32_t)tk[u]);
            if (cand > best) {
                best = cand;
                best_edge = e0 + 256 * u;
            }
        }
    }
    // workgroup maximum of (key, lowest token); the thread that holds it names the edge
    unsigned long long m = best;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const unsigned long long o = __shfl_xor(m, s, 64);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0) s_best[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long w = s_best[0];
        for (int i = 1; i < 4; ++i) w = s_best[i] > w ? s_best[i] : w;
        s_win = w;
    }
    __syncthreads();
    const unsigned long long win = s_win;
    if (win != 0 && best == win) s_edge = best_edge;           // one edge per allowed token: a single writer
    __syncthreads();
    if (threadIdx.x != 0) return;
    if (win == 0) {
        a.tokens[b] = TDFA_NO_TOKEN;
        a.new_states[b] = valid ? q : TDFA_DEAD;
        return;
    }
    const long long e = s_edge;
    const int np = a.n_pops[e], nu = a.n_push[e];
    const int m_keep = depth - np;
    if (m_keep + nu > a.stack_cap) {                           // the stack would outgrow its buffer: the sequence ends
        a.tokens[b] = TDFA_NO_TOKEN;
        a.new_states[b] = TDFA_DEAD;
        return;
    }
    for (int j = 0; j < nu; ++j) stack[m_keep + j] = a.pushes[e * kStr + j];
    a.depths[b] = m_keep + nu;
    a.tokens[b] = (int32_t)(0xFFFFFFFFu - (uint32_t)win);
    a.new_states[b] = a.dst[e];
}

// ---- classes of a state's edges by their pops

constexpr int kMaxClasses = 64;

// One workgroup per state.  Round k takes the first edge that has no class yet, makes its pops class
// k, and gives class k to every edge with the same pops; the rounds end when no edge is left (or
// after kMaxClasses rounds: then too_many[q] is set).
__global__ void __launch_bounds__(256)
pda_classes_kernel(const int64_t* __restrict__ edge_first, const int32_t* __restrict__ n_pops, const int32_t* __restrict__ pops,
                   uint8_t* __restrict__ edge_class, int32_t* __restrict__ n_classes, int32_t* __restrict__ cls_n_pops,
                   int32_t* __restrict__ cls_pops, uint32_t* __restrict__ too_many)
{
    __shared__ unsigned long long s_first;
    __shared__ int32_t s_np, s_str[kStr];
    const int q = (int)blockIdx.x;
    const int64_t e_lo = edge_first[q], e_hi = edge_first[q + 1];
    int k = 0;
    for (; k < kMaxClasses; ++k) {
        if (threadIdx.x == 0) s_first = ~0ull;
        __syncthreads();
        for (int64_t e = e_lo + threadIdx.x; e < e_hi; e += 256)
            if (edge_class[e] == 0xFF) {
                atomicMin(&s_first, (unsigned long long)e);
                break;                                          // the thread's edges ascend: its first is its lowest
            }
        __syncthreads();
        const unsigned long long first = s_first;
        if (first == ~0ull) break;
        if (threadIdx.x == 0) {
            s_np = n_pops[first];
            cls_n_pops[q * kMaxClasses + k] = s_np;
            for (int j = 0; j < kStr; ++j) {
                const int32_t v = j < s_np ? pops[first * kStr + j] : -1;
                s_str[j] = v;
                cls_pops[((int64_t)q * kMaxClasses + k) * kStr + j] = v;
            }
        }
        __syncthreads();
        const int np = s_np;
        for (int64_t e = e_lo + threadIdx.x; e < e_hi; e += 256) {
            if (edge_class[e] != 0xFF || n_pops[e] != np) continue;
            bool same = true;
            for (int j = 0; same && j < np; ++j) same = pops[e * kStr + j] == s_str[j];
            if (same) edge_class[e] = (uint8_t)k;
        }
        __syncthreads();                                        // (also: s_first and s_str are rewritten next round)
    }
    if (threadIdx.x == 0) {
        n_classes[q] = k;
        if (k == kMaxClasses) {
            // any edge left without a class?
            bool left = false;
            for (int64_t e = e_lo; e < e_hi && !left; ++e) left = edge_class[e] == 0xFF;
            if (left) *too_many = 1u;
        }
    }
}

// The class tables of all states, end to end, and the rows of allowed bits (zero on entry).
__global__ void __launch_bounds__(256)
pda_class_rows_kernel(const int64_t* __restrict__ edge_first, const int32_t* __restrict__ token, const uint8_t* __restrict__ edge_class,
                      const int32_t* __restrict__ class_first, const int32_t* __restrict__ cls_n_pops,
                      const int32_t* __restrict__ cls_pops, int32_t* __restrict__ class_n_pops, int32_t* __restrict__ class_pops,
                      uint32_t* __restrict__ class_bits, int64_t row_words)
{
    const int q = (int)blockIdx.y;
    const int32_t r0 = class_first[q], n = class_first[q + 1] - r0;
    if (blockIdx.x == 0 && (int)threadIdx.x < n) {
        const int np = cls_n_pops[q * kMaxClasses + threadIdx.x];
        class_n_pops[r0 + threadIdx.x] = np;
        for (int j = 0; j < kStr; ++j)                              // kept top first: the step compares them with the top of a stack
            class_pops[(int64_t)(r0 + threadIdx.x) * kStr + j] =
                j < np ? cls_pops[((int64_t)q * kMaxClasses + threadIdx.x) * kStr + (np - 1 - j)] : -1;
    }
    const int64_t e_lo = edge_first[q], e_hi = edge_first[q + 1];
    for (int64_t e = e_lo + (int64_t)blockIdx.x * 256 + threadIdx.x; e < e_hi; e += (int64_t)gridDim.x * 256) {
        const int32_t t = token[e];
        atomicOr(&class_bits[(int64_t)(r0 + edge_class[e]) * row_words + (t >> 5)], 1u << (t & 31));
    }
}

// The row of allowed bits of each sequence for this step: the OR of its state's class rows whose
// pops the stack ends with; zero for a sequence whose state or depth is out of range.
__global__ void __launch_bounds__(256)
pda_allow_kernel(const int32_t* __restrict__ states, const int32_t* __restrict__ stacks, const int32_t* __restrict__ depths,
                 int32_t stack_cap, int32_t n_states, const int32_t* __restrict__ class_first,
                 const int32_t* __restrict__ class_n_pops, const int32_t* __restrict__ class_pops,
                 const uint32_t* __restrict__ class_bits, int64_t row_words, uint32_t* __restrict__ out_rows,
                 int32_t* __restrict__ row_ids)
{
    __shared__ unsigned long long s_match;
    const int b = (int)blockIdx.x;
    const int32_t q = states[b], depth = depths[b];
    const bool valid = q >= 0 && q < n_states && depth >= 0 && depth <= stack_cap;
    const int32_t r0 = valid ? class_first[q] : 0, n = valid ? class_first[q + 1] - r0 : 0;
    if (threadIdx.x == 0) {
        s_match = 0ull;
        row_ids[b] = b;
    }
    __syncthreads();
    // the top kStr symbols of the stack (top first) and a class's pops are read whole, not symbol by
    // symbol as the comparison goes: no read then waits for the outcome of another
    int32_t top[kStr];
    {
        const int32_t* stack = stacks + (int64_t)b * stack_cap;
#pragma unroll
        for (int j = 0; j < kStr; ++j) top[j] = valid && depth - 1 - j >= 0 ? stack[depth - 1 - j] : -1;
    }
    if ((int)threadIdx.x < n) {
        const int np = class_n_pops[r0 + threadIdx.x];
        int32_t pops[kStr];
#pragma unroll
        for (int j = 0; j < kStr; ++j) pops[j] = class_pops[(int64_t)(r0 + threadIdx.x) * kStr + j];
        bool ok = np <= depth;
#pragma unroll
        for (int j = 0; j < kStr; ++j)                              // (the class's pops are stored top first)
            if (j < np) ok = ok && pops[j] == top[j];
        if (ok) atomicOr(&s_match, 1ull << threadIdx.x);
    }
    __syncthreads();
    const unsigned long long match = s_match;
    const uint4* rows = reinterpret_cast<const uint4*>(class_bits);
    uint4* out = reinterpret_cast<uint4*>(out_rows) + (int64_t)b * (row_words >> 2);
    for (int64_t w = threadIdx.x; w < (row_words >> 2); w += 256) {
        uint4 acc = make_uint4(0, 0, 0, 0);
        for (unsigned long long m = match; m; m &= m - 1) {
            const uint4 v = rows[(int64_t)(r0 + __builtin_ctzll(m)) * (row_words >> 2) + w];
            acc.x |= v.x; acc.y |= v.y; acc.z |= v.z; acc.w |= v.w;
        }
        out[w] = acc;
    }
}

// The same rows for a table that has kept no class rows (a state with more classes than kMaxClasses): the
// edges of the sequence's state are scanned, and every edge whose pops the stack ends with sets its
// token's bit.  One workgroup per sequence.
__global__ void __launch_bounds__(256)
pda_allow_edges_kernel(const int32_t* __restrict__ states, const int32_t* __restrict__ stacks, const int32_t* __restrict__ depths,
                       int32_t stack_cap, int32_t n_states, const int64_t* __restrict__ edge_first, const int32_t* __restrict__ token,
                       const int32_t* __restrict__ n_pops, const int32_t* __restrict__ pops, int64_t row_words,
                       uint32_t* out_rows, int32_t* __restrict__ row_ids)
{
    const int b = (int)blockIdx.x;
    const int32_t q = states[b], depth = depths[b];
    const bool valid = q >= 0 && q < n_states && depth >= 0 && depth <= stack_cap;
    uint32_t* row = out_rows + (int64_t)b * row_words;
    for (int64_t w = threadIdx.x; w < (row_words >> 2); w += 256) reinterpret_cast<uint4*>(row)[w] = make_uint4(0, 0, 0, 0);
    if (threadIdx.x == 0) row_ids[b] = b;
    __syncthreads();                                          // (the zeros are written before any bit is set)
    if (!valid) return;
    const int32_t* stack = stacks + (int64_t)b * stack_cap;
    for (int64_t e = edge_first[q] + threadIdx.x; e < edge_first[q + 1]; e += 256) {
        const int np = n_pops[e];
        bool ok = np <= depth;
        for (int j = 0; ok && j < np; ++j) ok = pops[e * kStr + j] == stack[depth - np + j];
        if (ok) {
            const int32_t t = token[e];
            atomicOr(&row[t >> 5], 1u << (t & 31));
        }
    }
}

// After the step kernel has chosen the tokens: one wavefront per sequence finds the edge of its token
// that the stack matches and traverses it.  The edges of a state ascend by token; the wavefront
// narrows the range 64 probes at a time (three rounds for 25,000 edges, where a binary search by one
// thread would make seventeen dependent reads), then its first lanes test the few edges of the token.
__global__ void __launch_bounds__(256)
pda_advance_kernel(PdaStepArgs a, int32_t batch)
{
    const int lane = (int)threadIdx.x & 63;
    const int b = (int)(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (b >= batch) return;                                     // (whole wavefronts leave)
    const int32_t q = a.states[b], depth = a.depths[b], tok = a.tokens[b];
    const bool valid = q >= 0 && q < a.n_states && depth >= 0 && depth <= a.stack_cap;
    if (tok < 0 || !valid) {
        if (lane == 0) {
            a.tokens[b] = TDFA_NO_TOKEN;
            a.new_states[b] = valid ? q : TDFA_DEAD;
        }
        return;
    }
    int32_t* stack = a.stacks + (int64_t)b * a.stack_cap;
    // lo: no edge below it has token >= tok is false ... invariant: token[i] < tok for i < lo, token[i] >= tok for i >= hi
    int64_t lo = a.edge_first[q], hi = a.edge_first[q + 1];
    const int64_t e_hi = hi;
    while (hi - lo > 64) {
        const int64_t span = hi - lo;
        const int64_t pos = lo + (span * (lane + 1)) / 65;       // 64 probes strictly inside, ascending with the lane
        const bool ge = a.token[pos] >= tok;
        const unsigned long long m = __builtin_amdgcn_ballot_w64(ge);
        const int first = m ? (int)__builtin_ctzll(m) : 64;       // the first probe that is not below tok
        const int64_t new_hi = first < 64 ? lo + (span * (first + 1)) / 65 : hi;
        const int64_t new_lo = first > 0 ? lo + (span * first) / 65 + 1 : lo;
        lo = new_lo;
        hi = new_hi;
    }
    {
        const int64_t pos = lo + lane;
        const bool ge = pos < hi && a.token[pos] >= tok;
        const unsigned long long m = __builtin_amdgcn_ballot_w64(ge);
        lo = m ? lo + (int64_t)__builtin_ctzll(m) : hi;
    }
    // the edges of the token (a few: one per pops string): lane i tests edge lo + i
    long long e = -1;
    for (int64_t base = lo; base < e_hi && e < 0; base += 64) {
        const int64_t c = base + lane;
        bool mine = c < e_hi && a.token[c] == tok;
        const bool more = c < e_hi && a.token[c] == tok;         // (uniform exit below: edges of the token are contiguous)
        if (mine) {
            const int np = a.n_pops[c];
            mine = np <= depth;
            for (int j = 0; mine && j < np; ++j) mine = a.pops[c * kStr + j] == stack[depth - np + j];
        }
        const unsigned long long hit = __builtin_amdgcn_ballot_w64(mine);
        if (hit) e = (long long)(base + (int64_t)__builtin_ctzll(hit));
        if (__builtin_amdgcn_ballot_w64(more) != ~0ull) break;    // the token's edges end inside this batch
    }
    if (lane != 0) return;
    if (e < 0) {                                                // cannot happen: the token was allowed through such an edge
        a.tokens[b] = TDFA_NO_TOKEN;
        a.new_states[b] = TDFA_DEAD;
        return;
    }
    const int np = a.n_pops[e], nu = a.n_push[e];
    const int m_keep = depth - np;
    if (m_keep + nu > a.stack_cap) {                            // the stack would outgrow its buffer: the sequence ends
        a.tokens[b] = TDFA_NO_TOKEN;
        a.new_states[b] = TDFA_DEAD;
        return;
    }
    for (int j = 0; j < nu; ++j) stack[m_keep + j] = a.pushes[e * kStr + j];
    a.depths[b] = m_keep + nu;
    a.new_states[b] = a.dst[e];
}

template <typename T>
int dev_alloc(T** p, size_t count)
{
    *p = nullptr;
    TDFA_HIP(hipMalloc(reinterpret_cast<void**>(p), (count ? count : 1) * sizeof(T)));
    return TDFA_OK;
}

bool suffix_of(const int32_t* x, int nx, const int32_t* y, int ny)
{
    return nx <= ny && std::memcmp(x, y + (ny - nx), sizeof(int32_t) * (size_t)nx) == 0;
}

}  // namespace
}  // namespace tdfa

using namespace tdfa;

extern "C" {

int tdfa_pda_create(int32_t n_states, int32_t start, const uint8_t* accept, int32_t n_edges, const int32_t* src,
                    const int32_t* input, const int32_t* dst, const int32_t* pop_begin, const int32_t* pop_syms,
                    const int32_t* push_begin, const int32_t* push_syms, void* stream, tdfa_pda** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_states <= 0 || n_edges < 0) return fail(TDFA_E_INVALID_ARG, "n_states %d or n_edges %d out of range", n_states, n_edges);
    if (start < 0 || start >= n_states) return fail(TDFA_E_INVALID_ARG, "start %d outside [0, %d)", start, n_states);
    if (n_edges > 0 && (!src || !input || !dst)) return fail(TDFA_E_INVALID_ARG, "edge arrays NULL");
    if (!pop_begin || !push_begin) return fail(TDFA_E_INVALID_ARG, "pop_begin or push_begin is NULL");
    for (int32_t e = 0; e < n_edges; ++e) {
        if (src[e] < 0 || src[e] >= n_states || dst[e] < 0 || dst[e] >= n_states)
            return fail(TDFA_E_INVALID_ARG, "edge %d: source %d or target %d is no state", e, src[e], dst[e]);
        if (input[e] < -1 || input[e] > 255) return fail(TDFA_E_INVALID_ARG, "edge %d: input %d is neither a byte nor -1", e, input[e]);
        if (e > 0 && src[e] < src[e - 1]) return fail(TDFA_E_INVALID_ARG, "edges are not sorted by source state (edge %d)", e);
        const int np = pop_begin[e + 1] - pop_begin[e], nu = push_begin[e + 1] - push_begin[e];
        if (np < 0 || nu < 0 || np > TDFA_PDA_STRING || nu > TDFA_PDA_STRING)
            return fail(TDFA_E_INVALID_ARG, "edge %d: %d pops / %d pushes outside [0, %d]", e, np, nu, TDFA_PDA_STRING);
        if ((np > 0 && !pop_syms) || (nu > 0 && !push_syms)) return fail(TDFA_E_INVALID_ARG, "pop_syms or push_syms is NULL");
        for (int j = pop_begin[e]; j < pop_begin[e + 1]; ++j)
            if (pop_syms[j] < 0) return fail(TDFA_E_INVALID_ARG, "edge %d pops a negative symbol", e);
        for (int j = push_begin[e]; j < push_begin[e + 1]; ++j)
            if (push_syms[j] < 0) return fail(TDFA_E_INVALID_ARG, "edge %d pushes a negative symbol", e);
    }
    if (pop_begin[0] != 0 || push_begin[0] != 0) return fail(TDFA_E_INVALID_ARG, "pop_begin[0] and push_begin[0] must be 0");
    // Section 3.1: a non-deterministic automaton is an error.  Two edges of a state whose inputs can
    // meet (equal, or one of them epsilon) must not have pops of which one is a suffix of the other.
    for (int32_t e = 0; e < n_edges; ++e)
        for (int32_t f = e + 1; f < n_edges && src[f] == src[e]; ++f) {
            if (input[e] != input[f] && input[e] != -1 && input[f] != -1) continue;
            const int ne = pop_begin[e + 1] - pop_begin[e], nf = pop_begin[f + 1] - pop_begin[f];
            const int32_t* pe = pop_syms ? pop_syms + pop_begin[e] : nullptr;
            const int32_t* pf = pop_syms ? pop_syms + pop_begin[f] : nullptr;
            if (suffix_of(pe, ne, pf, nf) || suffix_of(pf, nf, pe, ne))
                return fail(TDFA_E_INVALID_ARG, "the automaton is not deterministic: edges %d and %d of state %d can both be taken", e, f,
                            src[e]);
        }
    tdfa_pda* p = new (std::nothrow) tdfa_pda;
    if (!p) return fail(TDFA_E_OOM, "host allocation failed");
    p->n_states = n_states;
    p->start = start;
    p->n_edges = n_edges;
    std::vector<int32_t> first;
    std::vector<uint8_t> acc;
    try {
        first.assign((size_t)n_states + 1, 0);
        acc.assign((size_t)n_states, 0);
    } catch (const std::bad_alloc&) {
        delete p;
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    for (int32_t e = 0; e < n_edges; ++e) ++first[(size_t)src[e] + 1];
    for (int32_t q = 0; q < n_states; ++q) first[(size_t)q + 1] += first[(size_t)q];
    if (accept)
        for (int32_t q = 0; q < n_states; ++q) acc[(size_t)q] = accept[q] ? 1 : 0;
    const size_t n_pop = (size_t)pop_begin[n_edges], n_push = (size_t)push_begin[n_edges];
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = dev_alloc(&p->first, first.size());
    if (rc == TDFA_OK) rc = dev_alloc(&p->input, (size_t)n_edges);
    if (rc == TDFA_OK) rc = dev_alloc(&p->dst, (size_t)n_edges);
    if (rc == TDFA_OK) rc = dev_alloc(&p->pop_begin, (size_t)n_edges + 1);
    if (rc == TDFA_OK) rc = dev_alloc(&p->pop_syms, n_pop);
    if (rc == TDFA_OK) rc = dev_alloc(&p->push_begin, (size_t)n_edges + 1);
    if (rc == TDFA_OK) rc = dev_alloc(&p->push_syms, n_push);
    if (rc == TDFA_OK) rc = dev_alloc(&p->accept, (size_t)n_states);
    auto up = [&](void* d, const void* h, size_t bytes) {
        if (rc == TDFA_OK && bytes > 0) {
            const hipError_t e = hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, s);
            if (e != hipSuccess) rc = fail(TDFA_E_DEVICE, "upload: %s", hipGetErrorString(e));
        }
    };
    up(p->first, first.data(), first.size() * 4);
    up(p->input, input, (size_t)n_edges * 4);
    up(p->dst, dst, (size_t)n_edges * 4);
    up(p->pop_begin, pop_begin, ((size_t)n_edges + 1) * 4);
    up(p->pop_syms, pop_syms, n_pop * 4);
    up(p->push_begin, push_begin, ((size_t)n_edges + 1) * 4);
    up(p->push_syms, push_syms, n_push * 4);
    up(p->accept, acc.data(), (size_t)n_states);
    if (rc == TDFA_OK) {
        const hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess) rc = fail(TDFA_E_DEVICE, "hipStreamSynchronize: %s", hipGetErrorString(e));
    }
    if (rc != TDFA_OK) {
        tdfa_pda_destroy(p);
        return rc;
    }
    *out = p;
    return TDFA_OK;
}

int tdfa_pda_destroy(tdfa_pda* p)
{
    if (!p) return TDFA_OK;
    for (void* d : {(void*)p->first, (void*)p->input, (void*)p->dst, (void*)p->pop_begin, (void*)p->pop_syms, (void*)p->push_begin,
                    (void*)p->push_syms, (void*)p->accept})
        if (d) (void)hipFree(d);
    delete p;
    return TDFA_OK;
}

int tdfa_compile_token_pda(const tdfa_vocab* vocab, const tdfa_pda* pda, void* stream, tdfa_ptable** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!vocab || !pda) return fail(TDFA_E_INVALID_ARG, "vocab or pda is NULL");
    if (pda->n_states > 65535) return fail(TDFA_E_UNSUPPORTED, "more than 65,535 states");
    VocabView v;
    vocab_view(vocab, &v);
    hipStream_t s = static_cast<hipStream_t>(stream);
    tdfa_ptable* t = new (std::nothrow) tdfa_ptable;
    if (!t) return fail(TDFA_E_OOM, "host allocation failed");
    t->n_states = pda->n_states;
    t->n_tokens = v.n_tokens;
    uint32_t* counts = nullptr;
    unsigned long long* row_total = nullptr;
    uint32_t* err = nullptr;
    int rc = dev_alloc(&counts, (size_t)pda->n_states * (size_t)std::max(v.n_tokens, 1));
    if (rc == TDFA_OK) rc = dev_alloc(&row_total, (size_t)pda->n_states);
    if (rc == TDFA_OK) rc = dev_alloc(&err, 1);
    if (rc == TDFA_OK) rc = dev_alloc(&t->edge_first, (size_t)pda->n_states + 1);
    PdaDev a{pda->first, pda->input, pda->dst, pda->pop_begin, pda->pop_syms, pda->push_begin, pda->push_syms, pda->n_states};
    auto check = [&](hipError_t e, const char* what) {
        if (rc == TDFA_OK && e != hipSuccess) rc = fail(e == hipErrorOutOfMemory ? TDFA_E_OOM : TDFA_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
    };
    const dim3 grid((unsigned)((std::max(v.n_tokens, 1) + 255) / 256), (unsigned)pda->n_states);
    uint32_t err_host = 0;
    int64_t n_edges = 0;
    if (rc == TDFA_OK) {
        check(hipMemsetAsync(err, 0, sizeof(uint32_t), s), "hipMemsetAsync");
        if (v.n_tokens > 0) {
            pda_count_kernel<<<grid, 256, 0, s>>>(a, v.words, v.off, v.len, v.n_tokens, counts, err);
            check(hipGetLastError(), "pda_count_kernel");
        }
        pda_row_scan_kernel<<<(unsigned)pda->n_states, 1024, 0, s>>>(counts, v.n_tokens, row_total);
        check(hipGetLastError(), "pda_row_scan_kernel");
        pda_state_scan_kernel<<<1, 64, 0, s>>>(row_total, pda->n_states, t->edge_first);
        check(hipGetLastError(), "pda_state_scan_kernel");
        check(hipMemcpyAsync(&n_edges, t->edge_first + pda->n_states, sizeof(int64_t), hipMemcpyDeviceToHost, s), "hipMemcpyAsync");
        check(hipMemcpyAsync(&err_host, err, sizeof(uint32_t), hipMemcpyDeviceToHost, s), "hipMemcpyAsync");
        check(hipStreamSynchronize(s), "hipStreamSynchronize");
    }
    if (rc == TDFA_OK && err_host != 0)
        rc = fail(TDFA_E_UNSUPPORTED, "token edges outside the limits:%s%s%s",
                  (err_host & kErrString) ? " a pops / pushes string longer than 12 symbols;" : "",
                  (err_host & kErrEpsRun) ? " more than 64 epsilon edges in a row;" : "",
                  (err_host & kErrPending) ? " more than 8 open runs for one state and token;" : "");
    if (rc == TDFA_OK) {
        t->n_edges = n_edges;
        rc = dev_alloc(&t->token, (size_t)n_edges);
        if (rc == TDFA_OK) rc = dev_alloc(&t->dst, (size_t)n_edges);
        if (rc == TDFA_OK) rc = dev_alloc(&t->n_pops, (size_t)n_edges);
        if (rc == TDFA_OK) rc = dev_alloc(&t->pops, (size_t)n_edges * kStr);
        if (rc == TDFA_OK) rc = dev_alloc(&t->n_push, (size_t)n_edges);
        if (rc == TDFA_OK) rc = dev_alloc(&t->pushes, (size_t)n_edges * kStr);
    }
    if (rc == TDFA_OK && v.n_tokens > 0 && n_edges > 0) {
        EdgeOut eo{t->token, t->dst, t->n_pops, t->pops, t->n_push, t->pushes};
        pda_fill_kernel<<<grid, 256, 0, s>>>(a, v.words, v.off, v.len, v.n_tokens, counts, t->edge_first, eo, err);
        check(hipGetLastError(), "pda_fill_kernel");
        check(hipStreamSynchronize(s), "hipStreamSynchronize");
    }
    if (counts) (void)hipFree(counts);
    if (row_total) (void)hipFree(row_total);
    counts = nullptr;
    row_total = nullptr;
    // Classes of each state's edges by their pops, and a row of allowed bits per class.  Kept if no
    // state has more than kMaxClasses and the rows stay below 1 GiB; the step scans edges otherwise.
    t->row_words = tdfa_allow_row_words(v.n_tokens);
    if (rc == TDFA_OK && v.n_tokens > 0 && n_edges > 0 && (int64_t)pda->n_states * kMaxClasses * kStr * 4 <= (int64_t)1 << 28) {
        uint8_t* edge_class = nullptr;
        int32_t *n_cls = nullptr, *cls_np = nullptr, *cls_pops = nullptr;
        rc = dev_alloc(&edge_class, (size_t)n_edges);
        if (rc == TDFA_OK) rc = dev_alloc(&n_cls, (size_t)pda->n_states);
        if (rc == TDFA_OK) rc = dev_alloc(&cls_np, (size_t)pda->n_states * kMaxClasses);
        if (rc == TDFA_OK) rc = dev_alloc(&cls_pops, (size_t)pda->n_states * kMaxClasses * kStr);
        std::vector<int32_t> first((size_t)pda->n_states + 1, 0);
        if (rc == TDFA_OK) {
            check(hipMemsetAsync(edge_class, 0xFF, (size_t)n_edges, s), "hipMemsetAsync");
            check(hipMemsetAsync(err, 0, sizeof(uint32_t), s), "hipMemsetAsync");
            pda_classes_kernel<<<(unsigned)pda->n_states, 256, 0, s>>>(t->edge_first, t->n_pops, t->pops, edge_class, n_cls, cls_np,
                                                                       cls_pops, err);
            check(hipGetLastError(), "pda_classes_kernel");
            check(hipMemcpyAsync(first.data() + 1, n_cls, (size_t)pda->n_states * 4, hipMemcpyDeviceToHost, s), "hipMemcpyAsync");
            check(hipMemcpyAsync(&err_host, err, sizeof(uint32_t), hipMemcpyDeviceToHost, s), "hipMemcpyAsync");
            check(hipStreamSynchronize(s), "hipStreamSynchronize");
        }
        if (rc == TDFA_OK) {
            for (int32_t q = 0; q < pda->n_states; ++q) first[(size_t)q + 1] += first[(size_t)q];
            const int64_t rows = first[(size_t)pda->n_states];
            if (err_host == 0 && rows > 0 && rows * t->row_words * 4 <= (int64_t)1 << 30) {
                rc = dev_alloc(&t->class_first, (size_t)pda->n_states + 1);
                if (rc == TDFA_OK) rc = dev_alloc(&t->class_n_pops, (size_t)rows);
                if (rc == TDFA_OK) rc = dev_alloc(&t->class_pops, (size_t)rows * kStr);
                if (rc == TDFA_OK) rc = dev_alloc(&t->class_bits, (size_t)rows * (size_t)t->row_words);
                if (rc == TDFA_OK) {
                    check(hipMemcpyAsync(t->class_first, first.data(), first.size() * 4, hipMemcpyHostToDevice, s), "hipMemcpyAsync");
                    check(hipMemsetAsync(t->class_bits, 0, (size_t)rows * (size_t)t->row_words * 4, s), "hipMemsetAsync");
                    const dim3 cgrid(64, (unsigned)pda->n_states);
                    pda_class_rows_kernel<<<cgrid, 256, 0, s>>>(t->edge_first, t->token, edge_class, t->class_first, cls_np, cls_pops,
                                                                t->class_n_pops, t->class_pops, t->class_bits, t->row_words);
                    check(hipGetLastError(), "pda_class_rows_kernel");
                    check(hipStreamSynchronize(s), "hipStreamSynchronize");
                }
                if (rc == TDFA_OK) t->n_class_rows = (int32_t)rows;
            }
        }
        for (void* d : {(void*)edge_class, (void*)n_cls, (void*)cls_np, (void*)cls_pops})
            if (d) (void)hipFree(d);
    }
    if (err) (void)hipFree(err);
    if (rc != TDFA_OK) {
        tdfa_ptable_destroy(t);
        return rc;
    }
    *out = t;
    return TDFA_OK;
}

int tdfa_ptable_info(const tdfa_ptable* t, int32_t* n_states, int32_t* n_tokens, int64_t* n_edges, int64_t** edge_first_dev,
                     int32_t** token_dev, int32_t** dst_dev, int32_t** n_pops_dev, int32_t** pops_dev, int32_t** n_push_dev,
                     int32_t** pushes_dev)
{
    clear_error();
    if (!t) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (n_states) *n_states = t->n_states;
    if (n_tokens) *n_tokens = t->n_tokens;
    if (n_edges) *n_edges = t->n_edges;
    if (edge_first_dev) *edge_first_dev = t->edge_first;
    if (token_dev) *token_dev = t->token;
    if (dst_dev) *dst_dev = t->dst;
    if (n_pops_dev) *n_pops_dev = t->n_pops;
    if (pops_dev) *pops_dev = t->pops;
    if (n_push_dev) *n_push_dev = t->n_push;
    if (pushes_dev) *pushes_dev = t->pushes;
    return TDFA_OK;
}

int tdfa_ptable_destroy(tdfa_ptable* t)
{
    if (!t) return TDFA_OK;
    for (void* d : {(void*)t->edge_first, (void*)t->token, (void*)t->dst, (void*)t->n_pops, (void*)t->pops, (void*)t->n_push,
                    (void*)t->pushes, (void*)t->class_first, (void*)t->class_n_pops, (void*)t->class_pops, (void*)t->class_bits,
                    (void*)t->step_allow, (void*)t->step_rows, (void*)t->step_unused})
        if (d) (void)hipFree(d);
    for (void* d : t->retired) (void)hipFree(d);
    delete t;
    return TDFA_OK;
}

namespace {
struct Draw {                 // the sampled step: 1 / temperature, the cut and the generator's position
    float inv_t;
    int32_t top_k;
    uint64_t seed, offset;
};

int pda_step_impl(const tdfa_ptable* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                  const int32_t* states_dev, int32_t* stacks_dev, int32_t* depths_dev, int32_t stack_cap, int32_t* tokens_dev,
                  int32_t* new_states_dev, void* masked_out_dev, void* stream, const Draw* draw)
{
    if (!table) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (dtype != TDFA_F32 && dtype != TDFA_BF16) return fail(TDFA_E_INVALID_ARG, "unknown dtype %d", dtype);
    if (batch < 0 || stack_cap < 0) return fail(TDFA_E_INVALID_ARG, "batch %d or stack_cap %d is negative", batch, stack_cap);
    if (batch == 0) return TDFA_OK;
    if (!logits_dev || !states_dev || !stacks_dev || !depths_dev || !tokens_dev || !new_states_dev)
        return fail(TDFA_E_INVALID_ARG, "logits, states, stacks, depths, tokens or new_states is NULL");
    if (row_stride < table->n_tokens) return fail(TDFA_E_INVALID_ARG, "row_stride %lld < n_tokens %d", (long long)row_stride, table->n_tokens);
    if (masked_out_dev == logits_dev) return fail(TDFA_E_INVALID_ARG, "masked_out must not be the logits themselves");
    PdaStepArgs a;
    a.edge_first = table->edge_first;
    a.token = table->token;
    a.dst = table->dst;
    a.n_pops = table->n_pops;
    a.pops = table->pops;
    a.n_push = table->n_push;
    a.pushes = table->pushes;
    a.n_states = table->n_states;
    a.n_tokens = table->n_tokens;
    a.logits = logits_dev;
    a.row_stride = row_stride;
    a.states = states_dev;
    a.stacks = stacks_dev;
    a.depths = depths_dev;
    a.stack_cap = stack_cap;
    a.tokens = tokens_dev;
    a.new_states = new_states_dev;
    a.masked_out = masked_out_dev;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t esz = dtype == TDFA_F32 ? 4 : 2;
    const bool aligned = !(reinterpret_cast<uintptr_t>(logits_dev) & 15) && !((row_stride * esz) & 15) &&
                         !(reinterpret_cast<uintptr_t>(masked_out_dev) & 15);
    const bool rows_usable = aligned && (draw || table->n_class_rows > 0);
    if (!aligned && draw) return fail(TDFA_E_UNSUPPORTED, "a drawn step needs 16-byte aligned rows of logits");
    if (!rows_usable) {
        // no class rows, or logits the 16-byte loads of the step kernel cannot take: scan the state's edges
        if (dtype == TDFA_BF16) pda_step_kernel<true><<<(unsigned)batch, 256, 0, s>>>(a);
        else pda_step_kernel<false><<<(unsigned)batch, 256, 0, s>>>(a);
        TDFA_HIP(hipGetLastError());
        return TDFA_OK;
    }
    // a row of allowed bits per sequence: grown outside stream capture, never freed while the table lives
    if (batch > table->step_cap) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        TDFA_HIP(hipStreamIsCapturing(s, &cs));
        if (cs != hipStreamCaptureStatusNone)
            return fail(TDFA_E_UNSUPPORTED, "the first step at batch %d allocates: call it once before capturing", batch);
        for (void* d : {(void*)table->step_allow, (void*)table->step_rows, (void*)table->step_unused})
            if (d) table->retired.push_back(d);
        table->step_allow = nullptr;
        table->step_rows = nullptr;
        table->step_unused = nullptr;
        table->step_cap = 0;
        int rc = dev_alloc(&table->step_allow, (size_t)batch * (size_t)table->row_words);
        if (rc == TDFA_OK) rc = dev_alloc(&table->step_rows, (size_t)batch);
        if (rc == TDFA_OK) rc = dev_alloc(&table->step_unused, 2 * (size_t)batch);     // (the second half: a word per sequence for the cut of a drawn step)
        if (rc != TDFA_OK) return rc;
        table->step_cap = batch;
    }
    tdfa::MaskArgs m{};
    m.delta = nullptr;
    m.targets = nullptr;
    m.row_begin = nullptr;
    m.dir = nullptr;
    m.allow = table->step_allow;
    m.n_rows = batch;
    m.n_tokens = table->n_tokens;
    m.row_words = table->row_words;
    m.logits = logits_dev;
    m.dtype = dtype;
    m.batch = batch;
    m.row_stride = row_stride;
    m.states = table->step_rows;
    m.tokens = tokens_dev;
    m.new_states = table->step_unused;
    m.masked_out = masked_out_dev;
    {
        const int rc = tdfa::step_scratch(batch, s, &m.scratch_best, &m.scratch_count);
        if (rc != TDFA_OK) return rc;
    }
    // 16-bit logits: the step kernel finds a sequence's classes itself and ORs their rows as it reads them
    tdfa::MaskArgs fused = m;
    fused.allow = table->class_bits;
    fused.n_rows = table->n_class_rows;
    fused.states = states_dev;
    fused.pda.class_first = table->class_first;
    fused.pda.class_n_pops = table->class_n_pops;
    fused.pda.class_pops = table->class_pops;
    fused.pda.stacks = stacks_dev;
    fused.pda.depths = depths_dev;
    fused.pda.stack_cap = stack_cap;
    fused.pda.n_states = table->n_states;
    if (draw) {
        // the rows of the sequences first (from the class rows, or edge by edge where the table has none), then
        // the draw of the sampled step on them (it only chooses tokens)
        if (table->n_class_rows > 0)
            pda_allow_kernel<<<(unsigned)batch, 256, 0, s>>>(states_dev, stacks_dev, depths_dev, stack_cap, table->n_states,
                                                             table->class_first, table->class_n_pops, table->class_pops, table->class_bits,
                                                             table->row_words, table->step_allow, table->step_rows);
        else
            pda_allow_edges_kernel<<<(unsigned)batch, 256, 0, s>>>(states_dev, stacks_dev, depths_dev, stack_cap, table->n_states,
                                                                   table->edge_first, table->token, table->n_pops, table->pops,
                                                                   table->row_words, table->step_allow, table->step_rows);
        TDFA_HIP(hipGetLastError());
        const int rc = tdfa::launch_sample_step(m, draw->inv_t, draw->top_k, reinterpret_cast<uint32_t*>(table->step_unused + table->step_cap),
                                                draw->seed, draw->offset, nullptr, s);
        if (rc != TDFA_OK) return rc;
    } else if (tdfa::mask_step_takes_pda(fused)) {
        const int rc = tdfa::launch_mask_step(fused, s);
        if (rc != TDFA_OK) return rc;
    } else {
        pda_allow_kernel<<<(unsigned)batch, 256, 0, s>>>(states_dev, stacks_dev, depths_dev, stack_cap, table->n_states, table->class_first,
                                                         table->class_n_pops, table->class_pops, table->class_bits, table->row_words,
                                                         table->step_allow, table->step_rows);
        TDFA_HIP(hipGetLastError());
        const int rc = tdfa::launch_mask_step(m, s);
        if (rc != TDFA_OK) return rc;
    }
    pda_advance_kernel<<<(unsigned)((batch + 3) / 4), 256, 0, s>>>(a, batch);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}
}  // namespace

int tdfa_pda_step(const tdfa_ptable* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                  const int32_t* states_dev, int32_t* stacks_dev, int32_t* depths_dev, int32_t stack_cap, int32_t* tokens_dev,
                  int32_t* new_states_dev, void* masked_out_dev, void* stream)
{
    clear_error();
    return pda_step_impl(table, logits_dev, dtype, batch, row_stride, states_dev, stacks_dev, depths_dev, stack_cap, tokens_dev,
                         new_states_dev, masked_out_dev, stream, nullptr);
}

int tdfa_pda_sample_step(const tdfa_ptable* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                         const int32_t* states_dev, int32_t* stacks_dev, int32_t* depths_dev, int32_t stack_cap, float temperature,
                         int32_t top_k, uint64_t seed, uint64_t offset, int32_t* tokens_dev, int32_t* new_states_dev,
                         void* masked_out_dev, void* stream)
{
    clear_error();
    if (!(temperature > 0.0f)) return fail(TDFA_E_INVALID_ARG, "temperature %g is not positive", (double)temperature);
    if (top_k < 0) return fail(TDFA_E_INVALID_ARG, "top_k %d is negative", top_k);
    const volatile float one = 1.0f;                     // divided at run time, rounded once to binary32
    Draw draw;
    draw.inv_t = one / temperature;
    if (!(draw.inv_t > 0.0f) || draw.inv_t > 3.402823466e38f)
        return fail(TDFA_E_INVALID_ARG, "1 / temperature is not finite for temperature %g", (double)temperature);
    draw.top_k = top_k;
    draw.seed = seed;
    draw.offset = offset;
    return pda_step_impl(table, logits_dev, dtype, batch, row_stride, states_dev, stacks_dev, depths_dev, stack_cap, tokens_dev,
                         new_states_dev, masked_out_dev, stream, &draw);
}

}  // extern "C"
