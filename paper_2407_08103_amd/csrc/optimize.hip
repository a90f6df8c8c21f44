// Token-level optimisation of a compiled table (Appendix C.2, the fourth of the compile operations it
// times, applied to the composed automaton).  The paper does not name the optimisation; the reading taken is the
// classical one for a deterministic automaton: keep the states that some token sequence reaches
// from a start state and from which a final state can be reached, and merge the states that accept
// the same token sequences (Moore's partition refinement).  A set-up call.
//
// A row of a token table has many entries but few distinct targets (the character states one
// token away).  One pass over the table therefore reduces every row to its distinct targets r,
// each with the weight F(q, r) = sum of w(t) over the tokens t with delta_T[q][t] = r (w: a mixed,
// odd 64-bit number per token); all the rounds then run on these short lists:
//
//   reach      rounds from the start states: the targets of a marked row are marked
//   co-reach   rounds over the rows not yet known to reach a final state: a row with a target
//              that does becomes one
//   refine     a class is named by its smallest state.  A round gives every kept row the
//              signature sum of g(class of r) * F(q, r) (= the sum over its tokens of
//              w(t) * g(class of the target), in any order), rows with the same (class,
//              signature) find each other in a hash table on the device and take their smallest
//              row as the new name.  The host only reads the number of classes of each round.
//              Equal rows always get equal signatures, so a signature never splits wrongly; when
//              no class splits any more every row that joined another is compared with it entry
//              by entry over the dense table, so a signature never decides that rows are equal.
//   compact    the first row of each class, its entries renamed, is a row of the new table
//
// A row with more distinct targets than the workgroup's table in LDS holds (a table that is not
// sparse in this sense), or a failed comparison, sends the whole call down the dense path: the same
// steps with the host driving rounds of kernels that stream the table's rows.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kThreads = 256;

// rows[i] is scanned: every live entry marks its target in `mark` (bytes; equal stores may race).
__global__ void __launch_bounds__(kThreads)
mark_targets_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, const int32_t* __restrict__ rows,
                    uint8_t* __restrict__ mark)
{
    const int32_t* row = delta + (size_t)rows[blockIdx.y] * n_tokens;
    for (int t = blockIdx.x * kThreads + threadIdx.x; t < n_tokens; t += gridDim.x * kThreads) {
        const int32_t v = row[t];
        if (v >= 0 && !mark[v]) mark[v] = 1;
    }
}

// rows[i] becomes good (can reach a final state) if one of its entries leads to a good state.
__global__ void __launch_bounds__(kThreads)
reach_final_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, const int32_t* __restrict__ rows,
                   const uint8_t* __restrict__ kept, uint8_t* __restrict__ good, int32_t* __restrict__ changed)
{
    const int32_t q = rows[blockIdx.y];
    const int32_t* row = delta + (size_t)q * n_tokens;
    bool hit = false;
    for (int t = blockIdx.x * kThreads + threadIdx.x; t < n_tokens && !hit; t += gridDim.x * kThreads) {
        const int32_t v = row[t];
        hit = v >= 0 && kept[v] && good[v];
    }
    if (hit && !good[q]) {
        good[q] = 1;
        *changed = 1;
    }
}

__device__ __forceinline__ unsigned long long mix64(unsigned long long x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// hash[i] of rows[i]: sum over the tokens of mix(token, class of the entry's target); cls is -1
// for a state that is not kept, and a DEAD entry counts like one.
__global__ void __launch_bounds__(kThreads)
row_hash_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, const int32_t* __restrict__ rows,
                const int32_t* __restrict__ cls, unsigned long long seed, unsigned long long* __restrict__ hash)
{
    __shared__ unsigned long long part[kThreads / 64];
    const int32_t* row = delta + (size_t)rows[blockIdx.x] * n_tokens;
    unsigned long long h = 0;
    for (int t = threadIdx.x; t < n_tokens; t += kThreads) {
        const int32_t v = row[t];
        const int32_t c = v >= 0 ? cls[v] : -1;
        if (c >= 0) h += mix64(seed + (unsigned long long)t * 0x9E3779B97F4A7C15ull + (unsigned long long)(unsigned)c);
    }
    for (int off = 32; off > 0; off >>= 1) h += __shfl_xor(h, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) h += part[w];
        hash[blockIdx.x] = h;
    }
}

// rows[i] and first_of[i] (the first row of its class) must agree, entry by entry, on the class
// of the target.
__global__ void __launch_bounds__(kThreads)
verify_classes_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, const int32_t* __restrict__ rows,
                      const int32_t* __restrict__ first_of, const int32_t* __restrict__ cls, int32_t* __restrict__ mismatch)
{
    const int32_t* a = delta + (size_t)rows[blockIdx.y] * n_tokens;
    const int32_t* b = delta + (size_t)first_of[blockIdx.y] * n_tokens;
    bool bad = false;
    for (int t = blockIdx.x * kThreads + threadIdx.x; t < n_tokens; t += gridDim.x * kThreads) {
        const int32_t x = a[t], y = b[t];
        const int32_t cx = x >= 0 ? cls[x] : -1, cy = y >= 0 ? cls[y] : -1;
        bad |= cx != cy;
    }
    if (bad) *mismatch = 1;
}

// New row c = row first_row[c] of the old table with its entries renamed by `map` (-1 for a state
// that was dropped); allowed words from the new entries.
__global__ void __launch_bounds__(kThreads)
compact_rows_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, int64_t row_words,
                    const int32_t* __restrict__ first_row, const int32_t* __restrict__ map,
                    int32_t* __restrict__ out_delta, uint32_t* __restrict__ out_allow)
{
    const int t = blockIdx.x * kThreads + threadIdx.x;
    int v = TDFA_DEAD;
    if (t < n_tokens) {
        const int32_t old = delta[(size_t)first_row[blockIdx.y] * n_tokens + t];
        v = old >= 0 ? map[old] : TDFA_DEAD;
        out_delta[(size_t)blockIdx.y * n_tokens + t] = v;
    }
    const uint64_t m = __builtin_amdgcn_ballot_w64(v != TDFA_DEAD);
    const int lane = threadIdx.x & 63;
    const int64_t word = (int64_t)((t - lane) >> 5) + lane;
    if (lane < 2 && word < row_words) out_allow[(size_t)blockIdx.y * row_words + word] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
}

struct DeviceBuffers {
    int32_t* rows = nullptr;
    int32_t* aux = nullptr;       // first_of / map
    int32_t* cls = nullptr;
    uint8_t* mark = nullptr;
    uint8_t* good = nullptr;
    unsigned long long* hash = nullptr;
    int32_t* flag = nullptr;
    ~DeviceBuffers()
    {
        for (void* p : {(void*)rows, (void*)aux, (void*)cls, (void*)mark, (void*)good, (void*)hash, (void*)flag})
            if (p) (void)hipFree(p);
    }
};

constexpr size_t kMaxGridY = 65535;

unsigned grid_x(int32_t n_tokens) { return (unsigned)std::max(1, std::min(64, (n_tokens + kThreads * 8 - 1) / (kThreads * 8))); }


// ---------------------------------------------------------------------------------------------
// The sparse path: rows as lists of distinct targets.

constexpr int kListThreads = 512;      // workgroup of the pass that builds a row's list
constexpr int kSlots = 4096;           // its table of targets in LDS (open addressing, 48 KB)
constexpr int kMaxTargets = 3072;      // more distinct targets in one row: the dense path
constexpr int kLoadsAhead = 8;

__device__ __forceinline__ unsigned long long token_weight(unsigned long long seed, int t)
{
    return mix64(seed + (unsigned long long)t * 0x9E3779B97F4A7C15ull) | 1ull;
}

__device__ __forceinline__ void add_target(int32_t* key, unsigned long long* sum, int* n_used, int32_t v, unsigned long long w)
{
    unsigned slot = ((unsigned)v * 0x9E3779B1u) >> 20;
    for (int probe = 0; probe < kSlots; ++probe, slot = (slot + 1) & (kSlots - 1)) {
        int32_t k = key[slot];
        if (k == -1) {
            k = atomicCAS(&key[slot], -1, v);
            if (k == -1) {
                atomicAdd(n_used, 1);
                k = v;
            }
        }
        if (k == v) {
            atomicAdd(&sum[slot], w);
            return;
        }
    }
    atomicAdd(n_used, kSlots);          // the table is full of other targets: counts as too many
}

// Row blockIdx.x: its distinct targets and their weights, appended to (e_target, e_weight) at a
// position taken from `counter` (which keeps counting past e_cap, so that a second attempt knows the
// size).  *overflow is set when a row has more than kMaxTargets targets.
__global__ void __launch_bounds__(kListThreads)
row_targets_kernel(const int32_t* __restrict__ delta, int32_t n_tokens, unsigned long long seed, unsigned long long e_cap,
                   unsigned long long* __restrict__ counter, unsigned long long* __restrict__ row_begin,
                   int32_t* __restrict__ row_n, int32_t* __restrict__ e_target, unsigned long long* __restrict__ e_weight,
                   int32_t* overflow)
{
    __shared__ int32_t key[kSlots];
    __shared__ unsigned long long sum[kSlots];
    __shared__ int n_used, n_out, stop;
    __shared__ unsigned long long base;
    for (int i = threadIdx.x; i < kSlots; i += kListThreads) {
        key[i] = -1;
        sum[i] = 0;
    }
    if (threadIdx.x == 0) {
        n_used = 0;
        n_out = 0;
        stop = *(volatile int32_t*)overflow;        // another row has too many: the lists will not be used
    }
    __syncthreads();
    if (stop) return;
    const int32_t* row = delta + (size_t)blockIdx.x * n_tokens;
    int32_t last = TDFA_DEAD;
    unsigned long long acc = 0;
    for (int t0 = threadIdx.x; t0 < n_tokens; t0 += kListThreads * kLoadsAhead) {
        int32_t v[kLoadsAhead];
#pragma unroll
        for (int u = 0; u < kLoadsAhead; ++u) {
            const int t = t0 + u * kListThreads;
            v[u] = t < n_tokens ? row[t] : TDFA_DEAD;
        }
#pragma unroll
        for (int u = 0; u < kLoadsAhead; ++u) {
            if (v[u] != last) {             // runs of one target (a state that mostly loops) cost one update
                if (last >= 0) add_target(key, sum, &n_used, last, acc);
                last = v[u];
                acc = 0;
            }
            acc += token_weight(seed, t0 + u * kListThreads);
        }
        if (*(volatile int*)&n_used > kMaxTargets) break;
    }
    if (last >= 0) add_target(key, sum, &n_used, last, acc);
    __syncthreads();
    const int n = n_used;
    if (n > kMaxTargets) {
        if (threadIdx.x == 0) *overflow = 1;
        return;
    }
    if (threadIdx.x == 0) {
        base = atomicAdd(counter, (unsigned long long)n);
        row_begin[blockIdx.x] = base;
        row_n[blockIdx.x] = n;
    }
    __syncthreads();
    if (base + (unsigned long long)n > e_cap) return;
    for (int i = threadIdx.x; i < kSlots; i += kListThreads)
        if (key[i] != -1) {
            const int p = atomicAdd(&n_out, 1);
            e_target[base + p] = key[i];
            e_weight[base + p] = sum[i];
        }
}

// The kernels below give a wavefront to a row's list.
constexpr int kRowsPerBlock = kThreads / 64;

struct Lists {
    const unsigned long long* row_begin;
    const int32_t* row_n;
    const int32_t* e_target;
    const unsigned long long* e_weight;
    int32_t n_rows;
};

__global__ void __launch_bounds__(kThreads)
list_reach_kernel(Lists g, uint8_t* mark, uint8_t* done, int32_t* changed)
{
    const int32_t q = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (q >= g.n_rows || !mark[q] || done[q]) return;
    const int lane = threadIdx.x & 63;
    if (lane == 0) done[q] = 1;
    const int32_t* e = g.e_target + g.row_begin[q];
    for (int i = lane; i < g.row_n[q]; i += 64)
        if (!mark[e[i]]) {
            mark[e[i]] = 1;
            *changed = 1;
        }
}

__global__ void __launch_bounds__(kThreads)
list_good_start_kernel(int32_t n_rows, const uint8_t* __restrict__ mark, const uint8_t* __restrict__ accept, uint8_t* __restrict__ good)
{
    const int32_t q = blockIdx.x * kThreads + threadIdx.x;
    if (q < n_rows) good[q] = mark[q] && accept[q];
}

__global__ void __launch_bounds__(kThreads)
list_reach_final_kernel(Lists g, const uint8_t* mark, uint8_t* good, int32_t* changed)
{
    const int32_t q = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (q >= g.n_rows || !mark[q] || good[q]) return;
    const int lane = threadIdx.x & 63;
    const int32_t* e = g.e_target + g.row_begin[q];
    bool hit = false;
    for (int i = lane; i < g.row_n[q]; i += 64) hit |= mark[e[i]] && good[e[i]];
    if (__builtin_amdgcn_ballot_w64(hit) != 0 && lane == 0) {
        good[q] = 1;
        *changed = 1;
    }
}

__global__ void __launch_bounds__(kThreads) fill_i32_kernel(int32_t* p, size_t n, int32_t v)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = v;
}

// The first partition: kept rows by their final flag (cls 0 for every kept row, -1 for the rest).
__global__ void __launch_bounds__(kThreads)
list_first_keys_kernel(int32_t n_rows, const uint8_t* __restrict__ mark, const uint8_t* __restrict__ good,
                       const uint8_t* __restrict__ accept, unsigned long long seed, int32_t* __restrict__ cls,
                       unsigned long long* __restrict__ key)
{
    const int32_t q = blockIdx.x * kThreads + threadIdx.x;
    if (q >= n_rows) return;
    const bool kept = mark[q] && good[q];
    cls[q] = kept ? 0 : -1;
    key[q] = mix64(seed + (accept[q] ? 1 : 2)) | 1ull;
}

// key[q] of a kept row: its class and the signature of its targets' classes, mixed (never 0).
__global__ void __launch_bounds__(kThreads)
list_keys_kernel(Lists g, const int32_t* __restrict__ cls, unsigned long long seed, unsigned long long* __restrict__ key)
{
    const int32_t q = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (q >= g.n_rows || cls[q] < 0) return;
    const int lane = threadIdx.x & 63;
    const unsigned long long b = g.row_begin[q];
    unsigned long long h = 0;
    for (int i = lane; i < g.row_n[q]; i += 64) {
        const int32_t c = cls[g.e_target[b + i]];
        if (c >= 0) h += mix64(seed ^ (unsigned long long)(unsigned)c) * g.e_weight[b + i];
    }
    for (int off = 32; off > 0; off >>= 1) h += __shfl_xor(h, off, 64);
    if (lane == 0) key[q] = mix64(h ^ mix64(seed + 0x632BE59BD9B4E019ull + (unsigned long long)(unsigned)cls[q])) | 1ull;
}

// Rows with equal keys meet in one slot of the table (ht_key 0: free; more slots than rows) and
// leave their smallest row there.
__global__ void __launch_bounds__(kThreads)
list_insert_kernel(int32_t n_rows, const int32_t* __restrict__ cls, const unsigned long long* __restrict__ key,
                   unsigned long long* ht_key, int32_t* ht_min, uint32_t ht_mask, uint32_t* __restrict__ slot_of)
{
    const int32_t q = blockIdx.x * kThreads + threadIdx.x;
    if (q >= n_rows || cls[q] < 0) return;
    const unsigned long long k = key[q];
    uint32_t slot = (uint32_t)(k >> 20) & ht_mask;
    for (uint32_t probe = 0; probe <= ht_mask; ++probe, slot = (slot + 1) & ht_mask) {
        const unsigned long long was = atomicCAS(&ht_key[slot], 0ull, k);
        if (was == 0ull || was == k) {
            atomicMin(&ht_min[slot], q);
            slot_of[q] = slot;
            return;
        }
    }
}

__global__ void __launch_bounds__(kThreads)
list_assign_kernel(int32_t n_rows, const int32_t* __restrict__ cls, const uint32_t* __restrict__ slot_of,
                   const int32_t* __restrict__ ht_min, int32_t* __restrict__ cls_out, int32_t* n_classes)
{
    const int32_t q = blockIdx.x * kThreads + threadIdx.x;
    bool first = false;
    if (q < n_rows) {
        const int32_t c = cls[q] < 0 ? -1 : ht_min[slot_of[q]];
        cls_out[q] = c;
        first = c == q;
    }
    const uint64_t m = __builtin_amdgcn_ballot_w64(first);
    if ((threadIdx.x & 63) == 0 && m != 0) atomicAdd(n_classes, __builtin_popcountll(m));
}

// The dense path: every round streams rows of the table.
int minimize_dense(const int32_t* delta, int32_t n_rows, int32_t n_tokens, const uint8_t* accept, const int32_t* starts,
                   int32_t n_starts, hipStream_t s, std::vector<int32_t>* first_rows, std::vector<int32_t>* map_out)
{
    DeviceBuffers d;
    TDFA_HIP(hipMalloc(&d.rows, (size_t)n_rows * 4));
    TDFA_HIP(hipMalloc(&d.aux, (size_t)n_rows * 4));
    TDFA_HIP(hipMalloc(&d.cls, (size_t)n_rows * 4));
    TDFA_HIP(hipMalloc(&d.mark, (size_t)n_rows));
    TDFA_HIP(hipMalloc(&d.good, (size_t)n_rows));
    TDFA_HIP(hipMalloc(&d.hash, (size_t)n_rows * 8));
    TDFA_HIP(hipMalloc(&d.flag, 4));
    std::vector<uint8_t> mark((size_t)n_rows, 0), good((size_t)n_rows, 0), seen((size_t)n_rows, 0);
    std::vector<int32_t> rows;
    const unsigned gx = grid_x(n_tokens);

    // ---- states that a token sequence reaches
    for (int32_t i = 0; i < n_starts; ++i)
        if (!mark[(size_t)starts[i]]) {
            mark[(size_t)starts[i]] = 1;
            rows.push_back(starts[i]);
        }
    seen = mark;
    TDFA_HIP(hipMemcpyAsync(d.mark, mark.data(), (size_t)n_rows, hipMemcpyHostToDevice, s));
    while (!rows.empty() && n_tokens > 0) {
        TDFA_HIP(hipMemcpyAsync(d.rows, rows.data(), rows.size() * 4, hipMemcpyHostToDevice, s));
        for (size_t lo = 0; lo < rows.size(); lo += kMaxGridY) {
            mark_targets_kernel<<<dim3(gx, (unsigned)std::min(kMaxGridY, rows.size() - lo)), kThreads, 0, s>>>(delta, n_tokens, d.rows + lo,
                                                                                                          d.mark);
            TDFA_HIP(hipGetLastError());
        }
        TDFA_HIP(hipMemcpyAsync(mark.data(), d.mark, (size_t)n_rows, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        rows.clear();
        for (int32_t q = 0; q < n_rows; ++q)
            if (mark[(size_t)q] && !seen[(size_t)q]) {
                seen[(size_t)q] = 1;
                rows.push_back(q);
            }
    }
    // ---- of those, the states that can reach a final state
    for (int32_t q = 0; q < n_rows; ++q) good[(size_t)q] = mark[(size_t)q] && accept[q];
    TDFA_HIP(hipMemcpyAsync(d.good, good.data(), (size_t)n_rows, hipMemcpyHostToDevice, s));
    for (bool changed = n_tokens > 0; changed;) {
        rows.clear();
        for (int32_t q = 0; q < n_rows; ++q)
            if (mark[(size_t)q] && !good[(size_t)q]) rows.push_back(q);
        if (rows.empty()) break;
        int32_t zero = 0, flag = 0;
        TDFA_HIP(hipMemcpyAsync(d.flag, &zero, 4, hipMemcpyHostToDevice, s));
        TDFA_HIP(hipMemcpyAsync(d.rows, rows.data(), rows.size() * 4, hipMemcpyHostToDevice, s));
        for (size_t lo = 0; lo < rows.size(); lo += kMaxGridY) {
            reach_final_kernel<<<dim3(gx, (unsigned)std::min(kMaxGridY, rows.size() - lo)), kThreads, 0, s>>>(delta, n_tokens, d.rows + lo,
                                                                                                         d.mark, d.good, d.flag);
            TDFA_HIP(hipGetLastError());
        }
        TDFA_HIP(hipMemcpyAsync(&flag, d.flag, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipMemcpyAsync(good.data(), d.good, (size_t)n_rows, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        changed = flag != 0;
    }
    // ---- refinement over the kept states
    rows.clear();
    std::vector<int32_t> cls((size_t)n_rows, -1);
    for (int32_t q = 0; q < n_rows; ++q)
        if (mark[(size_t)q] && good[(size_t)q]) {
            rows.push_back(q);
            cls[(size_t)q] = accept[q] ? 1 : 0;
        }
    const size_t n = rows.size();
    map_out->assign((size_t)n_rows, TDFA_DEAD);
    first_rows->clear();
    if (n == 0) return TDFA_OK;
    TDFA_HIP(hipMemcpyAsync(d.rows, rows.data(), n * 4, hipMemcpyHostToDevice, s));
    std::vector<unsigned long long> hash(n);
    std::vector<int32_t> by(n), first_of(n);
    size_t n_cls = 0;
    for (unsigned attempt = 0;; ++attempt) {
        if (attempt == 4) return fail(TDFA_E_DEVICE, "row hashes collided in four attempts");
        for (size_t prev = 0;;) {
            TDFA_HIP(hipMemcpyAsync(d.cls, cls.data(), (size_t)n_rows * 4, hipMemcpyHostToDevice, s));
            row_hash_kernel<<<(unsigned)n, kThreads, 0, s>>>(delta, n_tokens, d.rows, d.cls, 0x243F6A8885A308D3ull * (attempt + 1), d.hash);
            TDFA_HIP(hipGetLastError());
            TDFA_HIP(hipMemcpyAsync(hash.data(), d.hash, n * 8, hipMemcpyDeviceToHost, s));
            TDFA_HIP(hipStreamSynchronize(s));
            for (size_t i = 0; i < n; ++i) by[i] = (int32_t)i;
            std::sort(by.begin(), by.end(), [&](int32_t x, int32_t y) {
                const int32_t cx = cls[(size_t)rows[(size_t)x]], cy = cls[(size_t)rows[(size_t)y]];
                if (cx != cy) return cx < cy;
                if (hash[(size_t)x] != hash[(size_t)y]) return hash[(size_t)x] < hash[(size_t)y];
                return x < y;
            });
            std::vector<int32_t> next(n);
            n_cls = 0;
            for (size_t i = 0; i < n; ++i) {
                const bool same = i > 0 && cls[(size_t)rows[(size_t)by[i]]] == cls[(size_t)rows[(size_t)by[i - 1]]] &&
                                  hash[(size_t)by[i]] == hash[(size_t)by[i - 1]];
                if (!same) {
                    ++n_cls;
                    first_of[n_cls - 1] = rows[(size_t)by[i]];          // the smallest row of the class (ties sorted by index)
                }
                next[(size_t)by[i]] = (int32_t)(n_cls - 1);
            }
            for (size_t i = 0; i < n; ++i) cls[(size_t)rows[i]] = next[i];
            if (n_cls == prev) break;
            prev = n_cls;
        }
        // no class splits any more: compare every row with the first row of its class
        std::vector<int32_t> first_of_row(n);
        for (size_t i = 0; i < n; ++i) first_of_row[i] = first_of[(size_t)cls[(size_t)rows[i]]];
        int32_t zero = 0, bad = 0;
        TDFA_HIP(hipMemcpyAsync(d.flag, &zero, 4, hipMemcpyHostToDevice, s));
        TDFA_HIP(hipMemcpyAsync(d.aux, first_of_row.data(), n * 4, hipMemcpyHostToDevice, s));
        TDFA_HIP(hipMemcpyAsync(d.cls, cls.data(), (size_t)n_rows * 4, hipMemcpyHostToDevice, s));
        if (n_tokens > 0) {
            for (size_t lo = 0; lo < n; lo += kMaxGridY) {
                verify_classes_kernel<<<dim3(gx, (unsigned)std::min(kMaxGridY, n - lo)), kThreads, 0, s>>>(delta, n_tokens, d.rows + lo,
                                                                                                      d.aux + lo, d.cls, d.flag);
                TDFA_HIP(hipGetLastError());
            }
        }
        TDFA_HIP(hipMemcpyAsync(&bad, d.flag, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        if (!bad) break;
        // a collision merged rows that differ: start over from {final, not final} with other hashes
        for (size_t i = 0; i < n; ++i) cls[(size_t)rows[i]] = accept[rows[i]] ? 1 : 0;
    }
    // ---- number the classes by their smallest state
    std::vector<int32_t> order(n_cls);
    for (size_t c = 0; c < n_cls; ++c) order[c] = (int32_t)c;
    std::sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return first_of[(size_t)x] < first_of[(size_t)y]; });
    std::vector<int32_t> new_id(n_cls);
    first_rows->resize(n_cls);
    for (size_t k = 0; k < n_cls; ++k) {
        new_id[(size_t)order[k]] = (int32_t)k;
        (*first_rows)[k] = first_of[(size_t)order[k]];
    }
    for (size_t i = 0; i < n; ++i) (*map_out)[(size_t)rows[i]] = new_id[(size_t)cls[(size_t)rows[i]]];
    return TDFA_OK;
}

// Device memory of one call, freed when it ends.
struct Arena {
    std::vector<void*> blocks;
    template <class T>
    hipError_t get(T** p, size_t n)
    {
        void* v = nullptr;
        const hipError_t e = hipMalloc(&v, std::max<size_t>(n, 1) * sizeof(T));
        if (e == hipSuccess) blocks.push_back(v);
        *p = static_cast<T*>(v);
        return e;
    }
    ~Arena()
    {
        for (void* b : blocks) (void)hipFree(b);
    }
};

constexpr int kNotSparse = -1000;       // minimize_lists: take the dense path

// The sparse path.  Returns kNotSparse when a row has too many distinct targets or the final
// comparison fails (two different rows with one signature).
int minimize_lists(const int32_t* delta, int32_t n_rows, int32_t n_tokens, const uint8_t* accept, const int32_t* starts,
                   int32_t n_starts, hipStream_t s, std::vector<int32_t>* first_rows, std::vector<int32_t>* map_out)
{
    const unsigned long long seed = 0x243F6A8885A308D3ull;
    Arena mem;
    unsigned long long *counter, *row_begin, *e_weight = nullptr, *key, *ht_key;
    int32_t *row_n, *e_target = nullptr, *flags, *cls_a, *cls_b, *ht_min, *rows_dev, *first_dev;
    uint32_t* slot_of;
    uint8_t *mark, *aux, *good, *accept_dev;
    uint32_t ht_size = 1024;
    while (ht_size < 2u * (uint32_t)n_rows && ht_size < 0x80000000u) ht_size <<= 1;
    TDFA_HIP(mem.get(&counter, 1));
    TDFA_HIP(mem.get(&row_begin, n_rows));
    TDFA_HIP(mem.get(&row_n, n_rows));
    TDFA_HIP(mem.get(&flags, 2));                  // [0] too many targets / changed / mismatch, [1] classes
    TDFA_HIP(mem.get(&key, n_rows));
    TDFA_HIP(mem.get(&ht_key, ht_size));
    TDFA_HIP(mem.get(&ht_min, ht_size));
    TDFA_HIP(mem.get(&slot_of, n_rows));
    TDFA_HIP(mem.get(&cls_a, n_rows));
    TDFA_HIP(mem.get(&cls_b, n_rows));
    TDFA_HIP(mem.get(&mark, n_rows));
    TDFA_HIP(mem.get(&aux, n_rows));
    TDFA_HIP(mem.get(&good, n_rows));
    TDFA_HIP(mem.get(&accept_dev, n_rows));
    int32_t flag = 0;

    // ---- the lists: one pass over the table (a second one when they need more room than guessed)
    unsigned long long e_cap = std::max<unsigned long long>(1u << 20, std::min<unsigned long long>((unsigned long long)n_rows * 512, 1ull << 26));
    for (int attempt = 0;; ++attempt) {
        TDFA_HIP(mem.get(&e_target, e_cap));
        TDFA_HIP(mem.get(&e_weight, e_cap));
        TDFA_HIP(hipMemsetAsync(counter, 0, 8, s));
        TDFA_HIP(hipMemsetAsync(flags, 0, 8, s));
        row_targets_kernel<<<(unsigned)n_rows, kListThreads, 0, s>>>(delta, n_tokens, seed, e_cap, counter, row_begin, row_n, e_target,
                                                                      e_weight, flags);
        TDFA_HIP(hipGetLastError());
        unsigned long long total = 0;
        TDFA_HIP(hipMemcpyAsync(&total, counter, 8, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipMemcpyAsync(&flag, flags, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        if (flag) return kNotSparse;
        if (total <= e_cap) break;
        if (attempt == 1) return fail(TDFA_E_DEVICE, "the lists of targets changed size between two passes");
        e_cap = total;
    }
    const Lists g = {row_begin, row_n, e_target, e_weight, n_rows};
    const unsigned by_wave = (unsigned)(((size_t)n_rows + kRowsPerBlock - 1) / kRowsPerBlock);
    const unsigned by_thread = (unsigned)(((size_t)n_rows + kThreads - 1) / kThreads);
    constexpr int kRoundsPerLook = 4;              // rounds between two looks at the flag

    // ---- states that a token sequence reaches, then of those the ones that reach a final state
    std::vector<uint8_t> mark_h((size_t)n_rows, 0);
    for (int32_t i = 0; i < n_starts; ++i) mark_h[(size_t)starts[i]] = 1;
    TDFA_HIP(hipMemcpyAsync(mark, mark_h.data(), (size_t)n_rows, hipMemcpyHostToDevice, s));
    TDFA_HIP(hipMemcpyAsync(accept_dev, accept, (size_t)n_rows, hipMemcpyHostToDevice, s));
    TDFA_HIP(hipMemsetAsync(aux, 0, (size_t)n_rows, s));
    TDFA_HIP(hipMemsetAsync(slot_of, 0, (size_t)n_rows * 4, s));
    for (flag = 1; flag;) {
        TDFA_HIP(hipMemsetAsync(flags, 0, 4, s));
        for (int r = 0; r < kRoundsPerLook; ++r) list_reach_kernel<<<by_wave, kThreads, 0, s>>>(g, mark, aux, flags);
        TDFA_HIP(hipGetLastError());
        TDFA_HIP(hipMemcpyAsync(&flag, flags, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
    }
    list_good_start_kernel<<<by_thread, kThreads, 0, s>>>(n_rows, mark, accept_dev, good);
    for (flag = 1; flag;) {
        TDFA_HIP(hipMemsetAsync(flags, 0, 4, s));
        for (int r = 0; r < kRoundsPerLook; ++r) list_reach_final_kernel<<<by_wave, kThreads, 0, s>>>(g, mark, good, flags);
        TDFA_HIP(hipGetLastError());
        TDFA_HIP(hipMemcpyAsync(&flag, flags, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
    }

    // ---- refinement: classes named by their smallest row
    int32_t *cls = cls_a, *cls_next = cls_b;
    list_first_keys_kernel<<<by_thread, kThreads, 0, s>>>(n_rows, mark, good, accept_dev, seed, cls, key);
    int32_t n_cls = 0;
    for (int32_t prev = -1;; prev = n_cls) {
        TDFA_HIP(hipMemsetAsync(ht_key, 0, (size_t)ht_size * 8, s));
        fill_i32_kernel<<<(ht_size + kThreads - 1) / kThreads, kThreads, 0, s>>>(ht_min, ht_size, 0x7FFFFFFF);
        TDFA_HIP(hipMemsetAsync(flags + 1, 0, 4, s));
        list_insert_kernel<<<by_thread, kThreads, 0, s>>>(n_rows, cls, key, ht_key, ht_min, ht_size - 1, slot_of);
        list_assign_kernel<<<by_thread, kThreads, 0, s>>>(n_rows, cls, slot_of, ht_min, cls_next, flags + 1);
        std::swap(cls, cls_next);
        list_keys_kernel<<<by_wave, kThreads, 0, s>>>(g, cls, seed, key);       // for the next round
        TDFA_HIP(hipGetLastError());
        TDFA_HIP(hipMemcpyAsync(&n_cls, flags + 1, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        if (n_cls == prev) break;
    }
    std::vector<int32_t> cls_h((size_t)n_rows);
    TDFA_HIP(hipMemcpyAsync(cls_h.data(), cls, (size_t)n_rows * 4, hipMemcpyDeviceToHost, s));
    TDFA_HIP(hipStreamSynchronize(s));

    // ---- every row that joined another one is compared with it
    std::vector<int32_t> joined, with;
    for (int32_t q = 0; q < n_rows; ++q) {
        const int32_t c = cls_h[(size_t)q];
        if (c < 0 || c == q) continue;
        if (c > q || cls_h[(size_t)c] != c || (accept[q] != 0) != (accept[c] != 0)) return kNotSparse;
        joined.push_back(q);
        with.push_back(c);
    }
    if (!joined.empty() && n_tokens > 0) {
        TDFA_HIP(mem.get(&rows_dev, joined.size()));
        TDFA_HIP(mem.get(&first_dev, joined.size()));
        TDFA_HIP(hipMemcpyAsync(rows_dev, joined.data(), joined.size() * 4, hipMemcpyHostToDevice, s));
        TDFA_HIP(hipMemcpyAsync(first_dev, with.data(), with.size() * 4, hipMemcpyHostToDevice, s));
        TDFA_HIP(hipMemsetAsync(flags, 0, 4, s));
        const unsigned gx = grid_x(n_tokens);
        for (size_t lo = 0; lo < joined.size(); lo += kMaxGridY) {
            verify_classes_kernel<<<dim3(gx, (unsigned)std::min(kMaxGridY, joined.size() - lo)), kThreads, 0, s>>>(
                delta, n_tokens, rows_dev + lo, first_dev + lo, cls, flags);
            TDFA_HIP(hipGetLastError());
        }
        TDFA_HIP(hipMemcpyAsync(&flag, flags, 4, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        if (flag) return kNotSparse;
    }

    // ---- the classes in the order of their smallest states
    map_out->assign((size_t)n_rows, TDFA_DEAD);
    first_rows->clear();
    for (int32_t q = 0; q < n_rows; ++q)
        if (cls_h[(size_t)q] == q) {
            (*map_out)[(size_t)q] = (int32_t)first_rows->size();
            first_rows->push_back(q);
        }
    for (int32_t q = 0; q < n_rows; ++q)
        if (cls_h[(size_t)q] >= 0) (*map_out)[(size_t)q] = (*map_out)[(size_t)cls_h[(size_t)q]];
    return TDFA_OK;
}

}  // namespace

int minimize_table(const int32_t* delta, int64_t n_rows64, int32_t n_tokens, const uint8_t* accept, const int32_t* starts,
                   int32_t n_starts, hipStream_t s, std::vector<int32_t>* first_rows, std::vector<int32_t>* map_out)
{
    const int32_t n_rows = (int32_t)n_rows64;
    const int rc = minimize_lists(delta, n_rows, n_tokens, accept, starts, n_starts, s, first_rows, map_out);
    if (rc != kNotSparse) return rc;
    return minimize_dense(delta, n_rows, n_tokens, accept, starts, n_starts, s, first_rows, map_out);
}

int launch_compact_rows(const int32_t* delta, int32_t n_tokens, int64_t row_words, const std::vector<int32_t>& first_rows,
                        const std::vector<int32_t>& map, int32_t* out_delta, uint32_t* out_allow, hipStream_t s)
{
    if (first_rows.empty()) return TDFA_OK;
    DeviceBuffers d;
    TDFA_HIP(hipMalloc(&d.rows, first_rows.size() * 4));
    TDFA_HIP(hipMalloc(&d.aux, map.size() * 4));
    TDFA_HIP(hipMemcpyAsync(d.rows, first_rows.data(), first_rows.size() * 4, hipMemcpyHostToDevice, s));
    TDFA_HIP(hipMemcpyAsync(d.aux, map.data(), map.size() * 4, hipMemcpyHostToDevice, s));
    const unsigned bx = (unsigned)((row_words * 32 + kThreads - 1) / kThreads);
    for (size_t lo = 0; lo < first_rows.size(); lo += kMaxGridY) {
        compact_rows_kernel<<<dim3(bx, (unsigned)std::min(kMaxGridY, first_rows.size() - lo)), kThreads, 0, s>>>(
            delta, n_tokens, row_words, d.rows + lo, d.aux, out_delta + lo * (size_t)n_tokens, out_allow + lo * (size_t)row_words);
        TDFA_HIP(hipGetLastError());
    }
    TDFA_HIP(hipStreamSynchronize(s));
    return TDFA_OK;
}

}  // namespace tdfa
