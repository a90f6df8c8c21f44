// Token-level optimisation of a compiled table (Appendix C.2, the fourth of the compile operations it
// times, applied to the composed automaton).  The paper does not name the optimisation; the reading taken is the
// classical one for a deterministic automaton: keep the states that some token sequence reaches
// from a start state and from which a final state can be reached, and merge the states that accept
// the same token sequences (Moore's partition refinement).  A set-up call: the host drives the
// rounds and waits for each; the kernels stream table rows.
//
//   reach      level by level from the start states: the rows of the frontier are scanned and their
//              targets marked
//   co-reach   rounds over the rows not yet known to reach a final state: a row with an entry
//              into such a state becomes one
//   refine     every round hashes, for each kept row, the classes of its 'n_tokens' targets (a
//              sum of mixed (token, class) pairs, so it reduces in any order); rows of one class
//              with different hashes are split.  When no class splits any more, every row is
//              compared entry by entry with its class's first row: the hash only ever decides
//              that two rows differ, never that they are equal.
//   compact    the first row of each class, its entries renamed, is a row of the new table
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

}  // namespace

int minimize_table(const int32_t* delta, int64_t n_rows64, int32_t n_tokens, const uint8_t* accept, const int32_t* starts,
                   int32_t n_starts, hipStream_t s, std::vector<int32_t>* first_rows, std::vector<int32_t>* map_out)
{
    const int32_t n_rows = (int32_t)n_rows64;
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
