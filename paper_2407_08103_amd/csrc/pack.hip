// Edge-list form of a compiled table.  The paper keeps A_{R o V} as a list of edges and remarks
// (Section 2.5.1) that it is the states with near-|V| out-degree that make this costly; the dense
// table pays |V| entries for every state instead, though most states of a constraint automaton
// allow a handful of tokens.  The packed form keeps what both need: the allowed-bit row of every
// state (the decode step streams it as before) and, in place of the dense row, only the targets
// of its edges, in token order.  The token of an edge is not stored: it is the position of the
// edge among the set bits of the row, found with a directory of per-128-token counts:
//
//   delta_T[q][t] = targets[row_begin[q] + dir[q][t / 128] + popcount(bits of q in [128 (t / 128), t))]
//
// Size: 4 B per edge + |V| (1/8 + 1/32) B per state; never more than the dense row plus 4 %.
// A set-up call: the host sums the per-state counts between the two kernels and waits for them.
#include <new>
#include <vector>

#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kThreads = 256;

// The bits of word `wi` of a row that stand for tokens: padding bits never count as edges.
__device__ __forceinline__ uint32_t token_bits(uint32_t w, int wi, int32_t n_tokens)
{
    const int rem = n_tokens - 32 * wi;
    return rem >= 32 ? w : (rem <= 0 ? 0u : w & ((1u << rem) - 1u));
}

__device__ __forceinline__ uint32_t block_count(const uint4* row, int k, int32_t n_tokens)
{
    const uint4 w = row[k];
    return __popc(token_bits(w.x, 4 * k, n_tokens)) + __popc(token_bits(w.y, 4 * k + 1, n_tokens)) +
           __popc(token_bits(w.z, 4 * k + 2, n_tokens)) + __popc(token_bits(w.w, 4 * k + 3, n_tokens));
}

// One workgroup per state: dir[q][k] for every block of 128 tokens, and the state's edge count.
__global__ void __launch_bounds__(kThreads)
pack_count_kernel(const uint32_t* __restrict__ allow, int32_t n_tokens, int64_t row_words, int32_t n_blocks,
                  uint32_t* __restrict__ dir, uint32_t* __restrict__ row_count)
{
    __shared__ uint32_t s_sum[kThreads];
    const int64_t q = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(allow + q * row_words);
    // thread i owns the contiguous blocks [i * per, (i + 1) * per)
    const int per = (n_blocks + kThreads - 1) / kThreads;
    const int k_lo = min(n_blocks, (int)threadIdx.x * per), k_hi = min(n_blocks, k_lo + per);
    uint32_t mine = 0;
    for (int k = k_lo; k < k_hi; ++k) mine += block_count(row, k, n_tokens);
    s_sum[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < kThreads; d <<= 1) {              // inclusive scan of the per-thread sums
        const uint32_t add = threadIdx.x >= (unsigned)d ? s_sum[threadIdx.x - d] : 0u;
        __syncthreads();
        s_sum[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t before = s_sum[threadIdx.x] - mine;
    for (int k = k_lo; k < k_hi; ++k) {
        dir[q * n_blocks + k] = before;
        before += block_count(row, k, n_tokens);
    }
    if (threadIdx.x == kThreads - 1) row_count[q] = s_sum[kThreads - 1];
}

// One workgroup per state: the targets of its edges in token order.  A wavefront takes 64 tokens at a
// time, one per lane: the entries are read and the targets written side by side, an edge's
// position being the directory count of its block plus the set bits below it.
__global__ void __launch_bounds__(kThreads)
pack_targets_kernel(const int32_t* __restrict__ delta, const uint32_t* __restrict__ allow, int32_t n_tokens,
                    int64_t row_words, int32_t n_blocks, const uint32_t* __restrict__ dir,
                    const int64_t* __restrict__ row_begin, int32_t* __restrict__ targets)
{
    const int64_t q = blockIdx.x;
    const uint32_t* bits = allow + q * row_words;
    const int32_t* row = delta + q * n_tokens;
    int32_t* out = targets + row_begin[q];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_chunks = (int)(row_words / 2);                   // 64 tokens each; two per directory block
    for (int c = wave; c < n_chunks; c += kThreads / 64) {
        const uint32_t lo = token_bits(bits[2 * c], 2 * c, n_tokens), hi = token_bits(bits[2 * c + 1], 2 * c + 1, n_tokens);
        const unsigned long long mask = ((unsigned long long)hi << 32) | lo;
        if (mask == 0) continue;                                  // the same in all lanes
        uint32_t base = dir[q * n_blocks + (c >> 1)];
        if (c & 1) base += __popc(token_bits(bits[2 * c - 2], 2 * c - 2, n_tokens)) + __popc(token_bits(bits[2 * c - 1], 2 * c - 1, n_tokens));
        if ((mask >> lane) & 1ull) out[base + __popcll(mask & ((1ull << lane) - 1ull))] = row[64 * c + lane];
    }
}

// One workgroup per state: how many tokens it allows.
__global__ void __launch_bounds__(kThreads)
row_allowed_kernel(const uint32_t* __restrict__ allow, int32_t n_tokens, int64_t row_words, uint32_t* __restrict__ out)
{
    __shared__ uint32_t s_part[kThreads / 64];
    const int64_t q = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(allow + q * row_words);
    uint32_t mine = 0;
    for (int k = threadIdx.x; k < (int)(row_words / 4); k += kThreads) mine += block_count(row, k, n_tokens);
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        for (int w = 0; w < kThreads / 64; ++w) total += s_part[w];
        out[q] = total;
    }
}

}  // namespace

int launch_row_allowed(const uint32_t* allow, int64_t n_rows, int32_t n_tokens, int64_t row_words, uint32_t* out, hipStream_t stream)
{
    if (n_rows <= 0) return TDFA_OK;
    row_allowed_kernel<<<(unsigned)n_rows, kThreads, 0, stream>>>(allow, n_tokens, row_words, out);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

int pack_table(const int32_t* delta, const uint32_t* allow, int64_t n_rows, int32_t n_tokens, int64_t row_words,
               hipStream_t stream, uint32_t** dir_out, int64_t** row_begin_out, int32_t** targets_out, int64_t* n_edges_out)
{
    const int32_t n_blocks = (int32_t)(row_words / 4);
    uint32_t* dir = nullptr;
    uint32_t* counts = nullptr;
    int64_t* row_begin = nullptr;
    int32_t* targets = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(dir);
        (void)hipFree(counts);
        (void)hipFree(row_begin);
        (void)hipFree(targets);
    };
#define PACK_HIP(expr)                                                                          \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            cleanup();                                                                          \
            return fail(e_ == hipErrorOutOfMemory ? TDFA_E_OOM : TDFA_E_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
        }                                                                                       \
    } while (0)
    const size_t rows = (size_t)(n_rows > 0 ? n_rows : 1);
    PACK_HIP(hipMalloc(reinterpret_cast<void**>(&dir), rows * (size_t)(n_blocks > 0 ? n_blocks : 1) * sizeof(uint32_t)));
    PACK_HIP(hipMalloc(reinterpret_cast<void**>(&counts), rows * sizeof(uint32_t)));
    PACK_HIP(hipMalloc(reinterpret_cast<void**>(&row_begin), (rows + 1) * sizeof(int64_t)));
    std::vector<uint32_t> h_counts;
    std::vector<int64_t> h_begin;
    try {
        h_counts.resize((size_t)n_rows);
        h_begin.resize((size_t)n_rows + 1);
    } catch (const std::bad_alloc&) {
        cleanup();
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    // grids of at most 2^31 - 1 workgroups: one per state
    if (n_rows > 0) {
        pack_count_kernel<<<(unsigned)n_rows, kThreads, 0, stream>>>(allow, n_tokens, row_words, n_blocks, dir, counts);
        PACK_HIP(hipGetLastError());
        PACK_HIP(hipMemcpyAsync(h_counts.data(), counts, (size_t)n_rows * sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
    }
    PACK_HIP(hipStreamSynchronize(stream));
    int64_t n_edges = 0;
    for (int64_t q = 0; q < n_rows; ++q) {
        h_begin[(size_t)q] = n_edges;
        n_edges += h_counts[(size_t)q];
    }
    h_begin[(size_t)n_rows] = n_edges;
    PACK_HIP(hipMalloc(reinterpret_cast<void**>(&targets), (size_t)(n_edges > 0 ? n_edges : 1) * sizeof(int32_t)));
    PACK_HIP(hipMemcpyAsync(row_begin, h_begin.data(), ((size_t)n_rows + 1) * sizeof(int64_t), hipMemcpyHostToDevice, stream));
    if (n_rows > 0 && n_edges > 0) {
        pack_targets_kernel<<<(unsigned)n_rows, kThreads, 0, stream>>>(delta, allow, n_tokens, row_words, n_blocks, dir,
                                                                     row_begin, targets);
        PACK_HIP(hipGetLastError());
    }
    PACK_HIP(hipStreamSynchronize(stream));                // h_begin is read by the copy until here
#undef PACK_HIP
    (void)hipFree(counts);
    *dir_out = dir;
    *row_begin_out = row_begin;
    *targets_out = targets;
    *n_edges_out = n_edges;
    return TDFA_OK;
}

}  // namespace tdfa
