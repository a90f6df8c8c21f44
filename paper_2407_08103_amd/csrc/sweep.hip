// Compile stage for large automata: delta_T by sweeping the vocabulary's prefix trie level by level
// with the automaton's columns held in LDS (Sections 2.3-2.4; Algorithm 2, statement 3).
//
// delta_T[q][t] = delta*(q, d(t)).  For a large automaton whose states reject most bytes, almost
// every walk dies within a few bytes, and what costs is not arithmetic but the scattered reads
// delta(r, b) with r anywhere in the table.  Here no such read leaves the compute unit: the work is
// ordered by the byte that is read next, and a workgroup keeps that byte's column delta(., b)
// (2 |Q| bytes) in LDS.  What moves through global memory are lists of the (state, target) pairs
// that are still alive, read and written front to back:
//
//   level 2   sweep_prefix_kernel: for every two-byte prefix (b1, b2) the list of (q, delta*(q, b1 b2)),
//             q ascending.  The compact T_V (Section 2.3) shares these among all tokens that begin
//             with (b1, b2): at most 65,536 lists however large the vocabulary is.
//   level 3   sweep_token_kernel<3>: for every token of three or more bytes, its prefix's list filtered
//             through the column of its third byte; tokens are grouped by that byte (a table made
//             once per vocabulary), a workgroup takes a few tokens of one group.
//   level 4   the same with the fourth byte, from the lists of level 3.
//   tail      sweep_tail_kernel: the few pairs that survive four bytes are walked to the end of
//             their token by one wavefront per token, in place.
//   expand    sweep_expand_kernel: the lists (q ascending) of 256 consecutive tokens are merged into
//             dense rows, 256 states at a time through an LDS tile, and leave with 16-byte
//             streaming stores; the allowed bits of the 256 tokens are written as whole 32-byte
//             sectors.  One-byte tokens take their column directly.
//
// A list may not be longer than the list it was filtered from, so every token owns a region as
// long as its prefix's list in each of two buffers, and no level has to be counted before it is
// written.
#include <algorithm>

#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kWgThreads = 512;
constexpr int kWgWaves = kWgThreads / 64;
constexpr int kPrefixPerWg = 16;      // first bytes b1 per workgroup of sweep_prefix_kernel (two per wavefront)
constexpr uint32_t kNoPair = 0xFFFFFFFFu;

struct SweepDesc {
    const uint16_t* tt;        // [256][q_stride] transposed table, offset form (entry = state * 2, sink = (q_stride - 1) * 2)
    int32_t n_states, q_stride;
    uint32_t* n1;              // [256] live states per column
    uint32_t* off1;            // [257] their exclusive sums
    uint32_t* list1;           // [off1[256]] per column the (q << 16) | target of its live states, q ascending
    uint32_t* list2;           // the list of prefix (b1, b2) starts at 256 * off1[b1] + b2 * n1[b1]; entry = (q << 16) | target
    uint32_t* cnt2;            // [65536] its length
    uint32_t* need;            // [n_tokens + 1] where the token's region begins in buf_a / buf_b
    unsigned long long* chunk_sum;   // [n_tokens / 1024 + 2] scratch of the scan; the last entry is the total
    uint32_t* cnt3;            // [n_tokens] pairs alive after three bytes (bufA)
    uint32_t* cntF;            // [n_tokens] tokens of four or more bytes: pairs alive at the end of the token (bufB)
    uint32_t* buf_a;
    uint32_t* buf_b;
    uint64_t buf_cap;          // entries in each of the two buffers
    uint32_t* err;             // set to 1 if a region would not fit (nothing is written outside)
    int32_t out_row, state_base;
};

struct SweepVocab {
    const uint32_t* vwords;
    const uint32_t* voff;
    const uint32_t* vlen;
    const uint32_t* vprefix;
    const int32_t* group_tokens[2];   // tokens with a third / fourth byte, grouped by that byte
    const int32_t* group_chunks[2];   // [n_chunks][3]: byte, first index into group_tokens, number of tokens (<= 16)
    int32_t n_chunks[2];
    const int32_t* tail_tokens;       // tokens of five or more bytes
    int32_t n_tail;
    int32_t n_tokens;
};

__device__ __forceinline__ uint32_t lanes_below(unsigned long long bal)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
}

__device__ __forceinline__ uint32_t prefix_of(const SweepVocab& v, int32_t t)
{
    const uint32_t w0 = v.vprefix[(size_t)t * 8];
    return ((w0 & 0xFFu) << 8) | ((w0 >> 8) & 0xFFu);
}

// n1[b] = states with an edge on byte b
__global__ void __launch_bounds__(256)
sweep_column_count_kernel(SweepDesc d)
{
    __shared__ uint32_t s_part[4];
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    const uint16_t* col = d.tt + (size_t)blockIdx.x * d.q_stride;
    uint32_t c = 0;
    for (int q = threadIdx.x; q < d.n_states; q += 256) c += col[q] != sink;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) c += __shfl_xor(c, s, 64);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) d.n1[blockIdx.x] = s_part[0] + s_part[1] + s_part[2] + s_part[3];
}

__global__ void __launch_bounds__(256)
sweep_column_scan_kernel(SweepDesc d)
{
    __shared__ uint32_t s_wave[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t v = d.n1[threadIdx.x];
    uint32_t incl = v;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const uint32_t o = __shfl_up(incl, s, 64);
        if (lane >= s) incl += o;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    d.off1[threadIdx.x] = before + incl - v;
    if (threadIdx.x == 255) d.off1[256] = before + incl;
}

// Level 1: list1[off1[b] ..] = (q << 16) | delta(q, b) for the states with an edge on b, q ascending.
__global__ void __launch_bounds__(256)
sweep_first_kernel(SweepDesc d)
{
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_carry;
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    const uint16_t* col = d.tt + (size_t)blockIdx.x * d.q_stride;
    uint32_t* out = d.list1 + d.off1[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int q0 = 0; q0 < d.n_states; q0 += 256) {
        const int q = q0 + (int)threadIdx.x;
        const uint32_t e = q < d.n_states ? (uint32_t)col[q] : sink;
        const bool live = e != sink;
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(live);
        if (lane == 0) s_wave[wave] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t pos = s_carry, all = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) pos += s_wave[w];
            all += s_wave[w];
        }
        if (live) out[pos + lanes_below(bal)] = ((uint32_t)q << 16) | (e >> 1);
        __syncthreads();
        if (threadIdx.x == 0) s_carry += all;
        __syncthreads();
    }
}

// Level 2.  Workgroup (b2, sixteen first bytes): the column of b2 in LDS; a wavefront filters the list of one
// b1 through it.
__global__ void __launch_bounds__(kWgThreads)
sweep_prefix_kernel(SweepDesc d)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* col = reinterpret_cast<uint16_t*>(smem);
    const int b2 = (int)blockIdx.x;
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(d.tt + (size_t)b2 * d.q_stride);
        uint32_t* dst = reinterpret_cast<uint32_t*>(col);
        for (int i = threadIdx.x; i < d.q_stride / 2; i += kWgThreads) dst[i] = src[i];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int k = wave; k < kPrefixPerWg; k += kWgWaves) {
        const int b1 = (int)blockIdx.y * kPrefixPerWg + k;
        const uint32_t n_in = d.n1[b1];
        const uint32_t* in = d.list1 + d.off1[b1];
        uint32_t* out = d.list2 + (size_t)256 * d.off1[b1] + (size_t)b2 * n_in;
        uint32_t pos = 0;
        for (uint32_t k0 = 0; k0 < n_in; k0 += 256) {
            uint32_t en[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = k0 + 64u * u + (uint32_t)lane;
                en[u] = i < n_in ? in[i] : kNoPair;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t x = en[u] != kNoPair ? (uint32_t)col[en[u] & 0xFFFFu] : sink;
                const bool live = x != sink;
                const unsigned long long bal = __builtin_amdgcn_ballot_w64(live);
                if (live) out[pos + lanes_below(bal)] = (en[u] & 0xFFFF0000u) | (x >> 1);
                pos += (uint32_t)__popcll(bal);
            }
        }
        if (lane == 0) d.cnt2[b1 * 256 + b2] = pos;
    }
}

// need[t] = where token t's region begins in the two buffers: the exclusive prefix sums of the lengths of
// the tokens' prefix lists (tokens of three or more bytes; the others need nothing), need[n_tokens] =
// their total.  Three steps: sums inside chunks of 1,024 tokens, a scan of the chunk sums, the addition.
__global__ void __launch_bounds__(1024)
sweep_need_chunks_kernel(SweepDesc d, SweepVocab v)
{
    __shared__ uint32_t s_wave[16];
    const int t = (int)(blockIdx.x * 1024 + threadIdx.x);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t n = 0;
    if (t < v.n_tokens && v.vlen[t] >= 3) n = d.cnt2[prefix_of(v, t)];
    uint32_t incl = n;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const uint32_t o = __shfl_up(incl, s, 64);
        if (lane >= s) incl += o;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if (t <= v.n_tokens) d.need[t] = before + incl - n;          // at most 1,024 lists of fewer than 32,768 pairs: no overflow
    if (threadIdx.x == 1023) d.chunk_sum[blockIdx.x] = (unsigned long long)(before + incl);
}

__global__ void __launch_bounds__(1024)
sweep_need_scan_kernel(SweepDesc d, int32_t n_chunks)
{
    __shared__ unsigned long long s_wave[16];
    __shared__ unsigned long long s_carry;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < n_chunks; base += 1024) {
        const int i = base + (int)threadIdx.x;
        const unsigned long long val = i < n_chunks ? d.chunk_sum[i] : 0ull;
        unsigned long long incl = val;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const unsigned long long o = __shfl_up(incl, s, 64);
            if (lane >= s) incl += o;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        unsigned long long before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        if (i < n_chunks) d.chunk_sum[i] = before + incl - val;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        d.chunk_sum[n_chunks] = s_carry;                         // the total, for the host that sizes the buffers
        if (s_carry > d.buf_cap) *d.err = 1u;                    // a total beyond the buffers: nothing will be written
    }
}

__global__ void __launch_bounds__(1024)
sweep_need_add_kernel(SweepDesc d, int32_t n_tokens)
{
    const int t = (int)(blockIdx.x * 1024 + threadIdx.x);
    if (t > n_tokens) return;
    const unsigned long long x = d.chunk_sum[blockIdx.x] + d.need[t];
    d.need[t] = x > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)x;
}

// Levels 3 and 4.  Workgroup = up to sixteen tokens whose byte at this level is the same: that byte's
// column in LDS, a wavefront filters one token's list through it at a time.
template <int LEVEL>
__global__ void __launch_bounds__(kWgThreads)
sweep_token_kernel(SweepDesc d, SweepVocab v)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* col = reinterpret_cast<uint16_t*>(smem);
    const int32_t* chunk = v.group_chunks[LEVEL - 3] + (size_t)blockIdx.x * 3;
    const int byte = chunk[0], first = chunk[1], n_tok = chunk[2];
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(d.tt + (size_t)byte * d.q_stride);
        uint32_t* dst = reinterpret_cast<uint32_t*>(col);
        for (int i = threadIdx.x; i < d.q_stride / 2; i += kWgThreads) dst[i] = src[i];
    }
    __syncthreads();
    if (*d.err) return;                                       // the buffers are too small: nothing may be written
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int k = wave; k < n_tok; k += kWgWaves) {
        const int32_t t = v.group_tokens[LEVEL - 3][first + k];
        const uint32_t region = d.need[t];
        const uint32_t* in;
        uint32_t n_in;
        uint32_t* out;
        if (LEVEL == 3) {
            const uint32_t p = prefix_of(v, t), b1 = p >> 8;
            in = d.list2 + (size_t)256 * d.off1[b1] + (size_t)(p & 255u) * d.n1[b1];
            n_in = d.cnt2[p];
            out = d.buf_a + region;
        } else {
            in = d.buf_a + region;
            n_in = d.cnt3[t];
            out = d.buf_b + region;
        }
        uint32_t pos = 0;
        for (uint32_t k0 = 0; k0 < n_in; k0 += 256) {
            uint32_t en[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = k0 + 64u * u + (uint32_t)lane;
                en[u] = i < n_in ? in[i] : kNoPair;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t x = en[u] != kNoPair ? (uint32_t)col[en[u] & 0xFFFFu] : sink;
                const bool live = x != sink;
                const unsigned long long bal = __builtin_amdgcn_ballot_w64(live);
                if (live) out[pos + lanes_below(bal)] = (en[u] & 0xFFFF0000u) | (x >> 1);
                pos += (uint32_t)__popcll(bal);
            }
        }
        if (lane == 0) (LEVEL == 3 ? d.cnt3 : d.cntF)[t] = pos;
    }
}

// Bytes five and later: one wavefront per token of five or more bytes walks what is left of its list (bufB)
// to the end of the token, in place; these are the few long walks, read from the table in memory.
__global__ void __launch_bounds__(256)
sweep_tail_kernel(SweepDesc d, SweepVocab v)
{
    const int lane = threadIdx.x & 63;
    const int i = (int)(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (i >= v.n_tail || *d.err) return;
    const int32_t t = v.tail_tokens[i];
    const uint32_t len = v.vlen[t];
    const uint8_t* bytes = reinterpret_cast<const uint8_t*>(v.vwords) + (size_t)v.voff[t] * 4;
    uint32_t* list = d.buf_b + d.need[t];
    uint32_t n = d.cntF[t];
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    for (uint32_t at = 4; at < len && n > 0; ++at) {
        const uint16_t* col = d.tt + (size_t)bytes[at] * d.q_stride;
        uint32_t pos = 0;
        for (uint32_t k0 = 0; k0 < n; k0 += 64) {
            const uint32_t k = k0 + (uint32_t)lane;
            const uint32_t en = k < n ? list[k] : kNoPair;
            const uint32_t x = en != kNoPair ? (uint32_t)col[en & 0xFFFFu] : sink;
            const bool live = x != sink;
            const unsigned long long bal = __builtin_amdgcn_ballot_w64(live);
            // written places lie at or before the places this round has read
            if (live) list[pos + lanes_below(bal)] = (en & 0xFFFF0000u) | (x >> 1);
            pos += (uint32_t)__popcll(bal);
        }
        n = pos;
    }
    if (lane == 0) d.cntF[t] = n;
}

// ---- expand

constexpr int kXS = 256;          // states per tile
constexpr int kXT = 64;           // tokens per sub-tile
constexpr int kXSub = 4;
constexpr int kXBlockT = kXT * kXSub;
constexpr int kXRS = kXT + 2;     // tile row stride in 16-bit entries: an odd number of 32-bit words
constexpr size_t kXTileBytes = (size_t)kXS * kXRS * 2;
// tile, allowed bits, per token: list pointer (8), end (4), length class (4)
constexpr size_t kXLdsBytes = kXTileBytes + (size_t)kXS * 8 * 4 + (size_t)kXBlockT * (8 + 4 + 4);
static_assert(3 * kXLdsBytes <= 160 * 1024, "three workgroups per compute unit");

// Workgroup (block of 256 tokens, run of state tiles).  Per token a cursor into its list (q ascending);
// per tile of 256 states the pairs below the tile's upper bound are taken off the lists into the LDS
// tile, 64 tokens at a time with eight lanes per token, and the rows are flushed.
template <bool WIDE_ROWS, bool BASE0>
__global__ void __launch_bounds__(kWgThreads) __attribute__((amdgpu_waves_per_eu(6, 6)))
sweep_expand_kernel(SweepDesc d, SweepVocab v, int n_blocks_t, int tiles_per_run, int n_tiles_q, int32_t* __restrict__ delta,
                    uint32_t* __restrict__ allow, int64_t row_words, int allow_vec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* tile = reinterpret_cast<uint16_t*>(smem);
    uint32_t* s_bits = reinterpret_cast<uint32_t*>(smem + kXTileBytes);          // [kXS][8]
    const uint32_t** s_list = reinterpret_cast<const uint32_t**>(s_bits + kXS * 8);   // [kXBlockT] start of the token's list
    uint32_t* s_end = reinterpret_cast<uint32_t*>(s_list + kXBlockT);             // [kXBlockT] its length
    int32_t* s_kind = reinterpret_cast<int32_t*>(s_end + kXBlockT);               // [kXBlockT] -1: a list; 0 .. 255: a one-byte token's byte; -2: nothing

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int bt = (int)(blockIdx.x % (unsigned)n_blocks_t), run = (int)(blockIdx.x / (unsigned)n_blocks_t);
    const int qt_lo = run * tiles_per_run, qt_hi = min(n_tiles_q, qt_lo + tiles_per_run);
    const int n_tokens = v.n_tokens, t_block = bt * kXBlockT;
    const uint32_t q_stride = (uint32_t)d.q_stride;
    const uint32_t SINK = (q_stride - 1u) * 2u;
    const int state_base = d.state_base;
    const uint32_t out_row32 = (uint32_t)d.out_row, nt32 = (uint32_t)n_tokens, rw32 = (uint32_t)row_words;

    // ---- set-up: where each token's list is, and where in it this run of tiles begins
    {
        uint32_t* w = reinterpret_cast<uint32_t*>(tile);
        for (int i = threadIdx.x; i < (int)(kXTileBytes / 4); i += kWgThreads) w[i] = 0u;      // entries are state + 1; 0 = DEAD
        for (int i = threadIdx.x; i < kXS * 8; i += kWgThreads) s_bits[i] = 0u;
    }
    uint32_t cur[kXSub];                                       // this thread's tokens: sub * 64 + threadIdx.x / 8
    if (threadIdx.x < kXBlockT) {
        const int tl = (int)threadIdx.x, t = t_block + tl;
        const uint32_t* list = nullptr;
        uint32_t n = 0;
        int kind = -2;
        if (t < n_tokens && !*d.err) {
            const uint32_t len = v.vlen[t];
            if (len == 1) {
                kind = (int)(v.vprefix[(size_t)t * 8] & 0xFFu);
            } else if (len == 2) {
                const uint32_t p = prefix_of(v, t), b1 = p >> 8;
                list = d.list2 + (size_t)256 * d.off1[b1] + (size_t)(p & 255u) * d.n1[b1];
                n = d.cnt2[p];
                kind = -1;
            } else if (len == 3) {
                list = d.buf_a + d.need[t];
                n = d.cnt3[t];
                kind = -1;
            } else if (len >= 4) {
                list = d.buf_b + d.need[t];
                n = d.cntF[t];
                kind = -1;
            }
        }
        s_list[tl] = list;
        s_end[tl] = n;
        s_kind[tl] = kind;
    }
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < kXSub; ++sub) {
        // the first pair at or above the run's first state (all eight lanes of a token search alike)
        const int tl = sub * kXT + ((int)threadIdx.x >> 3);
        const uint32_t* list = s_list[tl];
        uint32_t lo = 0, hi = s_end[tl];
        const uint32_t q_first = (uint32_t)qt_lo * kXS;
        if (q_first > 0) {
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if ((list[mid] >> 16) < q_first) lo = mid + 1;
                else hi = mid;
            }
        }
        cur[sub] = lo;
    }

    // the next eight pairs of each of this thread's four tokens: requested as soon as the cursor is known, one
    // tile ahead of their use, so that they arrive while the tile before is flushed
    uint32_t ahead[kXSub];
#pragma unroll
    for (int sub = 0; sub < kXSub; ++sub) {
        const int tl = sub * kXT + ((int)threadIdx.x >> 3);
        const uint32_t k = cur[sub] + ((uint32_t)threadIdx.x & 7u);
        ahead[sub] = k < s_end[tl] ? s_list[tl][k] : kNoPair;
    }
    for (int qt = qt_lo; qt < qt_hi; ++qt) {
        const uint32_t q_base = (uint32_t)qt * kXS, q_bound = q_base + kXS;
#pragma unroll
        for (int sub = 0; sub < kXSub; ++sub) {
            const int t0 = t_block + sub * kXT;
            if (t0 < n_tokens) {                               // uniform
                const int tls = (int)threadIdx.x >> 3;         // token inside the sub-tile
                const int tl = sub * kXT + tls;
                uint32_t en = ahead[sub];
                for (;;) {
                    const bool in_tile = en != kNoPair && (en >> 16) < q_bound;
                    if (in_tile) tile[((en >> 16) - q_base) * kXRS + tls] = (uint16_t)((en & 0xFFFFu) + 1u);
                    const unsigned long long bal = __builtin_amdgcn_ballot_w64(in_tile);
                    const uint32_t mine = (uint32_t)(bal >> (lane & ~7)) & 0xFFu;
                    cur[sub] += (uint32_t)__popc(mine);
                    // a token whose eight pairs all lay in the tile may have more there
                    const bool more = mine == 0xFFu;
                    if (__builtin_amdgcn_ballot_w64(more) == 0) break;
                    en = kNoPair;
                    if (more) {
                        const uint32_t k = cur[sub] + ((uint32_t)threadIdx.x & 7u);
                        if (k < s_end[tl]) en = s_list[tl][k];
                    }
                }
                {
                    const uint32_t k = cur[sub] + ((uint32_t)threadIdx.x & 7u);
                    ahead[sub] = k < s_end[tl] ? s_list[tl][k] : kNoPair;
                }
                // one-byte tokens: the column of the byte, lanes = states
                unsigned long long ones = __builtin_amdgcn_ballot_w64(s_kind[sub * kXT + lane] >= 0);
                while (ones) {
                    const int k = __builtin_ctzll(ones);
                    ones &= ones - 1;
                    if ((k & (kWgWaves - 1)) != wave) continue;        // the wavefronts share them out
                    const uint32_t b1 = (uint32_t)__builtin_amdgcn_readfirstlane(s_kind[sub * kXT + k]);
                    const uint16_t* col = d.tt + (size_t)b1 * q_stride;
#pragma unroll
                    for (int g = 0; g < kXS / 64; ++g) {
                        const uint32_t q = q_base + (uint32_t)(g * 64 + lane);
                        if (q < (uint32_t)d.n_states) {
                            const uint32_t e = col[q];
                            if (e != SINK) tile[(g * 64 + lane) * kXRS + k] = (uint16_t)((e >> 1) + 1u);
                        }
                    }
                }
            }
            __syncthreads();
            if (t0 < n_tokens) {
                // ---- flush the sub-tile's rows and put DEAD back; its allowed bits go to s_bits
                if (WIDE_ROWS) {
                    constexpr int LPR = kXT / 4, RPW = 64 / LPR;     // 16 lanes per row, 4 rows per wavefront pass
                    const int subr = lane / LPR, l = lane % LPR;
                    const int t = t0 + 4 * l;
                    const int lane_off = subr * kXRS + 4 * l;
                    const int base1 = state_base - 1;
                    for (int r0 = wave * RPW; r0 < kXS; r0 += kWgWaves * RPW) {
                        const uint32_t q = q_base + (uint32_t)(r0 + subr);
                        uint32_t* tw = reinterpret_cast<uint32_t*>(tile + r0 * kXRS + lane_off);
                        const uint32_t w0 = tw[0], w1 = tw[1];
                        tw[0] = 0u;
                        tw[1] = 0u;
                        const uint32_t e[4] = {w0 & 0xFFFFu, w0 >> 16, w1 & 0xFFFFu, w1 >> 16};
                        int val[4];
                        uint32_t bits = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            // an entry is the target state + 1, or 0: with no row offset to add, DEAD (-1) needs no test
                            val[j] = BASE0 ? (int)e[j] - 1 : (e[j] ? (int)e[j] + base1 : TDFA_DEAD);
                            bits |= min(e[j], 1u) << j;
                        }
                        if (q < (uint32_t)d.n_states && t < n_tokens) {
                            typedef int i32x4 __attribute__((ext_vector_type(4)));
                            const i32x4 pack4 = {val[0], val[1], val[2], val[3]};
                            __builtin_nontemporal_store(pack4, reinterpret_cast<i32x4*>(delta + ((uint64_t)(out_row32 + q) * nt32 + (uint32_t)t)));
                        }
                        bits <<= 4 * (l & 7);
                        bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
                        bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
                        bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x141, 0xF, 0xF, true);   // row_half_mirror
                        if ((l & 7) == 0) s_bits[(r0 + subr) * 8 + sub * 2 + (l >> 3)] = bits;
                    }
                } else {
                    for (int r = wave; r < kXS; r += kWgWaves) {
                        const uint32_t q = q_base + (uint32_t)r;
                        const int t = t0 + lane;
                        const uint32_t e = tile[r * kXRS + lane];
                        tile[r * kXRS + lane] = (uint16_t)0;
                        const int val = e ? (int)e - 1 + state_base : TDFA_DEAD;
                        if (q < (uint32_t)d.n_states && t < n_tokens) delta[(size_t)(d.out_row + (int)q) * n_tokens + t] = val;
                        const uint64_t m = __builtin_amdgcn_ballot_w64(val >= 0);
                        if (lane < 2) s_bits[r * 8 + sub * 2 + lane] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
                    }
                }
            }
            __syncthreads();
        }
        // ---- the allowed bits of the block's 256 tokens for this tile's rows: two 16-byte halves per row
        {
            const int r = (int)threadIdx.x >> 1, half = (int)threadIdx.x & 1;
            const uint32_t q = q_base + (uint32_t)r;
            const uint32_t word0 = (uint32_t)bt * 8u + (uint32_t)half * 4u;
            uint32_t* src = s_bits + r * 8 + half * 4;
            if (q < (uint32_t)d.n_states && word0 < rw32) {       // a row is a multiple of four words
                uint32_t* dst = allow + ((uint64_t)(out_row32 + q) * rw32 + word0);
                if (allow_vec) {
                    *reinterpret_cast<uint4*>(dst) = make_uint4(src[0], src[1], src[2], src[3]);
                } else {
                    dst[0] = src[0]; dst[1] = src[1]; dst[2] = src[2]; dst[3] = src[3];
                }
            }
            // (sub-tiles past the last token never write their words: they must read as zero for the next tile too)
            src[0] = 0u; src[1] = 0u; src[2] = 0u; src[3] = 0u;
        }
        // the next tile's first flush comes after a barrier, so these reads and clears are done by then
    }
}

}  // namespace

size_t sweep_column_lds_bytes(int32_t q_stride) { return (size_t)q_stride * 2; }

int launch_compile_sweep(const CompileArgs& a, const CompileEntry& e, hipStream_t stream)
{
    if (a.n_tokens <= 0) return TDFA_OK;
    const SweepWorkspace& ws = *e.sweep;
    SweepDesc d;
    d.tt = static_cast<const uint16_t*>(e.trans_t);
    d.n_states = e.n_states;
    d.q_stride = e.q_stride;
    d.n1 = ws.n1;
    d.off1 = ws.off1;
    d.list2 = ws.list2;
    d.cnt2 = ws.cnt2;
    d.need = ws.need;
    d.chunk_sum = ws.chunk_sum;
    d.list1 = ws.list1;
    d.cnt3 = ws.cnt3;
    d.cntF = ws.cntF;
    d.buf_a = ws.buf_a;
    d.buf_b = ws.buf_b;
    d.buf_cap = ws.buf_cap;
    d.err = ws.err;
    d.out_row = e.out_row;
    d.state_base = e.state_base;
    SweepVocab v;
    v.vwords = a.vwords;
    v.voff = a.voff;
    v.vlen = a.vlen;
    v.vprefix = a.vprefix;
    for (int i = 0; i < 2; ++i) {
        v.group_tokens[i] = a.group_tokens[i];
        v.group_chunks[i] = a.group_chunks[i];
        v.n_chunks[i] = a.n_group_chunks[i];
    }
    v.tail_tokens = a.tail_tokens;
    v.n_tail = a.n_tail;
    v.n_tokens = a.n_tokens;

    const bool resume = ws.lists_ready && ws.sized && ws.buffers_sized;    // (see SweepWorkspace::lists_ready)
    ws.lists_ready = false;
    if (!resume) {
        const int rc = launch_transpose(&e, 1, stream);
        if (rc != TDFA_OK) return rc;
    }
    const size_t col_bytes = sweep_column_lds_bytes(e.q_stride);
    static bool attr_set = false;
    if (!attr_set) {
        TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_prefix_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
        TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_token_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
        TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_token_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
        for (auto k : {sweep_expand_kernel<true, true>, sweep_expand_kernel<true, false>, sweep_expand_kernel<false, true>,
                       sweep_expand_kernel<false, false>})
            TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kXLdsBytes));
        attr_set = true;
    }
    if (!resume) {
        sweep_column_count_kernel<<<256, 256, 0, stream>>>(d);
        TDFA_HIP(hipGetLastError());
        sweep_column_scan_kernel<<<1, 256, 0, stream>>>(d);
        TDFA_HIP(hipGetLastError());
        if (!ws.sized) return TDFA_OK;                         // the caller reads off1[256], allocates the lists, and calls again
        TDFA_HIP(hipMemsetAsync(d.err, 0, sizeof(uint32_t), stream));
        sweep_first_kernel<<<256, 256, 0, stream>>>(d);
        TDFA_HIP(hipGetLastError());
        sweep_prefix_kernel<<<dim3(256, 256 / kPrefixPerWg), kWgThreads, col_bytes, stream>>>(d);
        TDFA_HIP(hipGetLastError());
        const int n_scan_chunks = a.n_tokens / 1024 + 1;       // covers entry n_tokens as well
        sweep_need_chunks_kernel<<<(unsigned)n_scan_chunks, 1024, 0, stream>>>(d, v);
        TDFA_HIP(hipGetLastError());
        sweep_need_scan_kernel<<<1, 1024, 0, stream>>>(d, n_scan_chunks);
        TDFA_HIP(hipGetLastError());
        sweep_need_add_kernel<<<(unsigned)n_scan_chunks, 1024, 0, stream>>>(d, a.n_tokens);
        TDFA_HIP(hipGetLastError());
        if (!ws.buffers_sized) return TDFA_OK;                 // the caller reads the total, allocates the buffers, and calls again
    } else {
        // the sizing launch met buffers that were too small and said so; the ones it was followed by hold the total
        TDFA_HIP(hipMemsetAsync(d.err, 0, sizeof(uint32_t), stream));
    }
    if (v.n_chunks[0] > 0) {
        sweep_token_kernel<3><<<(unsigned)v.n_chunks[0], kWgThreads, col_bytes, stream>>>(d, v);
        TDFA_HIP(hipGetLastError());
    }
    if (v.n_chunks[1] > 0) {
        sweep_token_kernel<4><<<(unsigned)v.n_chunks[1], kWgThreads, col_bytes, stream>>>(d, v);
        TDFA_HIP(hipGetLastError());
    }
    if (v.n_tail > 0) {
        sweep_tail_kernel<<<(unsigned)((v.n_tail + 3) / 4), 256, 0, stream>>>(d, v);
        TDFA_HIP(hipGetLastError());
    }
    const int n_tiles_q = (e.n_states + kXS - 1) / kXS;
    const int64_t n_blocks_t = (a.n_tokens + kXBlockT - 1) / kXBlockT;
    // enough workgroups to keep every compute unit supplied: runs of state tiles per block of tokens
    int n_runs = (int)std::min<int64_t>(n_tiles_q, (12288 + n_blocks_t - 1) / n_blocks_t);
    if (n_runs < 1) n_runs = 1;
    const int tiles_per_run = (n_tiles_q + n_runs - 1) / n_runs;
    n_runs = (n_tiles_q + tiles_per_run - 1) / tiles_per_run;
    const int64_t grid = n_blocks_t * n_runs;
    if (grid > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "table too large for one launch");
    const bool wide_rows = a.n_tokens % 4 == 0 && reinterpret_cast<uintptr_t>(a.delta) % 16 == 0;
    const int allow_vec = reinterpret_cast<uintptr_t>(a.allow) % 16 == 0 ? 1 : 0;
    const bool base0 = e.state_base == 0;
    auto kern = wide_rows ? (base0 ? sweep_expand_kernel<true, true> : sweep_expand_kernel<true, false>)
                          : (base0 ? sweep_expand_kernel<false, true> : sweep_expand_kernel<false, false>);
    kern<<<(unsigned)grid, kWgThreads, kXLdsBytes, stream>>>(d, v, (int)n_blocks_t, tiles_per_run, n_tiles_q, a.delta, a.allow,
                                                            a.row_words, allow_vec);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace tdfa
