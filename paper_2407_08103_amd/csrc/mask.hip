// Decode step: loop body of Algorithm 2 after ComputeLogits (allowed set, -inf penalty, greedy
// token choice, edge traversal), batched over sequences, for gfx950.
//
// The allowed set of a state is its row of allowed bits (1 bit per token, written by the compile
// stage), so a step has |V| logits and |V|/8 mask bytes per sequence before it, and one table
// entry for the chosen token.  Nothing here is a contraction: the kernels stream logits with
// 16-byte loads and reduce (value, position) pairs across lanes; `parts` workgroups share a row
// and meet through two device-scope atomics per workgroup.  A logit whose token is not allowed
// cannot matter, so a wavefront whose part of the row allows few tokens reads the mask bytes
// first and then only the groups of eight logits that hold an allowed token (unless the masked
// row is to be written, which takes every logit).
//
// Ordering of candidates (exact path).  Each allowed logit is mapped to an unsigned key that
// preserves the order of the floating-point values, with every NaN mapped to the key of -inf and
// -0 to +0.  Candidates are compared as the 64-bit number (key << 32) | (0xFFFFFFFF - token), so
// the largest value wins and the lowest token id wins ties; 0 means "nothing allowed" (the
// smallest key of an allowed token, that of -inf, is above 0).
//
// bf16 fast path.  Two logits per 32-bit register are turned into 16-bit unsigned keys with
// packed instructions (arithmetic shift, one three-input bit operation), multiplied by their
// allowed bit (0 or 1), and folded with packed max; a lane remembers its best key and the group
// of eight tokens that holds it.  The packed keys do not treat NaN and -0 specially, so a row
// whose winning key is NaN-like, not above -inf, or a zero is handed to the exact path, which the
// last workgroup of the row runs over the whole row.
#include "tdfa_internal.h"

#include <type_traits>

namespace tdfa {
namespace {

constexpr int kMaxThreads = 1024;      // workgroup sizes used: 256 .. 1024
constexpr int kMaxWaves = kMaxThreads / 64;

typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t key_bf16(uint32_t h)
{
    if ((h & 0x7FFFu) > 0x7F80u) h = 0xFF80u;                 // NaN ranks as -inf
    if ((h & 0x7FFFu) == 0) h = 0;                            // -0 equals +0
    return (h & 0x8000u) ? (~h & 0xFFFFu) : (h | 0x8000u);
}

__device__ __forceinline__ uint32_t key_f32(uint32_t u)
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) u = 0xFF800000u;     // NaN ranks as -inf
    if ((u & 0x7FFFFFFFu) == 0) u = 0;                        // -0 equals +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Maximum of a 32-bit value over the 64 lanes of a wavefront (all lanes must be active); the result
// is uniform.  Four cross-lane steps inside each row of 16 lanes (data-parallel primitives, no LDS
// traffic), then the four row results are read as scalars.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));   // row_half_mirror
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));   // row_mirror
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return max(max(r0, r1), max(r2, r3));
}

// 64-bit maximum over a wavefront: the high words first, then the low words of the lanes that hold
// the highest high word.
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    const uint32_t mh = wave_max_u32(hi);
    const uint32_t ml = wave_max_u32(hi == mh ? lo : 0u);
    return ((unsigned long long)mh << 32) | ml;
}

// Maximum over the workgroup; the result is valid in thread 0.  Ends with a barrier-free read, so
// callers that reuse `wave_best` must synchronise first.
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long* wave_best)
{
    v = wave_max_u64(v);
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int n_waves = (int)blockDim.x >> 6;
        for (int w = 1; w < n_waves; ++w) v = wave_best[w] > v ? wave_best[w] : v;
    }
    return v;
}

template <int DTYPE> struct ElemOf { using type = uint32_t; };
template <> struct ElemOf<TDFA_BF16> { using type = uint16_t; };

template <int DTYPE>
__device__ __forceinline__ void load_group(const typename ElemOf<DTYPE>::type* row, int t, int V,
                                           typename ElemOf<DTYPE>::type (&e)[8])
{
    using Elem = typename ElemOf<DTYPE>::type;
    constexpr Elem NEG_INF = DTYPE == TDFA_F32 ? (Elem)0xFF800000u : (Elem)0xFF80u;
    if (t + 8 <= V) {
        if constexpr (DTYPE == TDFA_F32) {
            const uint4 x0 = *reinterpret_cast<const uint4*>(row + t);
            const uint4 x1 = *reinterpret_cast<const uint4*>(row + t + 4);
            e[0] = x0.x; e[1] = x0.y; e[2] = x0.z; e[3] = x0.w;
            e[4] = x1.x; e[5] = x1.y; e[6] = x1.z; e[7] = x1.w;
        } else {
            const uint4 x = *reinterpret_cast<const uint4*>(row + t);
            e[0] = (Elem)(x.x & 0xFFFFu); e[1] = (Elem)(x.x >> 16);
            e[2] = (Elem)(x.y & 0xFFFFu); e[3] = (Elem)(x.y >> 16);
            e[4] = (Elem)(x.z & 0xFFFFu); e[5] = (Elem)(x.z >> 16);
            e[6] = (Elem)(x.w & 0xFFFFu); e[7] = (Elem)(x.w >> 16);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = t + j < V ? row[t + j] : NEG_INF;
    }
}

template <int DTYPE>
__device__ __forceinline__ void store_group(typename ElemOf<DTYPE>::type* orow, int t, int V,
                                            const typename ElemOf<DTYPE>::type (&e)[8])
{
    if (t + 8 <= V) {
        if constexpr (DTYPE == TDFA_F32) {
            *reinterpret_cast<uint4*>(orow + t) = make_uint4(e[0], e[1], e[2], e[3]);
            *reinterpret_cast<uint4*>(orow + t + 4) = make_uint4(e[4], e[5], e[6], e[7]);
        } else {
            *reinterpret_cast<uint4*>(orow + t) =
                make_uint4((uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                           (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16));
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (t + j < V) orow[t + j] = e[j];
    }
}

// Exact scan of groups [g_lo, g_hi) of one row by the whole workgroup: this thread's best
// candidate (key << 32 | ~token), 0 if it saw nothing allowed.  Writes the masked row if orow.
// (bits_at(g): the allowed bits of group g.)
template <int DTYPE, class BitsAt>
__device__ __forceinline__ unsigned long long exact_scan_with(const typename ElemOf<DTYPE>::type* row,
                                                              typename ElemOf<DTYPE>::type* orow, BitsAt bits_at,
                                                              bool valid, int V, int g_lo, int g_hi)
{
    using Elem = typename ElemOf<DTYPE>::type;
    constexpr Elem NEG_INF = DTYPE == TDFA_F32 ? (Elem)0xFF800000u : (Elem)0xFF80u;
    uint32_t best_key = 0, best_idx = 0;
    for (int g = g_lo + (int)threadIdx.x; g < g_hi; g += (int)blockDim.x) {
        const int t = g << 3;
        const uint32_t m = valid ? bits_at(g) : 0u;
        Elem e[8];
        load_group<DTYPE>(row, t, V, e);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = (m >> j) & 1u;
            const uint32_t key = DTYPE == TDFA_F32 ? key_f32((uint32_t)e[j]) : key_bf16((uint32_t)e[j]);
            if (ok && key > best_key) { best_key = key; best_idx = (uint32_t)(t + j); }
            if (!ok) e[j] = NEG_INF;
        }
        if (orow) store_group<DTYPE>(orow, t, V, e);
    }
    return best_key ? ((unsigned long long)best_key << 32) | (0xFFFFFFFFu - best_idx) : 0ull;
}

template <int DTYPE>
__device__ __forceinline__ unsigned long long exact_scan(const typename ElemOf<DTYPE>::type* row,
                                                         typename ElemOf<DTYPE>::type* orow, const uint8_t* bits,
                                                         bool valid, int V, int g_lo, int g_hi)
{
    return exact_scan_with<DTYPE>(row, orow, [bits](int g) { return (uint32_t)bits[g]; }, valid, V, g_lo, g_hi);
}

// Thread 0 of each of the `parts` workgroups of row b brings its candidate; returns true in the
// workgroup that arrives last, with the row's maximum in `cand`.  Both scratch words are zero
// again when it returns true.  All traffic on the two words is device-scope atomics, which
// execute at one place in arrival order; the counter update carries a dependency on the value
// the max returned, so it cannot be issued before the max has been performed.
__device__ __forceinline__ bool combine_parts(const MaskArgs& a, int b, int parts, unsigned long long& cand)
{
    if (parts == 1) return true;
    unsigned int inc = 1u;
    if (cand) {
        const unsigned long long old = __hip_atomic_fetch_max(&a.scratch_best[b], cand, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("" : "+v"(inc) : "v"((uint32_t)old), "v"((uint32_t)(old >> 32)));
    }
    const unsigned done = __hip_atomic_fetch_add(&a.scratch_count[b], inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (done != (unsigned)parts - 1) return false;
    cand = __hip_atomic_exchange(&a.scratch_best[b], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a.scratch_count[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// delta_T[q][token] for a row q and a token id; DEAD if the token has no edge.  A packed table
// keeps only the targets of the edges, in token order: the position of the edge is the number of
// allowed bits of the row below the token (a per-128-token directory plus the bits of one block).
struct PackedBlock {          // what a lookup in a packed row needs, for one block of 128 tokens
    uint32_t w[4];            // the allowed bits of the block
    uint32_t base;            // edges of the row below the block
    int64_t begin;            // first edge of the row
};

__device__ __forceinline__ PackedBlock packed_block(const MaskArgs& a, int q, int blk)
{
    PackedBlock pb;
    const uint32_t* words = a.allow + (int64_t)q * a.row_words + 4 * blk;
    pb.w[0] = words[0]; pb.w[1] = words[1]; pb.w[2] = words[2]; pb.w[3] = words[3];
    pb.base = a.dir[(int64_t)q * (a.row_words >> 2) + blk];
    pb.begin = a.row_begin[q];
    return pb;
}

__device__ __forceinline__ int32_t packed_entry(const MaskArgs& a, const PackedBlock& pb, int token)
{
    const int wi = (token >> 5) & 3, bit = token & 31;
    const uint32_t w = wi == 0 ? pb.w[0] : (wi == 1 ? pb.w[1] : (wi == 2 ? pb.w[2] : pb.w[3]));
    if (!((w >> bit) & 1u)) return TDFA_DEAD;
    const uint32_t below = (wi > 0 ? __popc(pb.w[0]) : 0) + (wi > 1 ? __popc(pb.w[1]) : 0) + (wi > 2 ? __popc(pb.w[2]) : 0) +
                           __popc(w & ((1u << bit) - 1u));
    return a.targets[pb.begin + pb.base + below];
}

__device__ __forceinline__ int32_t table_entry(const MaskArgs& a, int q, int token)
{
    if (a.delta) return a.delta[(int64_t)q * a.n_tokens + token];
    if (!a.targets) return q;                                  // no table: the caller traverses the edge
    return packed_entry(a, packed_block(a, q, token >> 7), token);
}

__device__ __forceinline__ void write_result(const MaskArgs& a, int b, int q, bool valid, unsigned long long cand)
{
    int32_t token = TDFA_NO_TOKEN, next = valid ? q : TDFA_DEAD;
    if (cand) {
        token = (int32_t)(0xFFFFFFFFu - (uint32_t)cand);
        next = table_entry(a, q, token);
    }
    a.tokens[b] = token;
    a.new_states[b] = next;
}

// Exact kernel (fp32 logits).
template <int DTYPE>
__global__ void __launch_bounds__(kMaxThreads)
mask_step_exact_kernel(MaskArgs a, int parts, int groups_per_part)
{
    using Elem = typename ElemOf<DTYPE>::type;
    __shared__ unsigned long long wave_best[kMaxWaves];
    const int b = blockIdx.x / parts, p = blockIdx.x % parts;
    const int V = a.n_tokens;
    const int q = a.states[b];
    const bool valid = q >= 0 && (int64_t)q < a.n_rows;
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid ? (int64_t)q * a.row_words : 0));
    const Elem* row = static_cast<const Elem*>(a.logits) + (int64_t)b * a.row_stride;
    Elem* orow = a.masked_out ? static_cast<Elem*>(a.masked_out) + (int64_t)b * a.row_stride : nullptr;
    const int n_groups = (V + 7) >> 3;
    const int g_lo = p * groups_per_part;
    const int g_hi = min(n_groups, g_lo + groups_per_part);
    unsigned long long cand = exact_scan<DTYPE>(row, orow, bits, valid, V, g_lo, g_hi);
    cand = block_max_u64(cand, wave_best);
    if (threadIdx.x != 0) return;
    if (combine_parts(a, b, parts, cand)) write_result(a, b, q, valid, cand);
}

// 16-bit unsigned order keys of two bf16 values: x ^ 0x8000 for non-negative x, ~x for negative.
__device__ __forceinline__ uint32_t keys2(uint32_t d)
{
    const s16x2 s = __builtin_bit_cast(s16x2, d) >> (s16x2){15, 15};
    return d ^ (__builtin_bit_cast(uint32_t, s) | 0x80008000u);
}

// Buffer descriptors for raw byte-offset access (no structure, 32-bit data format) and the cache
// policy of data that is read once and never again (non-temporal).
constexpr int kRawBuffer = 0x00020000;
constexpr int kReadOnce = 2;
constexpr int kMaxBitRowBytes = 128 * 1024;    // the most allowed bits (a byte per eight tokens) a workgroup keeps in LDS:
                                               // vocabularies of up to about a million tokens
constexpr int kPlainLdsBytes = 40 * 1024;      // what a launch may ask for without the kernel's limit being raised first

constexpr uint32_t KU_POS_INF = 0xFF80u;   // key of +inf: anything above is a NaN pattern
constexpr uint32_t KU_NEG_INF = 0x007Fu;   // key of -inf: anything below is a negative-sign NaN
constexpr uint32_t KU_POS_ZERO = 0x8000u, KU_NEG_ZERO = 0x7FFFu;

// Sum of a 32-bit value over the 64 lanes of a wavefront (all lanes active); the result is uniform.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);     // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);     // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);    // row_half_mirror
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true);    // row_mirror
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// Number of lanes below this one for which `flag` holds (all lanes active).
__device__ __forceinline__ uint32_t lanes_below(bool flag)
{
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(flag);
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Number of non-zero bytes of a word.
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t w)
{
    return (uint32_t)__builtin_popcount((((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u);
}

constexpr int kListCap = 256;          // groups a wavefront may fetch one by one instead of reading its stretch
constexpr int kEarlyWaves = 8;         // wavefronts of a workgroup that request their first group of logits before the state is known

// One step on 16-bit logits.  The groups [g_lo, g_hi) of a workgroup are cut into one stretch of
// `stretch` groups (a multiple of 16) per wavefront, read 64 consecutive groups per load.
//
// SKIP: a wavefront first reads the allowed bits of its whole stretch, 16 bytes (16 groups) per
// lane and pass, into its part of `s_pieces`.  If at most one group in 16 (and at most kListCap)
// holds an allowed token, only those groups' logits are fetched: a decode spends most steps in
// states that allow a few hundred of 10^5 tokens, and the logits of a group without an allowed
// token cannot matter.  Otherwise, and always when the masked row is written, the stretch is
// streamed.  The choice is a wavefront's own; the result does not depend on it.
//
// PDA: the step of a push-down constraint.  The allowed bits of a sequence are not one row but
// the OR of the rows of its state's classes of edges whose pops its stack ends with; the wavefront
// finds those classes (one per lane) before it reads its stretch of bits, and ORs the rows as it
// reads them.  The table lookup at the end is the caller's (the traversal also moves the stack).
template <bool WRITE, int kUnroll, bool SKIP, int kBuf = 2, bool PDA = false>
__global__ void __launch_bounds__(kMaxThreads)
mask_step_bf16_kernel(MaskArgs a, int parts, int groups_per_part, int stretch)
{
    static_assert(!PDA || (SKIP && !WRITE), "the push-down step reads its bits into LDS");
    extern __shared__ uint4 s_pieces[];
    __shared__ uint32_t s_list[SKIP ? kMaxWaves * kListCap : 1];
    __shared__ unsigned long long wave_best[kMaxWaves], wave_best_exact[kMaxWaves];
    __shared__ int s_exact;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int b = blockIdx.x / parts, p = blockIdx.x % parts;
    const int V = a.n_tokens;
    const uint16_t* row = static_cast<const uint16_t*>(a.logits) + (int64_t)b * a.row_stride;
    uint16_t* orow = WRITE ? static_cast<uint16_t*>(a.masked_out) + (int64_t)b * a.row_stride : nullptr;

    const int n_groups = (V + 7) >> 3;
    const int n_full = V >> 3;                                 // groups with all eight tokens inside the row
    const int g_lo = p * groups_per_part;
    const int g_hi = min(n_groups, g_lo + groups_per_part);
    const int g_hi_full = min(g_hi, n_full);
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);    // the same in every lane: kept in a scalar register
    const int w_lo = min(g_lo + wave * stretch, g_hi_full);    // this wavefront's full groups
    const int w_hi = min(w_lo + stretch, g_hi_full);

    // kBuf register buffers of kUnroll groups each: the loads of the next batches are in flight while
    // one is folded.  Logits and allowed bits are read through buffer descriptors that end
    // with the stretch: a group past the end reads as zeros without touching memory, so no load
    // sits under a branch and every lane runs the same number of passes.  Logits are requested
    // before the state is read, since they do not depend on it: every buffer where the wavefront
    // will stream for certain, one group per lane (1 KB per wavefront) where it may turn out to
    // fetch single groups instead, the rest then follows when it knows.  There the allowed bytes
    // of the stretch are in LDS by then, and the stream reads them from there.
    const __amdgpu_buffer_rsrc_t r_logits =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(row), 0, w_hi * 16, kRawBuffer);
    const __amdgpu_buffer_rsrc_t r_out =
        __builtin_amdgcn_make_buffer_rsrc(orow, 0, WRITE ? w_hi * 16 : 0, kRawBuffer);
    auto load_x = [&](int gb, uint4 (&x)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r_logits, (gb + u * 64) * 16, 0, kReadOnce);
            x[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    constexpr int step = 64 * kUnroll;
    int g0 = w_lo + lane;
    uint4 xr[kBuf][kUnroll];
    uint32_t mr[kBuf][kUnroll];
    constexpr bool kMaySkip = SKIP && !WRITE;
    auto load_x1 = [&](int g, uint4& x) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r_logits, g * 16, 0, kReadOnce);
        x = make_uint4(v.x, v.y, v.z, v.w);
    };
    if constexpr (!kMaySkip) {
#pragma unroll
        for (int r = 0; r < kBuf; ++r) load_x(g0 + r * step, xr[r]);
    } else {
        // (the first kEarlyWaves wavefronts of a workgroup only: the early request costs the rows that turn out to
        // allow little or nothing, and half of it serves the rows that stream as well as all of it)
        if (wave < kEarlyWaves) load_x1(g0, xr[0][0]);         // (the rest once the wavefront knows that it streams)
    }
    const int q = a.states[b];
    bool valid = q >= 0 && (int64_t)q < a.n_rows;
    bool surely_wide = false;                         // the state allows so many tokens that the row is streamed whatever the bits say
    if constexpr (!WRITE && !PDA) {
        if (a.row_allowed != nullptr && valid) {
            const uint32_t n_allowed = a.row_allowed[q];
            // A state that allows no token (a sequence whose text is complete): no token, the state stays.
            if (n_allowed == 0u) {
                if (threadIdx.x == 0) {
                    unsigned long long none = 0ull;
                    if (combine_parts(a, b, parts, none)) write_result(a, b, q, valid, none);
                }
                return;
            }
            surely_wide = n_allowed >= (uint32_t)V / 4u;
        }
    }
    unsigned long long classes = 0;                   // PDA: the classes of q (bit j: row class_row0 + j) the stack matches
    int32_t class_row0 = 0;
    if constexpr (PDA) {
        const int32_t depth = a.pda.depths[b];
        valid = q >= 0 && q < a.pda.n_states && depth >= 0 && depth <= a.pda.stack_cap;
        class_row0 = valid ? a.pda.class_first[q] : 0;
        const int n_classes = valid ? a.pda.class_first[q + 1] - class_row0 : 0;
        // the top symbols of the stack and a class's pops are read whole (top first), so that no read
        // waits for the outcome of a comparison
        const int32_t* stack = a.pda.stacks + (int64_t)b * a.pda.stack_cap;
        int32_t top[kPdaPops];
#pragma unroll
        for (int j = 0; j < kPdaPops; ++j) top[j] = valid && depth - 1 - j >= 0 ? stack[depth - 1 - j] : -1;
        bool ok = false;
        if (lane < n_classes) {
            const int np = a.pda.class_n_pops[class_row0 + lane];
            const int4* pp = reinterpret_cast<const int4*>(a.pda.class_pops + (int64_t)(class_row0 + lane) * kPdaPops);
            const int4 p0 = pp[0], p1 = pp[1], p2 = pp[2];
            const int32_t pops[kPdaPops] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w, p2.x, p2.y, p2.z, p2.w};
            ok = np <= depth;
#pragma unroll
            for (int j = 0; j < kPdaPops; ++j)
                if (j < np) ok = ok && pops[j] == top[j];
        }
        classes = __builtin_amdgcn_ballot_w64(ok);
    }
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid && !PDA ? (int64_t)q * a.row_words : 0));
    // the allowed bits of group g, from memory: (PDA: of every matching class)
    auto bits_at = [&](int g) -> uint32_t {
        if constexpr (PDA) {
            uint32_t m = 0;
            for (unsigned long long c = classes; c; c &= c - 1)
                m |= reinterpret_cast<const uint8_t*>(a.allow + (int64_t)(class_row0 + __builtin_ctzll(c)) * a.row_words)[g];
            return m;
        } else {
            return bits[g];
        }
    };
    const __amdgpu_buffer_rsrc_t r_bits =          // one byte per full group; empty for a state outside the table
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(bits), 0, valid ? w_hi : 0, kRawBuffer);
    const uint8_t* my_bits = nullptr;                 // kMaySkip: the stretch's allowed bytes in LDS (set below)
    auto load_m = [&](int gb, uint32_t (&m)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if constexpr (kMaySkip) m[u] = my_bits[gb + u * 64 - w_lo];
            else m[u] = __builtin_amdgcn_raw_buffer_load_b8(r_bits, gb + u * 64, 0, 0);
        }
    };
    if constexpr (!kMaySkip) {
#pragma unroll
        for (int r = 0; r < kBuf; ++r) load_m(g0 + r * step, mr[r]);
    }

    // A lane remembers its best key and the group of eight in which its maximum rose to it (the
    // lowest such group; the maximum rises a few times per row at most), with the group's logits
    // and allowed bits, so that the token inside the group is found from registers when needed.
    uint32_t best = 0, best_g = 0, best_m = 0, any = 0;
    uint4 best_x = make_uint4(0, 0, 0, 0);
    // `ANY_ORDER`: groups may come in any order, so an equal key from a lower group takes over.
    auto fold_one = [&](auto any_order, int g, const uint4& x, uint32_t m) {
        const uint32_t d[4] = {x.x, x.y, x.z, x.w};
        const uint32_t y = m | (m << 15);                      // allowed bit 2j at bit 2j, bit 2j+1 at bit 16+2j
        u16x2 acc = {0, 0};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t pj = (y >> (2 * j)) & 0x00010001u;
            const u16x2 km = __builtin_bit_cast(u16x2, keys2(d[j])) * __builtin_bit_cast(u16x2, pj);
            acc = __builtin_elementwise_max(acc, km);
            if constexpr (WRITE) {
                const uint32_t md = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, pj) * (u16x2){0xFFFF, 0xFFFF});
                o[j] = (d[j] & md) | (0xFF80FF80u & ~md);
            }
        }
        if constexpr (WRITE) {
            // written once, not read again by this step: a streaming store (dropped past the end of the stretch)
            const u32x4 pack = {o[0], o[1], o[2], o[3]};
            __builtin_amdgcn_raw_buffer_store_b128(pack, r_out, g * 16, 0, kReadOnce);
        }
        const uint32_t a2 = __builtin_bit_cast(uint32_t, acc);
        const uint32_t top = max(a2 & 0xFFFFu, a2 >> 16);
        any |= m;
        if (top > best || (decltype(any_order)::value && top == best && (uint32_t)g < best_g)) {
            best = top;
            best_g = (uint32_t)g;
            best_m = m;
            best_x = x;
        }
    };
    auto fold = [&](int gb, const uint4 (&x)[kUnroll], const uint32_t (&m)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) fold_one(std::false_type{}, gb + u * 64, x[u], m[u]);
    };
    // The lane's candidate, exactly: (has an allowed token, key, lowest token id first).
    auto candidate = [&]() -> unsigned long long {
        const uint32_t d[4] = {best_x.x, best_x.y, best_x.z, best_x.w};
        int j = 7;
#pragma unroll
        for (int pr = 3; pr >= 0; --pr) {
            const uint32_t k2 = keys2(d[pr]);
            if ((best_m >> (2 * pr + 1) & 1u) && (k2 >> 16) == best) j = 2 * pr + 1;
            if ((best_m >> (2 * pr) & 1u) && (k2 & 0xFFFFu) == best) j = 2 * pr;
        }
        const uint32_t tok = best_g * 8 + (uint32_t)j;
        return any ? (1ull << 63) | ((unsigned long long)best << 32) | (0xFFFFFFFFu - tok) : 0ull;
    };

    // Which way this wavefront goes: count the groups of the stretch that hold an allowed token.
    bool skip = false;
    uint32_t n_listed = 0;
    constexpr int kPad16 = 4 * step / 16;                          // zero bytes behind a stretch: the four batches read past its end
    uint4* my_pieces = s_pieces + wave * ((stretch >> 4) + kPad16);
    const int n_pieces = (w_hi - w_lo + 15) >> 4;              // (w_lo is a multiple of 16 unless the stretch is empty)
    my_bits = reinterpret_cast<const uint8_t*>(my_pieces);
    if constexpr (SKIP && !WRITE) {
        const __amdgpu_buffer_rsrc_t r_row =       // the whole bit row, a multiple of 16 bytes
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(bits), 0, valid ? a.row_words * 4 : 0, kRawBuffer);
        uint32_t nz = 0;
        // A state known to allow a quarter of the vocabulary or more is streamed: the rest of the buffers is
        // requested right behind the first bits, without waiting for them to be counted.
        u32x4 v_first = {0, 0, 0, 0};
        if constexpr (!PDA) {
            v_first = __builtin_amdgcn_raw_buffer_load_b128(r_row, w_lo + lane * 16, 0, 0);
            if (surely_wide) {
                if (wave >= kEarlyWaves) load_x1(g0, xr[0][0]);
#pragma unroll
                for (int u = 1; u < kUnroll; ++u) load_x1(g0 + u * 64, xr[0][u]);
#pragma unroll
                for (int r = 1; r < kBuf; ++r) load_x(g0 + r * step, xr[r]);
            }
        }
        for (int i = lane; i < n_pieces; i += 64) {
            u32x4 v = {0, 0, 0, 0};
            if constexpr (PDA) {
                for (unsigned long long c = classes; c; c &= c - 1) {       // (the same classes in every lane)
                    const uint32_t* class_row = a.allow + (int64_t)(class_row0 + __builtin_ctzll(c)) * a.row_words;
                    v |= __builtin_amdgcn_raw_buffer_load_b128(
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(class_row), 0, a.row_words * 4, kRawBuffer),
                        w_lo + i * 16, 0, 0);
                }
            } else {
                v = i == lane ? v_first : __builtin_amdgcn_raw_buffer_load_b128(r_row, w_lo + i * 16, 0, 0);
            }
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int left = w_hi - (w_lo + i * 16 + d * 4);       // bytes of this word inside the stretch
                if (left <= 0) w[d] = 0;
                else if (left < 4) w[d] &= (1u << (8 * left)) - 1u;
                nz += nonzero_bytes(w[d]);
            }
            my_pieces[i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
        for (int i = n_pieces + lane; i < (stretch >> 4) + kPad16; i += 64) my_pieces[i] = make_uint4(0, 0, 0, 0);
        n_listed = wave_sum_u32(nz);
        skip = !surely_wide && n_listed <= (uint32_t)kListCap && n_listed * 16u <= (uint32_t)(w_hi - w_lo);
        if (skip) {
            // Every lane lists the groups of its pieces: (group within the stretch) << 8 | bits.
            uint32_t slot = 0;
#pragma unroll
            for (int bit = 0; bit < 9; ++bit) slot += lanes_below((nz >> bit) & 1u) << bit;   // lanes' counts below this one's
            uint32_t* list = s_list + wave * kListCap;
            for (int i = lane; i < n_pieces; i += 64) {
                const uint4 pc = my_pieces[i];
                const uint32_t w[4] = {pc.x, pc.y, pc.z, pc.w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t rest = w[d];
                    while (rest) {
                        const int byte = (__builtin_ctz(rest)) >> 3;
                        list[slot++] = (uint32_t)((i * 16 + d * 4 + byte) << 8) | ((rest >> (8 * byte)) & 0xFFu);
                        rest &= ~(0xFFu << (8 * byte));
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // One listed group per lane, four loads in flight; a lane without one reads past the end.
            for (uint32_t r0 = 0; r0 < n_listed; r0 += 256) {
                uint4 x[4];
                uint32_t m[4];
                int g[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t idx = r0 + (uint32_t)(u * 64 + lane);
                    const uint32_t e = idx < n_listed ? list[idx] : 0u;
                    g[u] = w_lo + (int)(e >> 8);
                    m[u] = e & 0xFFu;
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r_logits, idx < n_listed ? g[u] * 16 : 0x7FFFFFF0, 0, kReadOnce);
                    x[u] = make_uint4(v.x, v.y, v.z, v.w);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) fold_one(std::true_type{}, g[u], x[u], m[u]);
            }
        }
    }

    // The traversal of the chosen edge (Algorithm 2, last statement) is one dependent read of the
    // table at the very end of the step.  It is taken off the critical path: after about three
    // quarters of a stretch, the wavefront requests the table entry of its best token so far; the
    // token that wins in the end has most often been seen by then, and its entry has long arrived
    // when the workgroup's maximum is known.
    const bool ahead = parts == 1 && a.delta != nullptr && a.n_rows > 0;       // (packed tables and split rows look the entry up at the end)
    uint32_t tok_ahead = 0xFFFFFFFFu;                                          // an id no token has
    int32_t val_ahead = TDFA_DEAD;
    if (!skip) {
        if constexpr (kMaySkip) {
            if (!surely_wide) {
                if (wave >= kEarlyWaves) load_x1(g0, xr[0][0]);
#pragma unroll
                for (int u = 1; u < kUnroll; ++u) load_x1(g0 + u * 64, xr[0][u]);
#pragma unroll
                for (int r = 1; r < kBuf; ++r) load_x(g0 + r * step, xr[r]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int r = 0; r < kBuf; ++r) load_m(g0 + r * step, mr[r]);
        }
        int base = w_lo;
        auto stream_until = [&](int limit) {           // every buffer is loaded on entry
            for (; base < limit; base += kBuf * step, g0 += kBuf * step) {
#pragma unroll
                for (int r = 0; r < kBuf; ++r) {
                    fold(g0 + r * step, xr[r], mr[r]);
                    load_x(g0 + (kBuf + r) * step, xr[r]);
                    load_m(g0 + (kBuf + r) * step, mr[r]);
                }
            }
        };
        const int span = w_hi - w_lo;
        stream_until(w_lo + span - span / 4);
        if (ahead) {
            const unsigned long long w = wave_max_u64(candidate());
            tok_ahead = 0xFFFFFFFFu - (uint32_t)w;
            // w != 0: a token is allowed, so q is a row of the table; otherwise its first entry is read and not used
            const int64_t row_first = w != 0 ? (int64_t)q * V : 0;
            uint32_t col = w != 0 ? tok_ahead : 0u;
            asm volatile("" : "+v"(col));                  // a vector load: the LDS reads of the loop do not wait for it
            val_ahead = a.delta[row_first + col];
        }
        stream_until(w_hi);
    }
    if (g_hi > g_hi_full && threadIdx.x == 0) {
        // the row's last, partial group: element loads, same 16-bit keys
        const int g = n_full, t = g << 3;
        const uint32_t m = (valid ? bits_at(g) : 0u) & ((1u << (V - t)) - 1u);
        uint32_t d[4] = {0, 0, 0, 0}, top = 0;
        for (int j = 0; j < V - t; ++j) {
            const uint32_t h = row[t + j];
            const bool ok = (m >> j) & 1u;
            d[j >> 1] |= h << (16 * (j & 1));
            if (ok) top = max(top, (h & 0x8000u) ? (~h & 0xFFFFu) : (h ^ 0x8000u));
            if (WRITE) orow[t + j] = ok ? (uint16_t)h : (uint16_t)0xFF80u;
        }
        any |= m;
        if (top > best) {
            best = top;
            best_g = (uint32_t)g;
            best_m = m;
            best_x = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
    // The wavefront that holds the workgroup's maximum finishes the row (the first one if nothing
    // is allowed): each reads the wavefronts' candidates one per lane and folds them across lanes.
    const unsigned long long wmax = wave_max_u64(candidate());         // the wavefront's final candidate
    if (lane == 0) wave_best[wave] = wmax;
    __syncthreads();
    unsigned long long cand = wave_max_u64(lane < ((int)blockDim.x >> 6) ? wave_best[lane] : 0ull);
    const bool finisher = lane == 0 && (cand == 0 ? threadIdx.x == 0 : wmax == cand);
    if (finisher) {
        int exact = 0;
        if (combine_parts(a, b, parts, cand)) {
            const uint32_t ku = (uint32_t)(cand >> 32) & 0xFFFFu;
            if (cand == 0) {
                write_result(a, b, q, valid, 0ull);
            } else if (ku > KU_POS_INF || ku <= KU_NEG_INF || ku == KU_POS_ZERO || ku == KU_NEG_ZERO) {
                exact = 1;
            } else {
                const uint32_t token = 0xFFFFFFFFu - (uint32_t)cand;
                int32_t next;
                if (ahead && token == tok_ahead) next = val_ahead;
                else next = table_entry(a, q, (int)token);
                a.tokens[b] = (int32_t)token;
                a.new_states[b] = next;
            }
        }
        s_exact = exact;
    }
    __syncthreads();
    if (!s_exact) return;
    // Rare: NaN, zeros or nothing above -inf at the top of the row.  The masked row is already
    // written, so this pass only chooses the token.
    unsigned long long c = exact_scan_with<TDFA_BF16>(row, nullptr, bits_at, valid, V, 0, n_groups);
    c = block_max_u64(c, wave_best_exact);
    if (threadIdx.x == 0) write_result(a, b, q, valid, c);
}

// One step on fp32 logits.  Like the 16-bit kernel, every wavefront first reads the allowed bytes of
// its stretch and lists the groups that hold an allowed token; if all wavefronts of the workgroup
// find at most one such group in 16, they fetch just those groups (32 bytes each) and compare their
// allowed logits exactly.  Otherwise the workgroup scans its part of the row as the exact kernel
// does.  Candidates are (key, lowest token) as everywhere, so the order of the groups does not matter.
__global__ void __launch_bounds__(kMaxThreads)
mask_step_f32_kernel(MaskArgs a, int parts, int groups_per_part, int stretch)
{
    extern __shared__ uint4 s_pieces[];
    __shared__ uint32_t s_list[kMaxWaves * kListCap];
    __shared__ unsigned long long wave_best[kMaxWaves];
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int b = blockIdx.x / parts, p = blockIdx.x % parts;
    const int V = a.n_tokens;
    const int q = a.states[b];
    const bool valid = q >= 0 && (int64_t)q < a.n_rows;
    if (a.row_allowed != nullptr && valid && a.row_allowed[q] == 0u) {          // nothing allowed: no token, the state stays
        if (threadIdx.x == 0) {
            unsigned long long none = 0ull;
            if (combine_parts(a, b, parts, none)) write_result(a, b, q, valid, none);
        }
        return;
    }
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid ? (int64_t)q * a.row_words : 0));
    const uint32_t* row = static_cast<const uint32_t*>(a.logits) + (int64_t)b * a.row_stride;
    const int n_groups = (V + 7) >> 3;
    const int n_full = V >> 3;
    const int g_lo = p * groups_per_part;
    const int g_hi = min(n_groups, g_lo + groups_per_part);
    const int g_hi_full = min(g_hi, n_full);
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int w_lo = min(g_lo + wave * stretch, g_hi_full);
    const int w_hi = min(w_lo + stretch, g_hi_full);

    // the allowed bytes of the stretch, 16 per lane and pass, and how many of them are not zero
    uint4* my_pieces = s_pieces + wave * (stretch >> 4);
    const int n_pieces = (w_hi - w_lo + 15) >> 4;
    const __amdgpu_buffer_rsrc_t r_row =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(bits), 0, valid ? a.row_words * 4 : 0, kRawBuffer);
    uint32_t nz = 0;
    for (int i = lane; i < n_pieces; i += 64) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r_row, w_lo + i * 16, 0, 0);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int left = w_hi - (w_lo + i * 16 + d * 4);
            if (left <= 0) w[d] = 0;
            else if (left < 4) w[d] &= (1u << (8 * left)) - 1u;
            nz += nonzero_bytes(w[d]);
        }
        my_pieces[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    const uint32_t n_listed = wave_sum_u32(nz);
    const bool few = n_listed <= (uint32_t)kListCap && n_listed * 16u <= (uint32_t)(w_hi - w_lo);
    unsigned long long best = 0;
    if (__syncthreads_and(few)) {
        uint32_t slot = 0;
#pragma unroll
        for (int bit = 0; bit < 9; ++bit) slot += lanes_below((nz >> bit) & 1u) << bit;
        uint32_t* list = s_list + wave * kListCap;
        for (int i = lane; i < n_pieces; i += 64) {
            const uint4 pc = my_pieces[i];
            const uint32_t w[4] = {pc.x, pc.y, pc.z, pc.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t rest = w[d];
                while (rest) {
                    const int byte = (__builtin_ctz(rest)) >> 3;
                    list[slot++] = (uint32_t)((i * 16 + d * 4 + byte) << 8) | ((rest >> (8 * byte)) & 0xFFu);
                    rest &= ~(0xFFu << (8 * byte));
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const __amdgpu_buffer_rsrc_t r_logits =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(row), 0, w_hi * 32, kRawBuffer);
        // one listed group per lane, two at a time
        for (uint32_t r0 = 0; r0 < n_listed; r0 += 128) {
            u32x4 lo[2], hi[2];
            uint32_t m[2];
            int g[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t idx = r0 + (uint32_t)(u * 64 + lane);
                const uint32_t e = idx < n_listed ? list[idx] : 0u;
                g[u] = w_lo + (int)(e >> 8);
                m[u] = e & 0xFFu;
                lo[u] = __builtin_amdgcn_raw_buffer_load_b128(r_logits, idx < n_listed ? g[u] * 32 : 0x7FFFFFF0, 0, kReadOnce);
                hi[u] = __builtin_amdgcn_raw_buffer_load_b128(r_logits, idx < n_listed ? g[u] * 32 + 16 : 0x7FFFFFF0, 0, kReadOnce);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t e8[8] = {lo[u].x, lo[u].y, lo[u].z, lo[u].w, hi[u].x, hi[u].y, hi[u].z, hi[u].w};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const unsigned long long c = ((unsigned long long)key_f32(e8[j]) << 32) | (0xFFFFFFFFu - (uint32_t)(g[u] * 8 + j));
                    if (((m[u] >> j) & 1u) && c > best) best = c;
                }
            }
        }
        if (g_hi > g_hi_full && threadIdx.x == 0 && valid) {
            // the row's last, partial group
            const int t = n_full << 3;
            const uint32_t m = bits[n_full];
            for (int j = 0; j < V - t; ++j) {
                const unsigned long long c = ((unsigned long long)key_f32(row[t + j]) << 32) | (0xFFFFFFFFu - (uint32_t)(t + j));
                if (((m >> j) & 1u) && c > best) best = c;
            }
        }
    } else {
        best = exact_scan<TDFA_F32>(row, nullptr, bits, valid, V, g_lo, g_hi);
    }
    best = block_max_u64(best, wave_best);
    if (threadIdx.x != 0) return;
    if (combine_parts(a, b, parts, best)) write_result(a, b, q, valid, best);
}

// ---------------------------------------------------------------------------------------------
// Sampling step: SampleNextToken of Algorithm 2 as a draw from softmax(l / T) over the allowed
// set, by the Gumbel-max rule: the allowed token with the largest fma(l_t, 1/T, g_t) wins, g_t
// standard Gumbel noise made from one word of Philox4x32-10 (Salmon et al. 2011) per token.  The
// chosen token is an integer decided by floating point, so the noise is defined operation by
// operation in IEEE-754 binary32 (see the declaration of tdfa_sample_step); nothing below may be
// contracted, reassociated or replaced by an approximate instruction.
// ---------------------------------------------------------------------------------------------
#pragma clang fp contract(off)

struct SampleParams {
    float inv_t;
    uint32_t seed_lo, seed_hi, off_lo, off_hi;
    const unsigned long long* off_dev;   // if not NULL: the offset is read from here by the kernel (off_lo / off_hi unused)
    const uint32_t* cut;      // top-k: per sequence, the order key of the smallest logit still drawn from; or NULL
};

// counter (c0, c1, c2, c3), key (k0, k1) -> four words, ten rounds
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&w)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const unsigned long long p0 = (unsigned long long)0xD2511F53u * c0;
        const unsigned long long p1 = (unsigned long long)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// Natural logarithm of a positive normal number: x = 2^e m, m in (sqrt(1/2), sqrt(2)],
// ln m = 2 atanh(s) with s = (m - 1) / (m + 1), five terms of the series by Horner's rule.
__device__ __forceinline__ float ln32(float x)
{
    const uint32_t i = __float_as_uint(x);
    int e = (int)(i >> 23) - 127;
    const uint32_t frac = i & 0x7FFFFFu;
    float m = __uint_as_float(frac | 0x3F800000u);
    if (frac > 0x3504F3u) {                                  // above sqrt(2): halve (exact)
        m = m * 0.5f;
        e += 1;
    }
    const float f = m - 1.0f;                                 // exact
    const float s = __fdiv_rn(f, 2.0f + f);
    const float z = s * s;
    float p = __builtin_fmaf(z, 2.0f / 9.0f, 2.0f / 7.0f);
    p = __builtin_fmaf(z, p, 2.0f / 5.0f);
    p = __builtin_fmaf(z, p, 2.0f / 3.0f);
    p = __builtin_fmaf(z, p, 2.0f);
    return __builtin_fmaf((float)e, 0.693147180559945309f, s * p);
}

// Standard Gumbel variate from one generator word: u = ((x >> 9) + 1/2) 2^-23, g = -ln(-ln u).
__device__ __forceinline__ float gumbel_of(uint32_t x)
{
    const float u = __builtin_fmaf((float)(x >> 9), 0x1p-23f, 0x1p-24f);
    return -ln32(-ln32(u));
}

// The noise alone: out[b][t] = g_t of sequence b, for callers that want to reproduce a draw.
__global__ void __launch_bounds__(256)
sample_noise_kernel(SampleParams sp, int32_t n_tokens, int64_t n_quads_total, int32_t quads_per_row, float* __restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_quads_total) return;
    const int32_t b = (int32_t)(i / quads_per_row), k = (int32_t)(i % quads_per_row);
    uint32_t w[4];
    philox4x32_10((uint32_t)k, (uint32_t)b, sp.off_lo, sp.off_hi, sp.seed_lo, sp.seed_hi, w);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (4 * k + j < n_tokens) out[(int64_t)b * n_tokens + 4 * k + j] = gumbel_of(w[j]);
}

// Top-k: the order key of the k-th largest allowed logit of each sequence (0 if the state allows
// fewer than k tokens: nothing is cut).  One workgroup per sequence.
//
// The selection itself is a radix selection over 32-bit order keys, most significant digit first
// (11 + 11 + 10 bits): a pass counts, in an LDS histogram, the keys whose higher digits equal those
// already fixed, and the digit is the bin in which the count from the top reaches what is still
// wanted.  Run over a whole wildcard-like row that would send a hundred thousand atomic adds
// through one LDS, so the row is thinned out first:
//   1. every thread takes the largest key among a few groups of the row, an eighth of a large
//      vocabulary in all (no atomics);
//   2. the k-th largest of these thread maxima, L, is selected in LDS: at least k allowed logits
//      reach L, so the k-th largest of the row does too;
//   3. a second pass over the row collects the keys that reach L (about k of them) in LDS, and the
//      k-th largest of the collected keys is selected there.
// If k exceeds the number of threads, or the collected keys do not fit (masses of equal logits),
// the selection runs over the row itself, restricted to the keys that reach L.
constexpr int kCutBins = 2048;
constexpr int kCutKeep = 2048;         // collected keys that fit in LDS

template <int DTYPE>
__global__ void __launch_bounds__(kMaxThreads)
topk_cut_kernel(MaskArgs a, int32_t top_k, uint32_t* __restrict__ cut)
{
    using Elem = typename ElemOf<DTYPE>::type;
    __shared__ uint32_t hist[kCutBins];
    __shared__ uint32_t s_scan[kMaxWaves];
    __shared__ __attribute__((aligned(16))) uint32_t s_keys[kCutKeep];
    __shared__ uint32_t s_bin, s_want, s_found, s_n;
    const int b = blockIdx.x;
    const int V = a.n_tokens;
    const int q = a.states[b];
    const bool valid = q >= 0 && (int64_t)q < a.n_rows;
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid ? (int64_t)q * a.row_words : 0));
    const Elem* row = static_cast<const Elem*>(a.logits) + (int64_t)b * a.row_stride;
    const int n_groups = (V + 7) >> 3;
    const int T = (int)blockDim.x, per = kCutBins / T;          // T is 256 or 1024

    // f(key) for every allowed logit of the row (NaN ranks as -inf).  Eight groups per thread are in
    // flight: their allowed bits first, then the logits of those that have an allowed token.
    auto for_groups = [&](int g_begin, int g_end, auto&& f) {
        constexpr int kU = 8;
        for (int base = g_begin; base < g_end; base += T * kU) {
            uint32_t m[kU];
            Elem e[kU][8];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int g = base + u * T + (int)threadIdx.x;
                m[u] = (valid && g < g_end) ? bits[g] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u)
                if (m[u]) load_group<DTYPE>(row, (base + u * T + (int)threadIdx.x) << 3, V, e[u]);
#pragma unroll
            for (int u = 0; u < kU; ++u) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t x = (uint32_t)e[u][j];
                    if ((m[u] >> j) & 1u) f(key_f32(DTYPE == TDFA_F32 ? x : x << 16));
                }
            }
        }
    };
    auto for_row = [&](auto&& f) { for_groups(0, n_groups, f); };
    // f(key) for the first n keys held in s_keys, zeros skipped
    auto for_kept = [&](uint32_t n, auto&& f) {
        for (uint32_t i = threadIdx.x; i < n; i += (uint32_t)T) {
            const uint32_t key = s_keys[i];
            if (key) f(key);
        }
    };
    // The want-th largest of the keys >= floor that `each` enumerates; false if there are fewer.
    // Called by all threads; ends with a barrier.
    auto select = [&](auto&& each, uint32_t want, uint32_t floor_key, uint32_t* result) -> bool {
        constexpr int kShift[3] = {21, 10, 0};
        constexpr int kWidth[3] = {11, 11, 10};
        uint32_t prefix = 0, fixed_mask = 0;
        for (int pass = 0; pass < 3; ++pass) {
            for (int i = threadIdx.x; i < kCutBins; i += T) hist[i] = 0;
            if (threadIdx.x == 0) s_found = 0;
            __syncthreads();
            const int shift = kShift[pass];
            const uint32_t digit_mask = (1u << kWidth[pass]) - 1u;
            each([&](uint32_t key) {
                if (key >= floor_key && (key & fixed_mask) == prefix) atomicAdd(&hist[(key >> shift) & digit_mask], 1u);
            });
            __syncthreads();
            // thread i owns bins [i * per, (i + 1) * per); `above` = count in the bins of the threads above
            // i: a suffix scan inside each wavefront by shuffles, then the totals of the wavefronts above
            uint32_t mine = 0;
            for (int i = 0; i < per; ++i) mine += hist[threadIdx.x * per + i];
            uint32_t incl = mine;
            const int ln = (int)(threadIdx.x & 63u);
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t other = __shfl_down(incl, d, 64);
                if (ln + d < 64) incl += other;
            }
            if (ln == 0) s_scan[threadIdx.x >> 6] = incl;       // total of this wavefront
            __syncthreads();
            uint32_t higher = 0;
            for (int w = (int)(threadIdx.x >> 6) + 1; w < (T >> 6); ++w) higher += s_scan[w];
            uint32_t above = higher + incl - mine;
            for (int i = per - 1; i >= 0; --i) {
                const uint32_t c = hist[threadIdx.x * per + i];
                if (above < want && want <= above + c) {          // true in exactly one bin, if there are enough keys
                    s_bin = (uint32_t)(threadIdx.x * per + i);
                    s_want = want - above;
                    s_found = 1;
                }
                above += c;
            }
            __syncthreads();
            const bool found = s_found != 0;
            const uint32_t bin = s_bin, next_want = s_want;
            __syncthreads();
            if (!found) return false;
            prefix |= bin << shift;
            fixed_mask |= digit_mask << shift;
            want = next_want;
        }
        *result = prefix;
        return true;
    };

    // The want-th largest of the first n <= 512 keys in s_keys, by counting: a key is the answer if
    // fewer than `want` keys are greater and at least `want` are greater or equal.
    auto select_few = [&](uint32_t n, uint32_t want, uint32_t* result) -> bool {
        if (threadIdx.x == 0) s_found = 0;
        for (uint32_t i = n + threadIdx.x; i < ((n + 3u) & ~3u); i += (uint32_t)T) s_keys[i] = 0;   // pad to whole uint4
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < n; i += (uint32_t)T) {
            const uint32_t mine = s_keys[i];
            uint32_t gt = 0, ge = 0;
            for (uint32_t j = 0; j < n; j += 4) {
                const uint4 o = *reinterpret_cast<const uint4*>(&s_keys[j]);
                gt += (o.x > mine) + (o.y > mine) + (o.z > mine) + (o.w > mine);
                ge += (o.x >= mine) + (o.y >= mine) + (o.z >= mine) + (o.w >= mine);
            }
            if (mine != 0 && gt < want && want <= ge) {        // equal keys all write the same value
                s_bin = mine;
                s_found = 1;
            }
        }
        __syncthreads();
        const bool found = s_found != 0;
        *result = s_bin;
        __syncthreads();
        return found;
    };

    const uint32_t k = (uint32_t)top_k;
    // how many tokens the state allows: the bit row alone tells
    uint32_t n_allowed = 0;
    {
        const uint32_t* words = reinterpret_cast<const uint32_t*>(bits);
        const int n_words = (V + 31) >> 5;
        uint32_t c = 0;
        for (int i = threadIdx.x; valid && i < n_words; i += T) c += __popc(words[i]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
        if ((threadIdx.x & 63u) == 0) s_scan[threadIdx.x >> 6] = c;
        __syncthreads();
        for (int w = 0; w < (T >> 6); ++w) n_allowed += s_scan[w];
        __syncthreads();
    }
    uint32_t floor_key = 0, result = 0;
    bool found = false;
    if (n_allowed >= k) {                                         // else nothing is cut, and no logit is read
        if (n_allowed > (uint32_t)kCutKeep && k <= (uint32_t)T) {
            // a part of the row is enough for a bound: two stretches of T groups, at the start and in the middle
            uint32_t top = 0;
            auto take_max = [&](uint32_t key) { top = max(top, key); };
            if (n_groups <= 4 * T) {
                for_row(take_max);
            } else {
                for_groups(0, T, take_max);
                for_groups(n_groups / 2, n_groups / 2 + T, take_max);
            }
            s_keys[threadIdx.x] = top;                            // 0: this thread saw no allowed token
            __syncthreads();
            if (!select([&](auto&& f) { for_kept((uint32_t)T, f); }, k, 0u, &floor_key)) floor_key = 0;
        }
        if (threadIdx.x == 0) s_n = 0;
        __syncthreads();
        for_row([&](uint32_t key) {
            if (key >= floor_key) {
                const uint32_t i = atomicAdd(&s_n, 1u);
                if (i < (uint32_t)kCutKeep) s_keys[i] = key;
            }
        });
        __syncthreads();
        const uint32_t n = s_n;
        if (n <= 512u)
            found = select_few(n, k, &result);
        else if (n <= (uint32_t)kCutKeep)
            found = select([&](auto&& f) { for_kept(n, f); }, k, 0u, &result);
        else
            found = select(for_row, k, floor_key, &result);
    }
    if (threadIdx.x == 0) cut[b] = found ? result : 0u;
}

constexpr int kQueue = 128;            // entries of a wavefront's queues (rings, a power of two)
constexpr float kNoiseMax = 16.64f;    // above every noise value: -ln(-ln(1 - 2^-24)) = 16.6355...
constexpr int kWordsAhead = 4;         // 32-bit words of allowed bits (four groups each) a thread has in flight

// One workgroup scans groups [g_lo, g_hi) of a row.  Only allowed tokens cost arithmetic (a
// generator block, two logarithms), and in the automata of constrained decoding most states
// allow few tokens, scattered over the row.  Two queues per wavefront, in LDS, keep the lanes
// busy all the same:
//   groups : the groups of eight tokens with an allowed token among them.  A thread reads the
//            allowed bits of 4 * kWordsAhead groups at once; the groups that need their logits are
//            queued and fetched 64 at a time, one per lane, so the logits of groups without an
//            allowed token are never read (unless the masked row is wanted: then all are queued).
//   tokens : the allowed tokens (id, logit) of the fetched groups, scored 64 at a time, one per
//            lane.  Where most lanes hold groups that are at least half allowed (a wildcard-like
//            state) the lanes score their own eight tokens in place instead, which shares a
//            generator block among four neighbouring tokens.
// A queue belongs to one wavefront, so the loop needs no workgroup barrier; the maximum does not
// depend on the order of scoring because candidates are compared as (score, lowest id).
//
// With SAMPLE off the same scan is the greedy step for packed tables, whose states mostly allow
// few tokens: the score of a token is its logit, fetched groups are compared in place (no token
// queue), and a state that allows at least an eighth of the vocabulary (its edge count is in the
// packed table) is scanned by the streaming loop instead, which reads every logit.
template <int DTYPE, bool WRITE, bool SAMPLE>
__global__ void __launch_bounds__(kMaxThreads)
gather_step_kernel(MaskArgs a, SampleParams sp, int parts, int groups_per_part)
{
    using Elem = typename ElemOf<DTYPE>::type;
    constexpr Elem NEG_INF = DTYPE == TDFA_F32 ? (Elem)0xFF800000u : (Elem)0xFF80u;
    __shared__ unsigned long long wave_best[kMaxWaves];
    __shared__ uint2 s_groups[kMaxWaves][kQueue];
    __shared__ uint2 s_tokens[kMaxWaves][kQueue];
    __shared__ uint32_t s_reached;                             // order key of the best score any wavefront has reached
    if (SAMPLE) {
        if (threadIdx.x == 0) s_reached = 0;
        __syncthreads();
    }
    const int b = blockIdx.x / parts, p = blockIdx.x % parts;
    const int V = a.n_tokens;
    const int q = a.states[b];
    const bool valid = q >= 0 && (int64_t)q < a.n_rows;
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid ? (int64_t)q * a.row_words : 0));
    const Elem* row = static_cast<const Elem*>(a.logits) + (int64_t)b * a.row_stride;
    Elem* orow = WRITE ? static_cast<Elem*>(a.masked_out) + (int64_t)b * a.row_stride : nullptr;
    const int n_groups = (V + 7) >> 3;
    const int g_lo = p * groups_per_part;
    const int g_hi = min(n_groups, g_lo + groups_per_part);
    const uint32_t lane = threadIdx.x & 63u;
    uint2* group_q = s_groups[threadIdx.x >> 6];
    uint2* token_q = s_tokens[threadIdx.x >> 6];
    auto below = [](unsigned long long bal) {                  // lanes below this one that are set in bal
        return __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
    };
    auto wave_sync = []() {                                    // LDS written by some lanes, read by others
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    if constexpr (!WRITE) {
        // A state that allows no token (its count, or in a packed table its edges): no token, the state stays.
        const bool none = valid && (a.delta ? (a.row_allowed != nullptr && a.row_allowed[q] == 0u)
                                            : (a.targets != nullptr && a.row_begin[q + 1] == a.row_begin[q]));
        if (none) {                                                                           // uniform in the workgroup
            if (threadIdx.x == 0) {
                unsigned long long nothing = 0ull;
                if (combine_parts(a, b, parts, nothing)) write_result(a, b, q, valid, nothing);
            }
            return;
        }
    }
    if constexpr (!SAMPLE) {
        if (valid && !a.delta && (a.row_begin[q + 1] - a.row_begin[q]) * 8 >= (int64_t)V) {   // uniform in the workgroup
            unsigned long long c = exact_scan<DTYPE>(row, orow, bits, valid, V, g_lo, g_hi);
            c = block_max_u64(c, wave_best);
            if (threadIdx.x == 0 && combine_parts(a, b, parts, c)) write_result(a, b, q, valid, c);
            return;
        }
    }

    const uint32_t cut_key = (SAMPLE && sp.cut) ? sp.cut[b] : 0u;
    if (SAMPLE && sp.off_dev) {                                // the same word for every thread
        const unsigned long long o = *sp.off_dev;
        sp.off_lo = (uint32_t)o;
        sp.off_hi = (uint32_t)(o >> 32);
    }
    uint32_t best_key = 0, best_idx = 0xFFFFFFFFu;           // key 0: no candidate yet
    auto consider = [&](uint32_t tok, uint32_t lb, uint32_t word) {
        if ((lb & 0x7FFFFFFFu) > 0x7F800000u) lb = 0xFF800000u;             // NaN counts as -inf
        if (SAMPLE && key_f32(lb) < cut_key) return;                         // below the k-th largest allowed logit
        const uint32_t key = SAMPLE ? key_f32(__float_as_uint(__builtin_fmaf(__uint_as_float(lb), sp.inv_t, gumbel_of(word))))
                                    : key_f32(lb);
        if (key > best_key || (key == best_key && tok < best_idx)) {
            best_key = key;
            best_idx = tok;
        }
    };

    uint32_t t_head = 0, t_tail = 0, g_head = 0, g_tail = 0;   // ring positions, the same in all lanes
    float reached = -__builtin_inff();                         // a score some token of this wavefront has reached
    auto score_tokens = [&](uint32_t n) __attribute__((always_inline)) {   // n <= 64 queued tokens, one per lane
        wave_sync();
        if (lane < n) {
            const uint2 en = token_q[(t_head + lane) & (kQueue - 1)];
            uint32_t w[4];
            philox4x32_10(en.x >> 2, (uint32_t)b, sp.off_lo, sp.off_hi, sp.seed_lo, sp.seed_hi, w);
            const uint32_t lo = (en.x & 1u) ? w[1] : w[0], hi = (en.x & 1u) ? w[3] : w[2];
            consider(en.x, en.y, (en.x & 2u) ? hi : lo);
        }
        t_head += n;
        wave_sync();
        const uint32_t top = wave_max_u32(best_key);           // 0: nothing scored yet
        if (top != 0) {
            if (lane == 0) atomicMax(&s_reached, top);           // the other wavefronts of the row prune by it too
            reached = fmaxf(reached, __uint_as_float((top & 0x80000000u) ? top & 0x7FFFFFFFu : ~top));
        }
    };
    // Fetched groups are worked on one batch late: the logits of a batch are requested when it is
    // taken from the queue and used when the next batch is taken (or at the end), so that a
    // wavefront always has a load in flight while it computes.
    uint32_t m = 0, m_next = 0;                                // allowed bits of this lane's group; 0: none
    int t = 0, t_next = 0;                                     // its first token
    Elem e[8], e_next[8];
    bool own = false, own_next = false;                        // this lane holds a group (WRITE: also when m is 0)
    auto take_batch = [&](uint32_t n) __attribute__((always_inline)) {   // n <= 64 queued groups: request their logits
        wave_sync();
        m_next = 0;
        own_next = lane < n;
        if (own_next) {
            const uint2 en = group_q[(g_head + lane) & (kQueue - 1)];
            t_next = (int)en.x << 3;
            m_next = en.y;
            load_group<DTYPE>(row, t_next, V, e_next);
        }
        g_head += n;
        wave_sync();
    };
    auto work_batch = [&]() __attribute__((always_inline)) {   // the batch whose logits were requested before
        if constexpr (!SAMPLE) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t x = (uint32_t)e[j];
                if ((m >> j) & 1u) consider((uint32_t)(t + j), DTYPE == TDFA_F32 ? x : x << 16, 0u);
            }
        } else if (__ballot(m != 0) != 0) {
            uint32_t take = m;                                 // tokens to queue for scoring
            if (cut_key != 0) {                                // top-k: nothing below the cut is drawn (uniform branch)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t x = (uint32_t)e[j];
                    uint32_t lb = DTYPE == TDFA_F32 ? x : x << 16;
                    if ((lb & 0x7FFFFFFFu) > 0x7F800000u) lb = 0xFF800000u;
                    if (key_f32(lb) < cut_key) take &= ~(1u << j);
                }
            }
            float lv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t x = (uint32_t)e[j];
                uint32_t lb = DTYPE == TDFA_F32 ? x : x << 16;
                if ((lb & 0x7FFFFFFFu) > 0x7F800000u) lb = 0xFF800000u;
                lv[j] = __uint_as_float(lb);
            }
            {
                const uint32_t rk = __hip_atomic_load(&s_reached, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                const uint32_t top = (uint32_t)__builtin_amdgcn_readfirstlane((int)rk);
                if (top != 0) reached = fmaxf(reached, __uint_as_float((top & 0x80000000u) ? top & 0x7FFFFFFFu : ~top));
            }
            if (reached == -__builtin_inff() && __ballot(take != 0) != 0) {
                // Nothing scored in this row yet: one token per lane is scored right away, so that the
                // rest of the group already has a score to be measured against.
                const unsigned long long first = __ballot(take != 0);
                if (take != 0) {
                    const int j = __builtin_ctz(take);
                    take &= take - 1u;
                    float l = lv[0];
#pragma unroll
                    for (int i = 1; i < 8; ++i) l = j == i ? lv[i] : l;
                    token_q[(t_tail + below(first)) & (kQueue - 1)] = make_uint2((uint32_t)(t + j), __float_as_uint(l));
                }
                t_tail += (uint32_t)__popcll(first);
                if (t_tail - t_head > 64u) score_tokens(64u);    // fewer than 64 waited, at most 64 came
                score_tokens(t_tail - t_head);
            }
            // No noise value exceeds kNoiseMax, so a logit too far below a score already reached cannot
            // win whatever its noise: dropped before any generator block is made.  With peaked
            // logits (a language model's, or a low temperature) that is nearly all of the row.
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (!(__builtin_fmaf(lv[j], sp.inv_t, kNoiseMax) >= reached)) take &= ~(1u << j);
            const uint32_t live = take;
            if (__popcll(__ballot(__popc(live) >= 2)) >= 32) {
                // Still many: one generator block per four tokens, and a token is queued only if its
                // own noise lets it win.  With n = 2^23 - (x >> 9), u = 1 - (n - 1/2) 2^-23 and
                // g = -ln(-ln u) <= -ln(1 - u) <= (clz(n) - 7) ln 2; the slack added covers the
                // rounding of the noise as computed.  fma is monotonic in its addend, so a token
                // whose bound stays below a score already reached scores below it as well.
                take = 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t mh = (live >> (4 * h)) & 15u;
                    if (mh == 0) continue;
                    uint32_t w[4];
                    philox4x32_10((uint32_t)(t >> 2) + h, (uint32_t)b, sp.off_lo, sp.off_hi, sp.seed_lo, sp.seed_hi, w);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t n = 0x800000u - (w[j] >> 9);
                        const float ub = __builtin_fmaf((float)(__clz((int)n) - 7), 0.693147180559945309f, 1.0e-3f);
                        const float bound = __builtin_fmaf(lv[4 * h + j], sp.inv_t, ub);
                        take |= (uint32_t)(bound >= reached) << (4 * h + j);
                    }
                }
                take &= live;
            }
            // each lane hands over its next token per round; a round adds at most 64
            unsigned long long bal = __ballot(take != 0);
            while (bal != 0) {
                if (take != 0) {
                    const int j = __builtin_ctz(take);
                    take &= take - 1u;
                    float l = lv[0];
#pragma unroll
                    for (int i = 1; i < 8; ++i) l = j == i ? lv[i] : l;
                    token_q[(t_tail + below(bal)) & (kQueue - 1)] = make_uint2((uint32_t)(t + j), __float_as_uint(l));
                }
                t_tail += (uint32_t)__popcll(bal);
                if (t_tail - t_head >= 64u) score_tokens(64u);       // fewer than 64 waited, at most 64 came
                bal = __ballot(take != 0);
            }
        }
        if (WRITE && own) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (!((m >> j) & 1u)) e[j] = NEG_INF;
            store_group<DTYPE>(orow, t, V, e);
        }
    };
    bool pending_batch = false;                                // uniform: a batch has been taken and not worked on
    auto fetch_groups = [&](uint32_t n) __attribute__((always_inline)) {
        take_batch(n);
        if (pending_batch) work_batch();
        m = m_next;
        t = t_next;
        own = own_next;
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = e_next[j];
        pending_batch = true;
    };

    // Allowed bits, one 32-bit word (four groups) per load and lane, kWordsAhead loads in flight; g_lo
    // is a multiple of four groups (the launcher sees to that).
    const uint32_t* words = reinterpret_cast<const uint32_t*>(bits);
    const int w_lo = g_lo >> 2, w_hi = (g_hi + 3) >> 2;
    const int NT = (int)blockDim.x;
    auto load_word = [&](int wi) { return (valid && wi < w_hi) ? words[wi] : 0u; };
    static_assert(kWordsAhead == 4, "the rotation below is written for four words in flight");
    int wi = w_lo + (int)threadIdx.x;
    uint32_t w0 = load_word(wi), w1 = load_word(wi + NT), w2 = load_word(wi + 2 * NT), w3 = load_word(wi + 3 * NT);
    for (int base = w_lo; base < w_hi; base += NT, wi += NT) {               // trip count uniform in the workgroup
        const uint32_t w = w0;
        w0 = w1;
        w1 = w2;
        w2 = w3;
        w3 = load_word(wi + 4 * NT);
        const int left = g_hi - (wi << 2);                                   // groups of this word inside the part
        const uint32_t wm = left >= 4 ? w : (left > 0 ? w & ((1u << (8 * left)) - 1u) : 0u);
        if (!WRITE && __ballot(wm != 0) == 0) continue;
        // The 64 words of the wavefront cover 256 consecutive groups.  They are handed over 64
        // consecutive groups at a time (lane L takes byte L mod 4 of the word of lane 16 i + L / 4), so
        // that neighbouring lanes fetch neighbouring logits.
#pragma unroll 1
        for (int i = 0; i < 4; ++i) {
            const int src = 16 * i + (int)(lane >> 2);
            const uint32_t ws = (uint32_t)__shfl((int)wm, src, 64);
            const int g = ((wi - (int)lane + src) << 2) + (int)(lane & 3u);
            const uint32_t mg = (ws >> (8 * (lane & 3u))) & 0xFFu;
            const bool has = WRITE ? g < g_hi : mg != 0;                     // the masked row needs every group
            const unsigned long long bal = __ballot(has);
            if (bal == 0) continue;
            if (has) group_q[(g_tail + below(bal)) & (kQueue - 1)] = make_uint2((uint32_t)g, mg);
            g_tail += (uint32_t)__popcll(bal);
            if (g_tail - g_head >= 64u) fetch_groups(64u);
        }
    }
    if (g_tail != g_head) fetch_groups(g_tail - g_head);
    if (pending_batch) work_batch();
    if (t_tail != t_head) score_tokens(t_tail - t_head);
    unsigned long long cand = best_key ? ((unsigned long long)best_key << 32) | (0xFFFFFFFFu - best_idx) : 0ull;
    cand = block_max_u64(cand, wave_best);
    if (threadIdx.x != 0) return;
    if (combine_parts(a, b, parts, cand)) write_result(a, b, q, valid, cand);
}

// Runs of speculated tokens (Section 5.3): one lane per sequence follows its k tokens through the
// table and records every state on the way.  The lookups of a sequence depend on one another;
// the sequences are independent.
__global__ void __launch_bounds__(64)
advance_tokens_kernel(MaskArgs a, int32_t batch, int32_t k, const int32_t* __restrict__ states,
                      const int32_t* __restrict__ tokens, int32_t* __restrict__ history, int32_t* __restrict__ n_valid)
{
    const int b = blockIdx.x * 64 + threadIdx.x;
    if (b >= batch) return;
    int32_t s = states[b];
    if (s < 0 || (int64_t)s >= a.n_rows) s = TDFA_DEAD;
    int32_t* h = history + (int64_t)b * (k + 1);
    const int32_t* run = tokens + (int64_t)b * k;
    h[0] = s;
    int32_t ok = 0;
    for (int32_t i = 0; i < k; ++i) {
        const int32_t t = run[i];
        s = (s != TDFA_DEAD && t >= 0 && t < a.n_tokens) ? table_entry(a, s, t) : TDFA_DEAD;
        h[i + 1] = s;
        if (s != TDFA_DEAD && ok == i) ok = i + 1;
    }
    if (n_valid) n_valid[b] = ok;
}

// best[0 .. n) <- 0, count[0 .. n) <- 0
__global__ void __launch_bounds__(256)
clear_scratch_kernel(unsigned long long* __restrict__ best, unsigned int* __restrict__ count, int32_t n)
{
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < n) {
        best[i] = 0ull;
        count[i] = 0u;
    }
}

template <bool SAMPLE>
void launch_gather(const MaskArgs& a, const SampleParams& sp, dim3 grid, unsigned threads, int parts, int gpp, hipStream_t stream)
{
    if (a.dtype == TDFA_F32 && a.masked_out)
        gather_step_kernel<TDFA_F32, true, SAMPLE><<<grid, threads, 0, stream>>>(a, sp, parts, gpp);
    else if (a.dtype == TDFA_F32)
        gather_step_kernel<TDFA_F32, false, SAMPLE><<<grid, threads, 0, stream>>>(a, sp, parts, gpp);
    else if (a.masked_out)
        gather_step_kernel<TDFA_BF16, true, SAMPLE><<<grid, threads, 0, stream>>>(a, sp, parts, gpp);
    else
        gather_step_kernel<TDFA_BF16, false, SAMPLE><<<grid, threads, 0, stream>>>(a, sp, parts, gpp);
}

// Launch shape of the gather kernel: a row per workgroup of 1024 threads when the batch fills the
// chip, else rows split over `parts` workgroups of 256, each part a whole number of 32-bit words
// of allowed bits.
void gather_shape(const MaskArgs& a, int* parts_out, int* threads_out, int* gpp_out)
{
    const int n_groups = (a.n_tokens + 7) >> 3;
    int parts = 1, threads = 1024;
    if (a.batch < 192 || n_groups < 4096) {
        threads = 256;
        parts = (2048 + a.batch - 1) / a.batch;
        const int max_parts = (n_groups + 1023) / 1024;
        if (parts > max_parts) parts = max_parts;
    }
    if (parts < 1) parts = 1;
    int gpp = ((n_groups + parts - 1) / parts + 3) / 4 * 4;
    if (gpp < 4) gpp = 4;
    *parts_out = parts;
    *threads_out = threads;
    *gpp_out = gpp;
}

}  // namespace

// Launch shape of the streaming kernels: a row per workgroup of 1024 threads when there are
// enough rows to fill the 256 compute units: the result then needs no meeting of workgroups.
// Smaller batches split each row over `parts` workgroups of 256 threads, enough to have about
// 2048 of them, each with at least one unrolled pass of work.
namespace {
void stream_shape(const MaskArgs& a, int* parts_out, int* threads_out, int* gpp_out)
{
    const int n_groups = (a.n_tokens + 7) >> 3;
    int parts = 1, threads = 1024;
    if (a.batch < 192 || n_groups < 4096) {
        threads = 256;
        parts = (2048 + a.batch - 1) / a.batch;
        const int max_parts = (n_groups + 1023) / 1024;
        if (parts > max_parts) parts = max_parts;
    }
    if (parts < 1) parts = 1;
    int gpp = (n_groups + parts - 1) / parts;
    if (gpp < 1) gpp = 1;
    gpp = (gpp + 15) & ~15;                    // the bits of 16 groups are read at once
    *parts_out = parts;
    *threads_out = threads;
    *gpp_out = gpp;
}
}  // namespace

bool mask_step_uses_scratch(const MaskArgs& a)
{
    if (a.batch <= 0) return false;
    int parts, threads, gpp;
    if (!a.delta && a.targets) gather_shape(a, &parts, &threads, &gpp);
    else stream_shape(a, &parts, &threads, &gpp);
    return parts > 1;
}

int launch_clear_scratch(unsigned long long* best, unsigned int* count, int32_t n, hipStream_t stream)
{
    if (n <= 0) return TDFA_OK;
    clear_scratch_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(best, count, n);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

namespace {
// The launch of the 16-bit kernel that keeps a stretch's bits in LDS: shape, LDS bytes, and whether they fit.
struct BitsInLds {
    int parts, threads, gpp, unroll, stretch;
    size_t lds;
    bool fits;
};
BitsInLds bits_in_lds(const MaskArgs& a)
{
    BitsInLds r;
    stream_shape(a, &r.parts, &r.threads, &r.gpp);
    // groups per load batch: one for the few small workgroups of a small batch
    r.unroll = r.threads < 1024 && (int64_t)a.batch * r.parts <= 384 ? 1 : 2;
    // A stretch of the row per wavefront, in whole 16-group pieces; the bits of the stretches fit
    // in LDS for any vocabulary of a few hundred thousand tokens, else every stretch is streamed.
    const int n_waves = r.threads / 64;
    r.stretch = ((r.gpp + n_waves - 1) / n_waves + 15) & ~15;
    r.lds = (size_t)n_waves * ((size_t)r.stretch + 4 * 64 * (size_t)r.unroll);
    r.fits = !a.masked_out && r.lds <= (size_t)kMaxBitRowBytes;
    return r;
}
}  // namespace

bool mask_step_takes_pda(const MaskArgs& a)
{
    return a.batch > 0 && a.dtype != TDFA_F32 && !a.delta && !a.targets && a.n_tokens <= (1 << 27) && bits_in_lds(a).fits;
}

int launch_mask_step(const MaskArgs& a, hipStream_t stream)
{
    if (a.batch <= 0) return TDFA_OK;
    if (a.pda.class_first && !mask_step_takes_pda(a)) return fail(TDFA_E_UNSUPPORTED, "this step wants one row of allowed bits per sequence");
    if (!a.delta && a.targets) {
        // a packed table: the scan that reads only the groups with allowed tokens
        int g_parts, g_threads, g_gpp;
        gather_shape(a, &g_parts, &g_threads, &g_gpp);
        if ((int64_t)a.batch * g_parts > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "batch too large for one launch");
        launch_gather<false>(a, SampleParams{}, dim3((unsigned)(a.batch * g_parts)), (unsigned)g_threads, g_parts, g_gpp, stream);
        TDFA_HIP(hipGetLastError());
        return TDFA_OK;
    }
    const BitsInLds sh = bits_in_lds(a);
    const int parts = sh.parts, threads = sh.threads, gpp = sh.gpp, unroll = sh.unroll, stretch = sh.stretch;
    const size_t lds = sh.lds;
    const bool skip = sh.fits;
    if ((int64_t)a.batch * parts > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "batch too large for one launch");
    // the 16-bit kernel addresses a row through 32-bit byte offsets
    if (a.dtype != TDFA_F32 && a.n_tokens > (1 << 27)) return fail(TDFA_E_UNSUPPORTED, "more than 2^27 tokens in a 16-bit row");
    const dim3 grid((unsigned)(a.batch * parts));
    const unsigned kThreads = (unsigned)threads;
    const int n_waves = threads / 64;
    if (skip && a.dtype != TDFA_F32 && lds > (size_t)kPlainLdsBytes) {
        // once per device: let the kernels that keep the bits in LDS take more than the default 64 KB
        static bool raised[64] = {};
        int dev = 0;
        TDFA_HIP(hipGetDevice(&dev));
        if (dev >= 0 && dev < 64 && !raised[dev]) {
            for (const void* k : {reinterpret_cast<const void*>(mask_step_bf16_kernel<false, 1, true>),
                                  reinterpret_cast<const void*>(mask_step_bf16_kernel<false, 2, true>),
                                  reinterpret_cast<const void*>(mask_step_bf16_kernel<false, 1, true, 2, true>),
                                  reinterpret_cast<const void*>(mask_step_bf16_kernel<false, 2, true, 2, true>)})
                TDFA_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxBitRowBytes));
            raised[dev] = true;
        }
    }
    if (a.pda.class_first) {
        if (unroll == 1) mask_step_bf16_kernel<false, 1, true, 2, true><<<grid, kThreads, lds, stream>>>(a, parts, gpp, stretch);
        else mask_step_bf16_kernel<false, 2, true, 2, true><<<grid, kThreads, lds, stream>>>(a, parts, gpp, stretch);
        TDFA_HIP(hipGetLastError());
        return TDFA_OK;
    }
    if (a.dtype == TDFA_F32 && !a.masked_out && (size_t)n_waves * (size_t)stretch <= (size_t)kPlainLdsBytes)
        mask_step_f32_kernel<<<grid, kThreads, (size_t)n_waves * (size_t)stretch, stream>>>(a, parts, gpp, stretch);
    else if (a.dtype == TDFA_F32)
        mask_step_exact_kernel<TDFA_F32><<<grid, kThreads, 0, stream>>>(a, parts, gpp);
    else if (a.masked_out)
        mask_step_bf16_kernel<true, 2, false><<<grid, kThreads, 0, stream>>>(a, parts, gpp, stretch);
    else if (skip && unroll == 1)
        mask_step_bf16_kernel<false, 1, true><<<grid, kThreads, lds, stream>>>(a, parts, gpp, stretch);
    else if (skip)
        mask_step_bf16_kernel<false, 2, true><<<grid, kThreads, lds, stream>>>(a, parts, gpp, stretch);
    else if (unroll == 1)
        mask_step_bf16_kernel<false, 1, false><<<grid, kThreads, 0, stream>>>(a, parts, gpp, stretch);
    else
        mask_step_bf16_kernel<false, 2, false><<<grid, kThreads, 0, stream>>>(a, parts, gpp, stretch);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

int launch_sample_step(const MaskArgs& a, float inv_t, int32_t top_k, uint32_t* cut_scratch, uint64_t seed,
                       uint64_t offset, const uint64_t* offset_dev, hipStream_t stream)
{
    if (a.batch <= 0) return TDFA_OK;
    if (top_k > 0) {
        const unsigned t = a.n_tokens >= 32768 ? 1024u : 256u;
        if (a.dtype == TDFA_F32)
            topk_cut_kernel<TDFA_F32><<<(unsigned)a.batch, t, 0, stream>>>(a, top_k, cut_scratch);
        else
            topk_cut_kernel<TDFA_BF16><<<(unsigned)a.batch, t, 0, stream>>>(a, top_k, cut_scratch);
        TDFA_HIP(hipGetLastError());
    }
    int parts, threads, gpp;
    gather_shape(a, &parts, &threads, &gpp);
    if ((int64_t)a.batch * parts > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "batch too large for one launch");
    const dim3 grid((unsigned)(a.batch * parts));
    SampleParams sp;
    sp.inv_t = inv_t;
    sp.seed_lo = (uint32_t)seed;
    sp.seed_hi = (uint32_t)(seed >> 32);
    sp.off_lo = (uint32_t)offset;
    sp.off_hi = (uint32_t)(offset >> 32);
    sp.cut = top_k > 0 ? cut_scratch : nullptr;
    sp.off_dev = reinterpret_cast<const unsigned long long*>(offset_dev);
    launch_gather<true>(a, sp, grid, (unsigned)threads, parts, gpp, stream);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

int launch_sample_noise(int32_t batch, int32_t n_tokens, uint64_t seed, uint64_t offset, float* out, hipStream_t stream)
{
    if (batch <= 0 || n_tokens <= 0) return TDFA_OK;
    const int32_t quads_per_row = (n_tokens + 3) / 4;
    const int64_t total = (int64_t)batch * quads_per_row;
    if ((total + 255) / 256 > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "batch * n_tokens too large for one launch");
    SampleParams sp;
    sp.inv_t = 1.0f;
    sp.cut = nullptr;
    sp.off_dev = nullptr;
    sp.seed_lo = (uint32_t)seed;
    sp.seed_hi = (uint32_t)(seed >> 32);
    sp.off_lo = (uint32_t)offset;
    sp.off_hi = (uint32_t)(offset >> 32);
    sample_noise_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(sp, n_tokens, total, quads_per_row, out);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

int launch_advance_tokens(const MaskArgs& table, int32_t batch, int32_t k, const int32_t* states, const int32_t* tokens,
                          int32_t* history, int32_t* n_valid, hipStream_t stream)
{
    if (batch <= 0) return TDFA_OK;
    advance_tokens_kernel<<<(batch + 63) / 64, 64, 0, stream>>>(table, batch, k, states, tokens, history, n_valid);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace tdfa
