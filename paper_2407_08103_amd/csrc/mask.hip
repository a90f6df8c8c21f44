// Decode step: loop body of Algorithm 2 after ComputeLogits (allowed set, -inf penalty, greedy
// token choice, edge traversal), batched over sequences, for gfx950.
//
// The allowed set of a state is its row of allowed bits (1 bit per token, written by the compile
// stage), so a step reads |V| logits plus |V|/8 mask bytes per sequence and one table entry
// for the chosen token.  Nothing here is a contraction: the kernel streams logits with 16-byte
// loads and reduces (value, token id) pairs with wavefront shuffles.
//
// Ordering of candidates.  Each allowed logit is mapped to an unsigned key that preserves the
// order of the floating-point values, with every NaN mapped to the key of -inf and -0 to +0.  Candidates are
// compared as the 64-bit number (key << 32) | (0xFFFFFFFF - token), so the largest value wins and
// the lowest token id wins ties; 0 means "nothing allowed" (the smallest key of an allowed
// token, that of -inf, is above 0).
#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

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

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// One workgroup handles one part of one sequence's row; `parts` workgroups share a row and are
// combined through scratch_best / scratch_count (both zero on entry and left zero on exit).
template <int DTYPE>
__global__ void __launch_bounds__(kThreads)
mask_step_kernel(MaskArgs a, int parts, int groups_per_part)
{
    using Elem = typename std::conditional<DTYPE == TDFA_F32, uint32_t, uint16_t>::type;
    const int b = blockIdx.x / parts, p = blockIdx.x % parts;
    const int V = a.n_tokens;
    const int q = a.states[b];
    const bool valid = q >= 0 && (int64_t)q < a.n_rows;
    const uint8_t* bits = reinterpret_cast<const uint8_t*>(a.allow + (valid ? (int64_t)q * a.row_words : 0));
    const Elem* row = static_cast<const Elem*>(a.logits) + (int64_t)b * a.row_stride;
    Elem* orow = a.masked_out ? static_cast<Elem*>(a.masked_out) + (int64_t)b * a.row_stride : nullptr;
    constexpr Elem NEG_INF = DTYPE == TDFA_F32 ? (Elem)0xFF800000u : (Elem)0xFF80u;

    const int n_groups = (V + 7) >> 3;
    const int g_lo = p * groups_per_part;
    const int g_hi = min(n_groups, g_lo + groups_per_part);

    uint32_t best_key = 0, best_idx = 0;
    for (int g = g_lo + (int)threadIdx.x; g < g_hi; g += kThreads) {
        const int t = g << 3;
        const uint32_t m = valid ? bits[g] : 0u;
        Elem e[8];
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
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = (m >> j) & 1u;
            const uint32_t key = DTYPE == TDFA_F32 ? key_f32((uint32_t)e[j]) : key_bf16((uint32_t)e[j]);
            if (ok && key > best_key) { best_key = key; best_idx = (uint32_t)(t + j); }
            if (!ok) e[j] = NEG_INF;
        }
        if (orow) {
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
    }

    unsigned long long cand = best_key ? ((unsigned long long)best_key << 32) | (0xFFFFFFFFu - best_idx) : 0ull;
    cand = wave_max_u64(cand);
    __shared__ unsigned long long wave_best[kWaves];
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = cand;
    __syncthreads();
    if (threadIdx.x != 0) return;
#pragma unroll
    for (int w = 1; w < kWaves; ++w) cand = wave_best[w] > cand ? wave_best[w] : cand;

    if (parts > 1) {
        if (cand) atomicMax(&a.scratch_best[b], cand);
        __threadfence();
        const unsigned done = atomicAdd(&a.scratch_count[b], 1u);
        if (done != (unsigned)parts - 1) return;
        __threadfence();
        cand = __hip_atomic_exchange(&a.scratch_best[b], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&a.scratch_count[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    int32_t token = TDFA_NO_TOKEN, next = valid ? q : TDFA_DEAD;
    if (cand) {
        token = (int32_t)(0xFFFFFFFFu - (uint32_t)cand);
        next = a.delta[(int64_t)q * V + token];
    }
    a.tokens[b] = token;
    a.new_states[b] = next;
}

}  // namespace

int launch_mask_step(const MaskArgs& a, hipStream_t stream)
{
    if (a.batch <= 0) return TDFA_OK;
    const int n_groups = (a.n_tokens + 7) >> 3;
    // enough workgroups to fill 256 compute units several times over, each with a few
    // thousand tokens at least
    int parts = (2048 + a.batch - 1) / a.batch;
    const int max_parts = (n_groups + 1023) / 1024;
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    int gpp = (n_groups + parts - 1) / parts;
    if (gpp < 1) gpp = 1;
    if ((int64_t)a.batch * parts > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "batch too large for one launch");
    const dim3 grid((unsigned)(a.batch * parts));
    if (a.dtype == TDFA_F32)
        mask_step_kernel<TDFA_F32><<<grid, kThreads, 0, stream>>>(a, parts, gpp);
    else
        mask_step_kernel<TDFA_BF16><<<grid, kThreads, 0, stream>>>(a, parts, gpp);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace tdfa
