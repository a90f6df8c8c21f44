// Compile stage: the token-level table delta_T of A_R o T_V (Sections 2.3-2.4; Algorithm 2,
// statement 3) and its allowed-bit rows, for gfx950.
//
// With a deterministic A_R, composing with T_V (Algorithm 1) and removing epsilon edges gives
// delta_T[q][t] = delta*(q, d(t)): walk the bytes of token t from state q, DEAD at the first
// missing transition (Theorems 1 and 2).  Every (q, t) entry is independent, the output is
// 4 bytes per entry, and for real constraints almost every entry is DEAD, so the kernel is a
// streaming writer with a sparse compute phase in front of it:
//
//   1. transpose_kernel: delta[q][b] (int32, as uploaded) -> delta^T[b][q], narrowed to int16
//      when the states fit.  One byte's column is then contiguous: the first step of a walk is
//      a coalesced load for 64 consecutive states, and later steps gather inside one column
//      (2|Q| bytes) instead of across the whole table.
//   2. compile_tile_kernel: a workgroup owns S states x T consecutive token ids.  The tile lives
//      in LDS, pre-filled with DEAD.  Each wavefront takes one token at a time (its bytes come
//      through scalar loads) with lanes = states; it stops as soon as no lane is alive, and only
//      live results are written to the tile.  Then the tile is flushed row by row: 64 lanes write
//      64 consecutive int32 entries (256 B) and one wave ballot gives the two 32-bit allowed
//      words for the same 64 tokens.
#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// delta[q][b] -> out[b][q]; columns q in [n_states, q_stride) are filled with DEAD.
template <typename ST>
__global__ void __launch_bounds__(kThreads)
transpose_kernel(const int32_t* __restrict__ trans, ST* __restrict__ out, int n_states, int q_stride)
{
    __shared__ int32_t tile[64][65];
    const int q0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < 64; r += kWaves) {
        const int q = q0 + r;
        tile[r][lane] = q < n_states ? trans[(size_t)q * 256 + b0 + lane] : TDFA_DEAD;
    }
    __syncthreads();
    for (int c = wave; c < 64; c += kWaves) {
        const int q = q0 + lane;
        if (q < q_stride) out[(size_t)(b0 + c) * q_stride + q] = (ST)tile[lane][c];
    }
}

template <typename ST, int S, int T>
__global__ void __launch_bounds__(kThreads)
compile_tile_kernel(const ST* __restrict__ tt, int n_states, int q_stride,
                    const uint32_t* __restrict__ vwords, const uint32_t* __restrict__ voff,
                    const uint32_t* __restrict__ vlen, int n_tokens, int n_tiles_t,
                    int32_t* __restrict__ delta, uint32_t* __restrict__ allow, int64_t row_words)
{
    static_assert(S % 64 == 0 && T % 128 == 0, "tile shape");
    // Row stride with an odd number of 32-bit words: lanes that write one token column for 64
    // consecutive states hit 64 different LDS banks.
    constexpr int RS = T + (sizeof(ST) == 2 ? 2 : 1);
    extern __shared__ __align__(16) unsigned char smem[];
    ST* tile = reinterpret_cast<ST*>(smem);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile_t = blockIdx.x % n_tiles_t, tile_q = blockIdx.x / n_tiles_t;
    const int t0 = tile_t * T, q0 = tile_q * S;

    {
        uint32_t* w = reinterpret_cast<uint32_t*>(smem);
        constexpr int n_words = S * RS * (int)sizeof(ST) / 4;
        for (int i = threadIdx.x; i < n_words; i += kThreads) w[i] = 0xFFFFFFFFu;
    }
    __syncthreads();

    const int t_end = min(T, n_tokens - t0);
    for (int tl = wave; tl < t_end; tl += kWaves) {
        const int t = t0 + tl;
        const uint32_t len = vlen[t];
        if (len == 0) continue;                       // no cycle in T_V: DEAD for every state
        const uint32_t* w = vwords + voff[t];
        const uint32_t w0 = w[0];
        const ST* col1 = tt + (size_t)(w0 & 0xFFu) * q_stride;
        for (int g = 0; g < S / 64; ++g) {
            const int r = g * 64 + lane;
            const int q = q0 + r;
            int v = q < n_states ? (int)col1[q] : TDFA_DEAD;
            uint32_t cur = w0;
            for (uint32_t i = 1; i < len && __builtin_amdgcn_ballot_w64(v >= 0) != 0; ++i) {
                if ((i & 3u) == 0) cur = w[i >> 2];
                const uint32_t b = (cur >> ((i & 3u) * 8)) & 0xFFu;
                if (v >= 0) v = (int)tt[(size_t)b * q_stride + v];
            }
            if (v >= 0) tile[r * RS + tl] = (ST)v;
        }
    }
    __syncthreads();

    for (int r = wave; r < S; r += kWaves) {
        const int q = q0 + r;
        if (q >= n_states) break;
        int32_t* drow = delta + (size_t)q * n_tokens;
        uint32_t* arow = allow + (size_t)q * row_words;
#pragma unroll
        for (int k = 0; k < T / 64; ++k) {
            const int tl = k * 64 + lane;
            const int t = t0 + tl;
            const int v = (int)tile[r * RS + tl];
            if (t < n_tokens) drow[t] = v;
            const uint64_t m = __builtin_amdgcn_ballot_w64(v >= 0);
            const int64_t word = (int64_t)((t0 + k * 64) >> 5) + lane;
            if (lane < 2 && word < row_words) arow[word] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
        }
    }
}

// dst rows [row_base, row_base + n_rows): copy of src with row_base added to live entries.
__global__ void __launch_bounds__(kThreads)
concat_delta_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int64_t n, int32_t base)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const int32_t v = src[i];
        dst[i] = v < 0 ? TDFA_DEAD : v + base;
    }
}

__global__ void __launch_bounds__(kThreads)
copy_words_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

template <typename ST, int S, int T>
int launch_tiles(const CompileArgs& a, hipStream_t stream)
{
    constexpr int RS = T + (sizeof(ST) == 2 ? 2 : 1);
    constexpr size_t lds = (size_t)S * RS * sizeof(ST);
    const int64_t n_tiles_t = (a.n_tokens + T - 1) / T;
    const int64_t n_tiles_q = (a.n_states + S - 1) / S;
    if (n_tiles_t * n_tiles_q > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "table too large for one launch");
    auto kern = compile_tile_kernel<ST, S, T>;
    static bool attr_set = false;
    if (!attr_set) {
        TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds));
        attr_set = true;
    }
    kern<<<dim3((unsigned)(n_tiles_t * n_tiles_q)), kThreads, lds, stream>>>(
        static_cast<const ST*>(a.trans_t), a.n_states, a.q_stride, a.vwords, a.voff, a.vlen, a.n_tokens,
        (int)n_tiles_t, a.delta, a.allow, a.row_words);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace

int launch_compile(const CompileArgs& a, hipStream_t stream)
{
    if (a.n_states <= 0 || a.n_tokens <= 0) return TDFA_OK;
    const dim3 tgrid((a.q_stride + 63) / 64, 4);
    if (a.narrow)
        transpose_kernel<int16_t><<<tgrid, kThreads, 0, stream>>>(a.trans, static_cast<int16_t*>(a.trans_t),
                                                                  a.n_states, a.q_stride);
    else
        transpose_kernel<int32_t><<<tgrid, kThreads, 0, stream>>>(a.trans, static_cast<int32_t*>(a.trans_t),
                                                                  a.n_states, a.q_stride);
    TDFA_HIP(hipGetLastError());
    return a.narrow ? launch_tiles<int16_t, 128, 256>(a, stream) : launch_tiles<int32_t, 64, 256>(a, stream);
}

int launch_concat_part(const int32_t* src_delta, const uint32_t* src_allow, int64_t n_rows, int32_t n_tokens,
                       int64_t row_words, int64_t row_base, int32_t* dst_delta, uint32_t* dst_allow,
                       hipStream_t stream)
{
    const int64_t n = n_rows * n_tokens, nw = n_rows * row_words;
    if (n <= 0) return TDFA_OK;
    const int64_t b1 = (n + kThreads - 1) / kThreads;
    const unsigned g1 = (unsigned)(b1 < 65536 ? b1 : 65536);
    concat_delta_kernel<<<g1, kThreads, 0, stream>>>(src_delta, dst_delta + row_base * n_tokens, n, (int32_t)row_base);
    TDFA_HIP(hipGetLastError());
    const int64_t b2 = (nw + kThreads - 1) / kThreads;
    const unsigned g2 = (unsigned)(b2 < 65536 ? b2 : 65536);
    copy_words_kernel<<<g2, kThreads, 0, stream>>>(src_allow, dst_allow + row_base * row_words, nw);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace tdfa
