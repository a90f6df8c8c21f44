// Compile stage for large automata without counter-like classes: delta_T through lists of the
// states that survive a token's first two bytes (Sections 2.3-2.4; Algorithm 2, statement 3).
//
// delta_T[q][t] = delta*(q, d(t)) factors over the prefix trie of the vocabulary (the compact T_V
// of Section 2.3 merges tokens that share a prefix): the state after the first two bytes (b1, b2)
// of a token depends on (q, b1, b2) only, and there are at most 65,536 such prefixes however large
// the vocabulary is.  In an automaton whose states accept a fraction p of the bytes, a fraction
// p^2 of the states survives two bytes, so the walks of all tokens that share a prefix start from a
// short list instead of from every state:
//
//   1. pair_count_kernel / pair_scan_kernel / pair_fill_kernel: for every tile of 256 states (in
//      lane order) and every prefix (b1, b2) the list of (row in tile, delta*(q, b1 b2)) of the
//      states that survive, stored back to back with an index of list starts.  A workgroup owns
//      (tile, b1): its surviving states after b1 are compacted in LDS, thread b2 reads row
//      delta[r][b2] of each of them (consecutive threads, consecutive entries) and counts, then
//      after an exclusive scan over all lists writes its own list.
//   2. pair_tile_kernel: a workgroup owns 256 states x 256 consecutive token ids.  Its wavefronts
//      read the lists of their tokens (lanes = surviving pairs, whatever token they belong to) and
//      walk the remaining bytes, one gather per byte and live pair, sixteen pairs per lane side by
//      side; the rows leave through an LDS tile of 64 tokens at a time with 16-byte streaming
//      stores, and the allowed bits of the 256 tokens are written once per row as a whole 32-byte
//      sector.  Details at the kernel.
#include <algorithm>

#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kPS = 256;          // states per tile
constexpr int kPT = 64;           // tokens per sub-tile: the tokens of two wavefronts
constexpr int kPSub = 4;          // sub-tiles per workgroup
constexpr int kPBlockT = kPT * kPSub;
constexpr int kPThreads = 512;
constexpr int kPWaves = kPThreads / 64;
constexpr int kPRS = kPT + 2;     // tile row stride in 16-bit entries: an odd number of 32-bit words
constexpr uint32_t kDead16 = 0xFFFFu;

struct PairDesc {
    const uint16_t* tt;        // [256][q_stride] transposed table, offset form (entry = state * 2, sink = (q_stride - 1) * 2)
    const int32_t* trans;      // [n_states][256] as uploaded
    uint16_t* rows16;          // [n_states][256] workspace: target state or 0xFFFF
    uint32_t* live_bits;       // [256][q_stride / 32] workspace: bit q & 31 of word q >> 5 of column b set = delta(q, b) is defined
    const int32_t* order;      // [n_order] states in lane order, -1 = idle lane
    uint32_t* idx;             // [n_tiles_q * 65536 + 1] list starts (counts between the first and the third kernel)
    uint32_t* block_tot;       // [n_tiles_q * 256] pairs per (tile, b1); after the scan: pairs before it
    uint32_t* pairs;           // [n_pairs] (row in tile << 24) | state after two bytes
    int32_t n_states, n_order, q_stride, n_tiles_q;
    int32_t out_row, state_base;
};

__global__ void __launch_bounds__(256)
narrow_rows_kernel(PairDesc d)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)d.n_states * 256) return;
    const int32_t v = d.trans[i];
    d.rows16[i] = v < 0 ? (uint16_t)kDead16 : (uint16_t)v;
}

// One word of live_bits per thread, from 32 consecutive entries of a column of the transposed table.
__global__ void __launch_bounds__(256)
live_bits_kernel(PairDesc d)
{
    const int words = d.q_stride >> 5;
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i >= 256 * words) return;
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    const uint16_t* src = d.tt + (size_t)i * 32;             // column i / words, states 32 (i % words) ..
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) w |= (src[j] != sink ? 1u : 0u) << j;
    d.live_bits[i] = w;
}

// The states of tile qt that survive byte b1, compacted into s_list as (row in tile << 16) | target.
// Called by all 256 threads; returns the number of entries.  Ends with a barrier.
__device__ __forceinline__ int survivors_after_b1(const PairDesc& d, int qt, int b1, uint32_t* s_list, int* s_wave)
{
    const int l = (int)threadIdx.x, lane = l & 63, wave = l >> 6;
    const int i = qt * kPS + l;
    const int q = i < d.n_order ? d.order[i] : -1;
    const uint32_t sink = (uint32_t)(d.q_stride - 1) * 2u;
    uint32_t e = sink;
    if (q >= 0) e = d.tt[(size_t)b1 * (size_t)d.q_stride + (size_t)q];
    const bool live = e != sink;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(live);
    if (lane == 0) s_wave[wave] = __popcll(bal);
    __syncthreads();
    int base = 0, n = 0;
    for (int w = 0; w < 4; ++w) {
        const int c = s_wave[w];
        if (w < wave) base += c;
        n += c;
    }
    if (live) {
        const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
        s_list[pos] = ((uint32_t)l << 16) | (e >> 1);
    }
    __syncthreads();
    return n;
}

// counts: idx[(qt * 256 + b1) * 256 + b2] = number of states of tile qt that survive (b1, b2)
__global__ void __launch_bounds__(256)
pair_count_kernel(PairDesc d)
{
    __shared__ uint32_t s_list[kPS];
    __shared__ int s_wave[4];
    const int qt = (int)(blockIdx.x >> 8), b1 = (int)(blockIdx.x & 255u);
    const int n = survivors_after_b1(d, qt, b1, s_list, s_wave);
    const int b2 = (int)threadIdx.x;
    const uint16_t* __restrict__ rows = d.rows16;
    uint32_t cnt = 0;
    int j = 0;
    for (; j + 4 <= n; j += 4) {
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = rows[(size_t)(s_list[j + u] & 0xFFFFu) * 256 + b2];
#pragma unroll
        for (int u = 0; u < 4; ++u) cnt += v[u] != kDead16;
    }
    for (; j < n; ++j) cnt += rows[(size_t)(s_list[j] & 0xFFFFu) * 256 + b2] != kDead16;
    d.idx[(size_t)blockIdx.x * 256 + b2] = cnt;
    // pairs of the whole block
    uint32_t tot = cnt;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) tot += __shfl_xor(tot, s, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = (int)tot;
    __syncthreads();
    if (threadIdx.x == 0) d.block_tot[blockIdx.x] = (uint32_t)(s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3]);
}

// block_tot <- its exclusive prefix sums; idx[last] <- the total.  One workgroup.
__global__ void __launch_bounds__(1024)
pair_scan_kernel(PairDesc d)
{
    __shared__ uint32_t s_wave[16];
    __shared__ uint32_t s_carry;
    const int n = d.n_tiles_q * 256;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < n; base += 1024) {
        const int i = base + (int)threadIdx.x;
        const uint32_t v = i < n ? d.block_tot[i] : 0u;
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
        if (i < n) d.block_tot[i] = before + incl - v;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) d.idx[(size_t)n * 256] = s_carry;
}

// idx <- list starts; pairs <- the lists.  The lists of a workgroup's 256 prefixes (b1, 0 .. 255) lie
// back to back, so they are put together in LDS and leave as one run of consecutive words; a
// workgroup with more pairs than the staging buffer holds writes them where they go directly.
constexpr int kPStage = 8192;
__global__ void __launch_bounds__(256)
pair_fill_kernel(PairDesc d)
{
    __shared__ uint32_t s_list[kPS];
    __shared__ int s_wave[4];
    __shared__ uint32_t s_scan[4];
    __shared__ uint32_t s_stage[kPStage];
    const int qt = (int)(blockIdx.x >> 8), b1 = (int)(blockIdx.x & 255u);
    const int n = survivors_after_b1(d, qt, b1, s_list, s_wave);
    const int b2 = (int)threadIdx.x, lane = b2 & 63, wave = b2 >> 6;
    const uint32_t cnt = d.idx[(size_t)blockIdx.x * 256 + b2];
    uint32_t incl = cnt;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const uint32_t o = __shfl_up(incl, s, 64);
        if (lane >= s) incl += o;
    }
    if (lane == 63) s_scan[wave] = incl;
    __syncthreads();
    const uint32_t block_base = d.block_tot[blockIdx.x];
    const uint32_t block_total = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
    uint32_t local = incl - cnt;
    for (int w = 0; w < wave; ++w) local += s_scan[w];
    d.idx[(size_t)blockIdx.x * 256 + b2] = block_base + local;
    const bool staged = block_total <= (uint32_t)kPStage;                 // uniform
    const uint16_t* __restrict__ rows = d.rows16;
    uint32_t* out = staged ? s_stage + local : d.pairs + block_base + local;
    uint32_t k = 0;
    int j = 0;
    for (; j + 4 <= n; j += 4) {
        uint32_t en[4], v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            en[u] = s_list[j + u];
            v[u] = rows[(size_t)(en[u] & 0xFFFFu) * 256 + b2];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (v[u] != kDead16) out[k++] = ((en[u] >> 16) << 24) | v[u];
    }
    for (; j < n; ++j) {
        const uint32_t en = s_list[j];
        const uint32_t v = rows[(size_t)(en & 0xFFFFu) * 256 + b2];
        if (v != kDead16) out[k++] = ((en >> 16) << 24) | v;
    }
    if (!staged) return;
    __syncthreads();
    uint32_t* __restrict__ dst = d.pairs + block_base;
    for (uint32_t i = threadIdx.x; i < block_total; i += 256) dst[i] = s_stage[i];
}

struct PairVocab {
    const uint32_t* vwords;
    const uint32_t* voff;
    const uint32_t* vlen;
    const uint32_t* vprefix;
    int32_t n_tokens;
};

constexpr int kPChains = 16;      // pairs a lane walks side by side; a wavefront's first 64 * kPChains pairs
constexpr size_t kPairTileBytes = (size_t)kPS * kPRS * 2;
// tile, allowed bits, token bytes, lengths, list starts, list lengths (16-bit), states (16-bit), prefix sums:
// 54,400 bytes, so that three workgroups share a compute unit's 160 KB
constexpr size_t kPairLdsBytes = kPairTileBytes + (size_t)kPS * 8 * 4 + (size_t)kPBlockT * (32 + 4 + 4 + 2) + (size_t)kPS * 2 +
                                 (size_t)kPWaves * 36 * 4;
static_assert(3 * kPairLdsBytes <= 160 * 1024, "three workgroups per compute unit");
static_assert(kPT == 64 && kPSub * 2 == kPWaves, "a sub-tile holds the tokens of two wavefronts");

// One workgroup: 256 states (tile qt, in lane order) x 256 consecutive token ids.
//   set-up   the block's tokens (length, first 32 bytes) and the bounds of their lists come to LDS
//   walk     wavefront w owns tokens 32 w .. 32 w + 31 of the block.  Its pairs (all tokens' lists one
//            after the other) are dealt to the lanes, kPChains per lane, and walked together: a
//            level issues up to kPChains independent lookups per lane, so the latency of a level is
//            paid once per block and not once per token; after every level the pairs still alive
//            are packed into the lowest chains (through the tile's LDS, idle until the turns).
//            Results stay in registers.
//   4 turns  sub-tile s = tokens 64 s .. 64 s + 63: the two wavefronts that own them put their
//            results into the LDS tile (all DEAD before; an entry is the target state + 1), one-byte
//            tokens take their byte's column with lanes = states, pairs beyond a wavefront's
//            register chains are walked now; then all wavefronts flush the tile's rows with 16-byte
//            streaming stores, put DEAD back, and collect the allowed bits in LDS
//   bits     eight words (32 bytes) per row, written once
// (six wavefronts per SIMD = three workgroups per compute unit: the register budget is set to match the LDS budget)
template <bool WIDE_ROWS, bool BASE0>
__global__ void __launch_bounds__(kPThreads) __attribute__((amdgpu_waves_per_eu(6, 6)))
pair_tile_kernel(PairDesc d, PairVocab v, int n_blocks_t, int32_t* __restrict__ delta, uint32_t* __restrict__ allow,
                 int64_t row_words, int allow_vec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* tile = reinterpret_cast<uint16_t*>(smem);
    uint32_t* s_bits = reinterpret_cast<uint32_t*>(smem + kPairTileBytes);   // [kPS][8]
    uint32_t* s_bytes = s_bits + kPS * 8;                                      // [kPBlockT][8]
    uint32_t* s_len = s_bytes + kPBlockT * 8;
    uint32_t* s_beg = s_len + kPBlockT;
    uint32_t* s_pre = s_beg + kPBlockT;                                        // [kPWaves][36]
    uint16_t* s_cnt = reinterpret_cast<uint16_t*>(s_pre + kPWaves * 36);       // [kPBlockT] at most 256 pairs per list
    int16_t* s_state = reinterpret_cast<int16_t*>(s_cnt + kPBlockT);           // [kPS] the automaton has at most 32,767 states

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int bt = (int)(blockIdx.x % (unsigned)n_blocks_t), qt = (int)(blockIdx.x / (unsigned)n_blocks_t);
    const int n_tokens = v.n_tokens;
    const int t_block = bt * kPBlockT;
    const uint16_t* __restrict__ tt = d.tt;
    const uint32_t q_stride = (uint32_t)d.q_stride;
    const uint32_t SINK = (q_stride - 1u) * 2u;
    const uint32_t* __restrict__ idx = d.idx + (size_t)qt * 65536;
    const uint32_t* __restrict__ pairs = d.pairs;
    const int state_base = d.state_base;
    const uint32_t out_row32 = (uint32_t)d.out_row, nt32 = (uint32_t)n_tokens, rw32 = (uint32_t)row_words;

    // ---- set-up
    {
        for (int r = threadIdx.x; r < kPS; r += kPThreads) s_state[r] = (int16_t)(qt * kPS + r < d.n_order ? d.order[qt * kPS + r] : -1);
        for (int i = threadIdx.x; i < kPBlockT * 8; i += kPThreads)
            s_bytes[i] = t_block + (i >> 3) < n_tokens ? v.vprefix[(size_t)t_block * 8 + i] : 0u;
        if (threadIdx.x < kPBlockT) {
            const int tl = (int)threadIdx.x, t = t_block + tl;
            uint32_t len = 0, beg = 0, cnt = 0;
            if (t < n_tokens) {
                len = v.vlen[t];
                if (len >= 2) {
                    const uint32_t w0 = v.vprefix[(size_t)t * 8];
                    const uint32_t p = ((w0 & 0xFFu) << 8) | ((w0 >> 8) & 0xFFu);
                    beg = idx[p];
                    cnt = idx[p + 1] - beg;
                }
            }
            s_len[tl] = len;
            s_beg[tl] = beg;
            s_cnt[tl] = (uint16_t)cnt;
        }
    }
    __syncthreads();

    // ---- walk: this wavefront's 32 tokens
    const int tl0 = wave * 32;
    uint32_t* pre = s_pre + wave * 36;                  // pre[k] = pairs of the wavefront's tokens before token k; pre[32] = all
    uint32_t total;
    {
        const uint32_t c = lane < 32 ? s_cnt[tl0 + lane] : 0u;
        uint32_t incl = c;
#pragma unroll
        for (int sft = 1; sft < 32; sft <<= 1) {
            const uint32_t o = __shfl_up(incl, sft, 64);
            if (lane >= sft) incl += o;
        }
        if (lane < 32) pre[lane + 1] = incl;
        if (lane == 0) pre[0] = 0u;
        total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 31);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // pair f of the wavefront -> (token in block, entry): the token is the last k with pre[k] <= f
    auto locate = [&](uint32_t f, int& tl, uint32_t& pr) {
        int k = 0;
#pragma unroll
        for (int sft = 16; sft >= 1; sft >>= 1)
            if (pre[k + sft] <= f) k += sft;
        tl = tl0 + k;
        pr = pairs[(size_t)s_beg[tl] + (f - pre[k])];
    };
    uint32_t cur[kPChains], meta[kPChains];             // meta = token in block | row in tile << 8 | min(len, 255) << 16 | scratch byte << 24
    int nch = (int)min((total + 63u) / 64u, (uint32_t)kPChains);   // chains in use (uniform)
#pragma unroll
    for (int c = 0; c < kPChains; ++c) {
        const uint32_t f = 64u * c + (uint32_t)lane;
        cur[c] = SINK;
        meta[c] = 0;
        if (c < nch && f < total) {
            int tl;
            uint32_t pr;
            locate(f, tl, pr);
            cur[c] = (pr & 0xFFFFFFu) << 1;
            meta[c] = (uint32_t)tl | ((pr >> 24) << 8) | (min(s_len[tl], 255u) << 16);
        }
    }
    const char* tt_bytes = reinterpret_cast<const char*>(tt);
    const uint32_t col_bytes = q_stride * 2u;
    // A level first asks the bit table (80 bytes per column and 640 states: it stays in the caches)
    // whether the edge exists, and fetches the target from the full transposed table only if it
    // does; most pairs die at each level, and their lookups never leave the L2.  After a level the
    // pairs that are still alive (walking, or done with their token) are packed into the lowest
    // chains through this wavefront's share of the tile's LDS, which nothing else uses before the
    // turns: the work of a level follows the number of live pairs, not the number of chains.
    const uint32_t* __restrict__ live_bits = d.live_bits;
    const uint32_t col_words = q_stride >> 5;
    constexpr int kPackCap = (int)(kPairTileBytes / kPWaves / 8);        // pairs a wavefront's share holds
    uint2* pack = reinterpret_cast<uint2*>(smem) + wave * kPackCap;
    for (uint32_t i = 2; i < 32u; ++i) {
        bool any = false;
#pragma unroll
        for (int c = 0; c < kPChains; ++c)
            if (c < nch) any |= cur[c] != SINK && i < ((meta[c] >> 16) & 0xFFu);
        if (__builtin_amdgcn_ballot_w64(any) == 0) break;
        // eight chains at a time: their bit words first, then the targets of those that live
#pragma unroll
        for (int c0 = 0; c0 < kPChains; c0 += 8) {
            if (c0 >= nch) break;
            uint32_t bw[8];                               // the level's byte goes to the top byte of meta
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = c0 + j;
                bw[j] = 0;
                if (c < nch) {
                    const bool go = cur[c] != SINK && i < ((meta[c] >> 16) & 0xFFu);
                    if (go) {
                        const uint32_t b = reinterpret_cast<const uint8_t*>(s_bytes)[(meta[c] & 0xFFu) * 32u + i];
                        meta[c] = (meta[c] & 0x00FFFFFFu) | (b << 24);
                        bw[j] = live_bits[b * col_words + (cur[c] >> 6)];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = c0 + j;
                if (c < nch) {
                    const bool go = cur[c] != SINK && i < ((meta[c] >> 16) & 0xFFu);
                    if (go) {
                        const bool live = (bw[j] >> ((cur[c] >> 1) & 31u)) & 1u;
                        uint32_t nx = SINK;
                        if (live) nx = *reinterpret_cast<const uint16_t*>(tt_bytes + (uint32_t)((meta[c] >> 24) * col_bytes + cur[c]));
                        cur[c] = nx;
                    }
                }
            }
        }
        // pack the live pairs
        uint32_t n_alive = 0;
#pragma unroll
        for (int c = 0; c < kPChains; ++c)
            if (c < nch) n_alive += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(cur[c] != SINK));
        const int packed = (int)((n_alive + 63u) / 64u);
        if (packed < nch && n_alive <= (uint32_t)kPackCap) {
            uint32_t at = 0;
#pragma unroll
            for (int c = 0; c < kPChains; ++c) {
                if (c < nch) {
                    const unsigned long long bal = __builtin_amdgcn_ballot_w64(cur[c] != SINK);
                    if (cur[c] != SINK)
                        pack[at + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u))] =
                            make_uint2(cur[c], meta[c]);
                    at += (uint32_t)__popcll(bal);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int c = 0; c < kPChains; ++c) {
                if (c < nch) {
                    cur[c] = SINK;
                    if (c < packed && 64u * c + (uint32_t)lane < n_alive) {
                        const uint2 en = pack[64 * c + lane];
                        cur[c] = en.x;
                        meta[c] = en.y;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            nch = packed;
        }
    }
    // tokens longer than the 32 bytes kept in LDS: the rest of their bytes come from the vocabulary
#pragma unroll 1
    for (int c = 0; c < kPChains; ++c) {
        if (c >= nch) continue;
        if (__builtin_amdgcn_ballot_w64(cur[c] != SINK && ((meta[c] >> 16) & 0xFFu) > 32u) == 0) continue;
        const int tl = (int)(meta[c] & 0xFFu);
        const uint32_t len = s_len[tl];
        const uint8_t* bytes = reinterpret_cast<const uint8_t*>(v.vwords) + (size_t)v.voff[min(t_block + tl, n_tokens - 1)] * 4;
        for (uint32_t i = 32;; ++i) {
            const bool go = cur[c] != SINK && i < len && ((meta[c] >> 16) & 0xFFu) > 32u;
            if (__builtin_amdgcn_ballot_w64(go) == 0) break;
            if (go) cur[c] = *reinterpret_cast<const uint16_t*>(tt_bytes + (uint32_t)((uint32_t)bytes[i] * col_bytes + cur[c]));
        }
    }

    __syncthreads();
    {
        uint32_t* w = reinterpret_cast<uint32_t*>(tile);
        for (int i = threadIdx.x; i < (int)(kPairTileBytes / 4); i += kPThreads) w[i] = 0u;     // entries are state + 1; 0 = DEAD
        for (int i = threadIdx.x; i < kPS * 8; i += kPThreads) s_bits[i] = 0u;
    }
    __syncthreads();

    // ---- four turns
    for (int sub = 0; sub < kPSub; ++sub) {
        const int t0 = t_block + sub * kPT;
        if (t0 >= n_tokens) break;                      // uniform; the bits of the remaining sub-tiles stay zero
        if ((wave >> 1) == sub) {
            const int col0 = sub * kPT;                 // the sub-tile's first token, in block-local numbering
#pragma unroll
            for (int c = 0; c < kPChains; ++c)
                if (c < nch && cur[c] != SINK) tile[((meta[c] >> 8) & 0xFFu) * kPRS + ((meta[c] & 0xFFu) - col0)] = (uint16_t)((cur[c] >> 1) + 1u);
            // pairs beyond the register chains (a wavefront with more than 64 * kPChains pairs)
            for (uint32_t f0 = 64u * kPChains; f0 < total; f0 += 64u) {
                const uint32_t f = f0 + (uint32_t)lane;
                uint32_t x = SINK, ql = 0, len = 0;
                int tl = tl0;
                if (f < total) {
                    uint32_t pr;
                    locate(f, tl, pr);
                    x = (pr & 0xFFFFFFu) << 1;
                    ql = pr >> 24;
                    len = s_len[tl];
                }
                const uint8_t* bytes = reinterpret_cast<const uint8_t*>(v.vwords) + (size_t)v.voff[min(t_block + tl, n_tokens - 1)] * 4;
                for (uint32_t i = 2;; ++i) {
                    const bool go = x != SINK && i < len;
                    if (__builtin_amdgcn_ballot_w64(go) == 0) break;
                    if (go) x = *reinterpret_cast<const uint16_t*>(tt_bytes + (uint32_t)((uint32_t)bytes[i] * col_bytes + x));
                }
                if (x != SINK) tile[ql * kPRS + (tl - col0)] = (uint16_t)((x >> 1) + 1u);
            }
            // one-byte tokens: the column of the byte, lanes = states
            unsigned long long ones = __builtin_amdgcn_ballot_w64(lane < 32 && s_len[tl0 + (lane & 31)] == 1u);
            while (ones) {
                const int k = __builtin_ctzll(ones);
                ones &= ones - 1;
                const int tl = tl0 + k;
                const uint32_t b1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_bytes[tl * 8]) & 0xFFu;
                const uint16_t* col = tt + (size_t)b1 * q_stride;
#pragma unroll
                for (int g = 0; g < kPS / 64; ++g) {
                    const int q = s_state[g * 64 + lane];
                    if (q >= 0) {
                        const uint32_t e = col[q];
                        if (e != SINK) tile[(g * 64 + lane) * kPRS + (tl - col0)] = (uint16_t)((e >> 1) + 1u);
                    }
                }
            }
        }
        __syncthreads();

        // ---- flush the sub-tile's rows and put DEAD back; its allowed bits go to s_bits
        if (WIDE_ROWS) {
            constexpr int LPR = kPT / 4, RPW = 64 / LPR;     // 16 lanes per row, 4 rows per wavefront pass
            const int subr = lane / LPR, l = lane % LPR;
            const int t = t0 + 4 * l;
            const int lane_off = subr * kPRS + 4 * l;
            const int base1 = state_base - 1;
            for (int r0 = wave * RPW; r0 < kPS; r0 += kPWaves * RPW) {
                const int q = s_state[r0 + subr];
                uint32_t* tw = reinterpret_cast<uint32_t*>(tile + r0 * kPRS + lane_off);
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
                if (q >= 0 && t < n_tokens) {
                    typedef int i32x4 __attribute__((ext_vector_type(4)));
                    const i32x4 pack4 = {val[0], val[1], val[2], val[3]};
                    __builtin_nontemporal_store(pack4, reinterpret_cast<i32x4*>(delta + ((uint64_t)(out_row32 + (uint32_t)q) * nt32 + (uint32_t)t)));
                }
                bits <<= 4 * (l & 7);
                bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
                bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
                bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x141, 0xF, 0xF, true);   // row_half_mirror
                if ((l & 7) == 0) s_bits[(r0 + subr) * 8 + sub * 2 + (l >> 3)] = bits;
            }
        } else {
            for (int r = wave; r < kPS; r += kPWaves) {
                const int q = __builtin_amdgcn_readfirstlane(s_state[r]);
                const int t = t0 + lane;
                const uint32_t e = tile[r * kPRS + lane];
                tile[r * kPRS + lane] = (uint16_t)0;
                const int val = e ? (int)e - 1 + state_base : TDFA_DEAD;
                if (q >= 0 && t < n_tokens) delta[(size_t)(d.out_row + q) * n_tokens + t] = val;
                const uint64_t m = __builtin_amdgcn_ballot_w64(val >= 0);
                if (lane < 2) s_bits[r * 8 + sub * 2 + lane] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
            }
        }
        __syncthreads();
    }
    // ---- the allowed bits of the block's 256 tokens: eight words per row, written as two 16-byte halves
    {
        const int r = (int)threadIdx.x >> 1, half = (int)threadIdx.x & 1;
        const int q = s_state[r];
        const uint32_t word0 = (uint32_t)bt * 8u + (uint32_t)half * 4u;
        if (q >= 0 && word0 < rw32) {                 // a row is a multiple of four words
            uint32_t* dst = allow + ((uint64_t)(out_row32 + (uint32_t)q) * rw32 + word0);
            const uint32_t* src = s_bits + r * 8 + half * 4;
            if (allow_vec) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(src[0], src[1], src[2], src[3]);
            } else {
                dst[0] = src[0]; dst[1] = src[1]; dst[2] = src[2]; dst[3] = src[3];
            }
        }
    }
}

}  // namespace

int launch_compile_pairs(const CompileArgs& a, const CompileEntry& e, hipStream_t stream)
{
    if (a.n_tokens <= 0) return TDFA_OK;
    PairDesc d;
    d.tt = static_cast<const uint16_t*>(e.trans_t);
    d.trans = e.trans;
    d.rows16 = e.pair_rows16;
    d.live_bits = e.pair_live_bits;
    d.order = e.order;
    d.idx = e.pair_idx;
    d.block_tot = e.pair_block_tot;
    d.pairs = e.pair_list;
    d.n_states = e.n_states;
    d.n_order = e.n_order;
    d.q_stride = e.q_stride;
    d.n_tiles_q = (e.n_order + kPS - 1) / kPS;
    d.out_row = e.out_row;
    d.state_base = e.state_base;
    int rc = launch_transpose(&e, 1, stream);
    if (rc != TDFA_OK) return rc;
    const int64_t n_entries = (int64_t)e.n_states * 256;
    narrow_rows_kernel<<<(unsigned)((n_entries + 255) / 256), 256, 0, stream>>>(d);
    TDFA_HIP(hipGetLastError());
    live_bits_kernel<<<(unsigned)((256 * (e.q_stride / 32) + 255) / 256), 256, 0, stream>>>(d);
    TDFA_HIP(hipGetLastError());
    const unsigned n_blocks = (unsigned)d.n_tiles_q * 256u;
    pair_count_kernel<<<n_blocks, 256, 0, stream>>>(d);
    TDFA_HIP(hipGetLastError());
    pair_scan_kernel<<<1, 1024, 0, stream>>>(d);
    TDFA_HIP(hipGetLastError());
    pair_fill_kernel<<<n_blocks, 256, 0, stream>>>(d);
    TDFA_HIP(hipGetLastError());

    PairVocab v;
    v.vwords = a.vwords;
    v.voff = a.voff;
    v.vlen = a.vlen;
    v.vprefix = a.vprefix;
    v.n_tokens = a.n_tokens;
    const int64_t n_blocks_t = (a.n_tokens + kPBlockT - 1) / kPBlockT;
    const int64_t grid = n_blocks_t * d.n_tiles_q;
    if (grid > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "table too large for one launch");
    const bool wide_rows = a.n_tokens % 4 == 0 && reinterpret_cast<uintptr_t>(a.delta) % 16 == 0;
    const int allow_vec = reinterpret_cast<uintptr_t>(a.allow) % 16 == 0 ? 1 : 0;
    const bool base0 = e.state_base == 0;
    auto kern = wide_rows ? (base0 ? pair_tile_kernel<true, true> : pair_tile_kernel<true, false>)
                          : (base0 ? pair_tile_kernel<false, true> : pair_tile_kernel<false, false>);
    static bool attr_set = false;
    if (!attr_set) {
        for (auto k : {pair_tile_kernel<true, true>, pair_tile_kernel<true, false>, pair_tile_kernel<false, true>, pair_tile_kernel<false, false>})
            TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPairLdsBytes));
        attr_set = true;
    }
    kern<<<(unsigned)grid, kPThreads, kPairLdsBytes, stream>>>(d, v, (int)n_blocks_t, a.delta, a.allow, a.row_words, allow_vec);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace tdfa
