// Compile stage: the token-level table delta_T of A_R o T_V (Sections 2.3-2.4; Algorithm 2,
// statement 3) and its allowed-bit rows, for gfx950.
//
// With a deterministic A_R, composing with T_V (Algorithm 1) and removing epsilon edges gives
// delta_T[q][t] = delta*(q, d(t)): walk the bytes of token t from state q, DEAD at the first
// missing transition (Theorems 1 and 2).  Every (q, t) entry is independent and costs 4 bytes of
// output plus one table lookup per byte walked; the kernels are built so that a lookup is one
// memory instruction and nothing else:
//
//   1. transpose_kernel: delta[q][b] (int32, as uploaded) -> delta^T[b][q] in "offset form": the
//      entry is the byte offset of the target state inside a column (state * element size), 16-bit
//      when that fits.  DEAD becomes the offset of a sink state appended after the real ones
//      (the largest entry there is, so "some lane alive" is one min and one compare).  One byte's
//      column is contiguous: every step of a walk gathers inside one column (2|Q| bytes), addressed
//      as scalar column base + the lane's current entry, with no address arithmetic.
//   2. start_bytes_kernel: one byte per (64-state group, token) that says how the pair starts:
//      nothing to do, an ordinary first lookup, or a jump over the token's clean prefix (the
//      default-chain tables of plan.hip).
//   3. compile_tile_kernel: a workgroup owns S states x T consecutive token ids; the tile lives in
//      LDS.  Its phases are described at the kernel.
#include <algorithm>

#include "tdfa_internal.h"

namespace tdfa {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBatch = 48;

// Up to kMaxBatch automata per launch, described by value in the kernel arguments.
struct DfaDesc {
    const int32_t* trans;     // [n_states][256] as uploaded
    void* tt;                 // [256][q_stride] transposed table in offset form
    const int32_t* order;     // [n_order] states in lane order, -1 = idle lane
    const unsigned char* plan;  // clean sets, group classes, group live sets, jump tables
    uint8_t* start_bytes;     // [ceil(n_order / 64)][n_tokens] workspace, or NULL
    int32_t n_states;
    int32_t q_stride;
    int32_t tile_q_begin;     // first state tile of this automaton in the launch
    int32_t out_row;          // row of the output buffers where this automaton's rows start
    int32_t state_base;       // added to every live entry
    int32_t n_order;
};
struct BatchDesc {
    int32_t n;
    int32_t n_tiles_q;        // state tiles of all automata together
    DfaDesc d[kMaxBatch];
};

// delta[q][b] -> out[b][q] in offset form; rows q in [n_states, q_stride) are sink rows.
template <typename ST>
__global__ void __launch_bounds__(kThreads)
transpose_kernel(BatchDesc batch)
{
    __shared__ int32_t tile[64][65];
    const DfaDesc& d = batch.d[blockIdx.z];
    const int n_states = d.n_states, q_stride = d.q_stride;
    const int q0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
    if (q0 >= q_stride) return;
    const int32_t* __restrict__ trans = d.trans;
    ST* __restrict__ out = static_cast<ST*>(d.tt);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sink = q_stride - 1;
    for (int r = wave; r < 64; r += kWaves) {
        const int q = q0 + r;
        const int t = q < n_states ? trans[(size_t)q * 256 + b0 + lane] : TDFA_DEAD;
        tile[r][lane] = t < 0 ? sink : t;
    }
    __syncthreads();
    for (int c = wave; c < 64; c += kWaves) {
        const int q = q0 + lane;
        if (q < q_stride) out[(size_t)(b0 + c) * q_stride + q] = (ST)(tile[lane][c] * (int)sizeof(ST));
    }
}

// What every (64-state group, token) pair starts with, one byte each:
//   0xFF  no state of the group survives the token's first byte (or the token is empty): nothing
//         to look up, the whole group x token block stays DEAD
//   m>=1  the group is of a jump class and the token begins with m clean bytes of that class (at
//         most kJumpDepth): one lookup in the jump table takes all m bytes
//   0     an ordinary lookup of the first byte
// One thread per token and chunk of kStartChunk groups; the groups of an automaton are listed class
// by class, so the clean prefix is recomputed only where the class changes.
constexpr int kStartChunk = 16;

__global__ void __launch_bounds__(kThreads)
start_bytes_kernel(BatchDesc batch, const uint32_t* __restrict__ vprefix, const uint32_t* __restrict__ vlen, int n_tokens)
{
    __shared__ uint32_t s_set[kMaxJumpClasses * 8];
    __shared__ uint32_t s_live[kStartChunk * 8];
    __shared__ int s_class[kStartChunk];
    const DfaDesc& d = batch.d[blockIdx.y];
    uint8_t* __restrict__ out = d.start_bytes;
    const int n_groups = (d.n_order + 63) / 64;
    const int g_lo = blockIdx.z * kStartChunk, g_hi = min(n_groups, g_lo + kStartChunk);
    if (!out || g_lo >= n_groups) return;
    const int8_t* __restrict__ group_class = reinterpret_cast<const int8_t*>(d.plan + kPlanSetBytes);
    const uint32_t* __restrict__ group_live = reinterpret_cast<const uint32_t*>(d.plan + plan_live_offset(d.n_order));
    if (threadIdx.x < kMaxJumpClasses * 8) s_set[threadIdx.x] = reinterpret_cast<const uint32_t*>(d.plan)[threadIdx.x];
    if (threadIdx.x < (g_hi - g_lo) * 8) s_live[threadIdx.x] = group_live[g_lo * 8 + threadIdx.x];
    if (threadIdx.x < g_hi - g_lo) s_class[threadIdx.x] = group_class[g_lo + threadIdx.x];
    __syncthreads();
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_tokens) return;
    const uint32_t len = vlen[t];
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = vprefix[(size_t)t * 8 + k];
    const uint32_t b1 = w[0] & 0xFFu;
    int cur_class = -1;
    uint32_t m = 0;
    for (int g = g_lo; g < g_hi; ++g) {
        const int c = s_class[g - g_lo];
        if (c != cur_class) {
            cur_class = c;
            m = 0;
            if (c >= 0) {
                const uint32_t n = min(len, (uint32_t)kJumpDepth);
                while (m < n) {
                    uint32_t word = w[0];
#pragma unroll
                    for (int k = 1; k < 8; ++k) word = (m >> 2) == (uint32_t)k ? w[k] : word;
                    const uint32_t b = (word >> ((m & 3u) * 8)) & 0xFFu;
                    if (!((s_set[c * 8 + (b >> 5)] >> (b & 31u)) & 1u)) break;
                    ++m;
                }
            }
        }
        const bool live = len != 0 && ((s_live[(g - g_lo) * 8 + (b1 >> 5)] >> (b1 & 31u)) & 1u);
        out[(size_t)g * n_tokens + t] = (uint8_t)(m != 0 ? m : live ? 0u : 0xFFu);
    }
}

// One workgroup owns S states x T consecutive token ids.  The S states are consecutive entries of
// `order`: first the states of the jump classes, class by class in whole groups of 64, then the
// others listed so that states with about as many live bytes are neighbours; the 64 lanes of a
// group then tend to live and die together.
//   phase 0  tile <- sink; one round of loads brings the tile's states, group classes, token
//            lengths, word offsets, first 32 bytes, sorted order and start bytes to LDS
//   phase 1  walks: a wavefront takes KT tokens at a time, lanes = 64 consecutive states, S/64
//            state groups per token.  Per byte and group the work is one gather (column base in
//            scalar registers + the lane's entry) under the mask of live lanes; a group with no
//            live lane issues nothing.  The KT * S/64 chains of a wavefront are independent and
//            their loads are in flight together; the walk stops as soon as no lane of a token
//            with bytes left is alive.  Only live results go to the tile.  Tiles without a jump
//            group and tiles with one run different loops (see there).
//   phase 2  rows are flushed: a lane converts four consecutive entries and writes 16 bytes, the
//            allowed bits of eight lanes are merged into one word (rows that cannot be written
//            16 bytes at a time: one entry per lane and a wave ballot)
constexpr int kTileThreads = 1024;             // largest workgroup of the tile kernel
constexpr int kLdsWords = 8;    // words of each token kept in LDS (32 bytes)
constexpr int kXcds = 8;        // accelerator dies of the MI355X
constexpr int kSortBlock = 64;  // tokens per block of the vocabulary's blocked trie order (= tdfa::kVocabSortBlock)

template <typename ST, int S, int T>
struct TileShape {
    static constexpr int RS = T + (sizeof(ST) == 2 ? 2 : 1);   // odd number of 32-bit words per row
    static constexpr size_t tile_bytes = (size_t)S * RS * sizeof(ST);
    static constexpr int CW = (S / 64 + 3) / 4;                 // words of clean-prefix lengths per token
    static constexpr size_t meta_bytes = (size_t)(3 + kLdsWords + CW) * T * 4 + (size_t)S * 4 + S / 64 * 4;
    static constexpr size_t lds_bytes = tile_bytes + meta_bytes;
};
constexpr int kNear = kLdsWords * 4;     // bytes of a token that a wavefront holds one per lane

template <typename ST>
__device__ __forceinline__ uint32_t gather(const ST* col, uint32_t byte_off)
{
    return *reinterpret_cast<const ST*>(reinterpret_cast<const char*>(col) + byte_off);
}

// STAGED: the automaton's whole transposed table ([256][q_stride], at most kStagedTableBytes) is
// copied into LDS behind the tile before the walk, and every lookup of the walk is an LDS read.
template <typename ST, int S, int T, int KT, bool HAS_JUMP, int kTileWaves, bool STAGED = false>
__global__ void __launch_bounds__(kTileWaves * 64)
compile_tile_kernel(BatchDesc batch,
                    const uint32_t* __restrict__ vwords, const uint32_t* __restrict__ voff,
                    const uint32_t* __restrict__ vlen, const uint8_t* __restrict__ vsorted,
                    const uint32_t* __restrict__ vprefix, int n_tokens,
                    int n_tiles_t, int share_columns, int wide_rows, int32_t* __restrict__ delta, uint32_t* __restrict__ allow,
                    int64_t row_words)
{
    static_assert(S % 64 == 0 && T % kSortBlock == 0 && T % (kTileWaves * KT) == 0, "tile shape");
    constexpr int kTileThreads = kTileWaves * 64;
    using Shape = TileShape<ST, S, T>;
    constexpr int RS = Shape::RS;
    constexpr int G = S / 64;
    extern __shared__ __align__(16) unsigned char smem[];
    ST* tile = reinterpret_cast<ST*>(smem);
    uint32_t* s_len = reinterpret_cast<uint32_t*>(smem + Shape::tile_bytes);
    uint32_t* s_off = s_len + T;
    uint32_t* s_bytes = s_off + T;                 // [T][kLdsWords]
    int32_t* s_state = reinterpret_cast<int32_t*>(s_bytes + T * kLdsWords);   // [S] state of each tile row, -1 past the end
    uint32_t* s_sorted = reinterpret_cast<uint32_t*>(s_state + S);              // [T] block-local token index by sorted position
    uint32_t* s_clean = s_sorted + T;              // [T][CW] one byte per state group: length of the token's clean prefix
    int32_t* s_gc = reinterpret_cast<int32_t*>(s_clean + T * Shape::CW);   // [G] jump class of each state group, -1 = none

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Two orders of the tiles.  Token-major (table small enough to sit in every L2): consecutive
    // workgroups write neighbouring pieces of the same rows.  Column-sharing (large tables):
    // workgroups go round-robin to the 8 XCDs, each with an L2 of its own; XCD x takes the token
    // tiles x, x + 8, ... and runs through all state tiles of one token tile before the next, so
    // the workgroups that share an L2 at any moment walk the same tokens, i.e. the same columns
    // of the transposed table.  The grid is padded to a multiple of 8 token tiles for that.
    const int n_tiles_q = batch.n_tiles_q;
    int tile_t, tile_q;
    if (share_columns) {
        const int xcd = blockIdx.x % kXcds, seq = blockIdx.x / kXcds;
        tile_t = (seq / n_tiles_q) * kXcds + xcd;
        tile_q = seq % n_tiles_q;
        if (tile_t >= n_tiles_t) return;
    } else {
        // Of every 32 consecutive workgroups the four that go to one XCD take four neighbouring
        // token tiles, so the pieces of a row (and of a 32-byte sector of allowed bits) that are
        // written at about the same time meet in one L2.
        const unsigned r = blockIdx.x & 31u;
        const unsigned b = (blockIdx.x & ~31u) + (r & 7u) * 4u + (r >> 3);
        tile_t = (int)(b % (unsigned)n_tiles_t);
        tile_q = (int)(b / (unsigned)n_tiles_t);
        if (tile_q >= n_tiles_q) return;              // the grid is padded to a multiple of 32
    }
    // which automaton of the launch this state tile belongs to
    int di = 0;
    while (di + 1 < batch.n && tile_q >= batch.d[di + 1].tile_q_begin) ++di;
    const DfaDesc& dd = batch.d[di];
    const ST* s_tt = reinterpret_cast<const ST*>(smem + Shape::lds_bytes);        // STAGED: [256][q_stride]
    const ST* __restrict__ tt = STAGED ? s_tt : static_cast<const ST*>(dd.tt);
    const int32_t* __restrict__ order = dd.order;
    const int n_order = dd.n_order, q_stride = dd.q_stride, state_base = dd.state_base;
    const int8_t* __restrict__ group_class = reinterpret_cast<const int8_t*>(dd.plan + kPlanSetBytes);
    const uint8_t* __restrict__ start_bytes = dd.start_bytes;
    const ST* __restrict__ jt = reinterpret_cast<const ST*>(dd.plan + plan_jump_offset(n_order));
    const int64_t out_row = dd.out_row;
    const int t0 = tile_t * T, q0 = (tile_q - dd.tile_q_begin) * S;
    const uint32_t SINK = (uint32_t)(q_stride - 1) * (uint32_t)sizeof(ST);   // the largest entry there is

    // ---- phase 0
    if constexpr (STAGED) {
        // 16 bytes per thread and pass (q_stride is a multiple of 64 entries)
        const uint4* src = static_cast<const uint4*>(dd.tt);
        uint4* dst = reinterpret_cast<uint4*>(smem + Shape::lds_bytes);
        const int n16 = (int)((size_t)256 * dd.q_stride * sizeof(ST) / 16);
        for (int i = threadIdx.x; i < n16; i += kTileThreads) dst[i] = src[i];
    }
    {
        uint32_t* w = reinterpret_cast<uint32_t*>(smem);
        constexpr int n_words = (int)(Shape::tile_bytes / 4);
        const uint32_t fill = sizeof(ST) == 2 ? (SINK | (SINK << 16)) : SINK;
        for (int i = threadIdx.x; i < n_words; i += kTileThreads) w[i] = fill;
        for (int r = threadIdx.x; r < S; r += kTileThreads) s_state[r] = q0 + r < n_order ? order[q0 + r] : -1;
        if (threadIdx.x < G) s_gc[threadIdx.x] = q0 + (int)threadIdx.x * 64 < n_order ? (int)group_class[q0 / 64 + threadIdx.x] : -1;
        // what each (token, group) pair starts with (see start_bytes_kernel); without the workspace
        // every group looks up every non-empty token's first byte
        for (int i = threadIdx.x; i < T * G; i += kTileThreads) {
            const int g = i / T, tl = i % T, t = t0 + tl;
            unsigned char sb = 0xFF;
            if (t < n_tokens && q0 + g * 64 < n_order)
                sb = start_bytes ? start_bytes[(size_t)(q0 / 64 + g) * n_tokens + t] : (vlen[t] ? 0 : 0xFF);
            reinterpret_cast<unsigned char*>(s_clean)[tl * (Shape::CW * 4) + g] = sb;
        }
        for (int tl = threadIdx.x; tl < T; tl += kTileThreads) {
            const int t = t0 + tl;
            s_sorted[tl] = t < n_tokens ? (uint32_t)vsorted[t] : (uint32_t)(tl & (kSortBlock - 1));
            s_len[tl] = t < n_tokens ? vlen[t] : 0u;
            s_off[tl] = t < n_tokens ? voff[t] : 0u;
        }
        static_assert(kLdsWords == 8, "the vocabulary's prefix array holds 8 words per token");
        for (int i = threadIdx.x; i < T * kLdsWords; i += kTileThreads)
            s_bytes[i] = t0 + i / kLdsWords < n_tokens ? vprefix[(size_t)t0 * kLdsWords + i] : 0u;
    }
    __syncthreads();
    int gc[G];
    bool any_jump = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        gc[g] = __builtin_amdgcn_readfirstlane(s_gc[g]);
        any_jump |= gc[g] >= 0;
    }
    if (!HAS_JUMP) any_jump = false;                 // no automaton of the launch has a jump class

    // ---- phase 1
    uint32_t start[G];                               // this lane's states, as offsets into a column
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int q = s_state[g * 64 + lane];
        start[g] = q < 0 ? SINK : (uint32_t)q * (uint32_t)sizeof(ST);
    }
    // The tokens of every block of kSortBlock ids are visited in byte-lexicographic (prefix trie)
    // order: `sorted` lists each block's tokens that way.  A wavefront owns KT runs of
    // consecutive sorted tokens and walks the KT runs side by side.
    constexpr int kRun = T / (kTileWaves * KT);
    auto token_byte = [&](uint32_t byte_lane, uint32_t off, uint32_t i) -> uint32_t {
        // lane i holds byte i of the token (its first kNear bytes): a step gets its byte with one
        // v_readlane instead of an LDS read, a wait and shifts
        return i < (uint32_t)kNear ? (uint32_t)__builtin_amdgcn_readlane(byte_lane, i)
                                   : (__builtin_amdgcn_readfirstlane(vwords[off + (i >> 2)]) >> ((i & 3u) * 8)) & 0xFFu;
    };
    if (!any_jump) {
        // Plain tiles.  When the next token of a run starts with the same byte as the one before
        // it, the states after that byte are reused.
        uint32_t prev_b1[KT];
        uint32_t first[KT][G];                       // states after the first byte of the run's previous token
#pragma unroll
        for (int u = 0; u < KT; ++u) prev_b1[u] = 0xFFFFFFFFu;
        for (int step = 0; step < kRun; ++step) {
            if constexpr (KT == 1 && G == 4) {
                // no state of the tile survives this token's first byte: nothing to do
                const int k = wave * kRun + step;
                const int tl = (k & ~(kSortBlock - 1)) + (int)__builtin_amdgcn_readfirstlane(s_sorted[k]);
                if (__builtin_amdgcn_readfirstlane(s_clean[tl]) == 0xFFFFFFFFu) continue;
            }
            uint32_t len[KT], off[KT], byte_lane[KT];
            int tls[KT];
            uint32_t v[KT][G];
            uint32_t max_len = 0;
#pragma unroll
            for (int u = 0; u < KT; ++u) {
                const int k = (wave * KT + u) * kRun + step;                    // position in sorted order
                const int tl = (k & ~(kSortBlock - 1)) + (int)__builtin_amdgcn_readfirstlane(s_sorted[k]);
                tls[u] = tl;
                len[u] = __builtin_amdgcn_readfirstlane(s_len[tl]);
                off[u] = __builtin_amdgcn_readfirstlane(s_off[tl]);
                max_len = max(max_len, len[u]);
                byte_lane[u] = (s_bytes[tl * kLdsWords + ((lane & (kNear - 1)) >> 2)] >> ((lane & 3) * 8)) & 0xFFu;
                const uint32_t b1 = len[u] ? (uint32_t)__builtin_amdgcn_readlane(byte_lane[u], 0) : 0xFFFFFFFEu;
                if (b1 != prev_b1[u]) {
                    uint32_t cw[Shape::CW];
#pragma unroll
                    for (int j = 0; j < Shape::CW; ++j) cw[j] = __builtin_amdgcn_readfirstlane(s_clean[tl * Shape::CW + j]);
                    const ST* col = tt + (b1 & 0xFFu) * (uint32_t)q_stride;
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        // nothing to look up for a group that no state of survives this byte
                        const uint32_t live_below = ((cw[g >> 2] >> ((g & 3) * 8)) & 0xFFu) == 0xFFu ? 0u : SINK;
                        first[u][g] = SINK;
                        if (start[g] < live_below) first[u][g] = gather(col, start[g]);
                    }
                    prev_b1[u] = b1;
                }
            }
            // (the lookups of all KT tokens are issued before any result is used)
#pragma unroll
            for (int u = 0; u < KT; ++u)
#pragma unroll
                for (int g = 0; g < G; ++g) v[u][g] = first[u][g];
            for (uint32_t i = 1; i < max_len; ++i) {
#pragma unroll
                for (int u = 0; u < KT; ++u) {
                    if (i < len[u]) {
                        const ST* col = tt + token_byte(byte_lane[u], off[u], i) * (uint32_t)q_stride;
#pragma unroll
                        for (int g = 0; g < G; ++g)
                            if (v[u][g] != SINK) v[u][g] = gather(col, v[u][g]);
                    }
                }
                uint32_t lowest = SINK;              // below SINK iff a lane of a token with bytes left is alive
#pragma unroll
                for (int u = 0; u < KT; ++u) {
                    if (i + 1 < len[u]) {
#pragma unroll
                        for (int g = 0; g < G; ++g) lowest = min(lowest, v[u][g]);
                    }
                }
                if (__builtin_amdgcn_ballot_w64(lowest < SINK) == 0) break;
            }
#pragma unroll
            for (int u = 0; u < KT; ++u)
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (v[u][g] != SINK) tile[(g * 64 + lane) * RS + tls[u]] = (ST)v[u][g];
        }
    } else {
        // Tiles with groups of a jump class.  Such a group takes the token's clean prefix (m bytes)
        // in one lookup in the jump table and joins the byte-by-byte walk at byte m; the other
        // groups, and a jump group whose token starts with a byte that is not clean, start with
        // an ordinary lookup of the first byte.  All conditions that differ between groups are
        // folded into scalar operands (a base pointer, a threshold), so the G lookups of a step
        // are issued back to back like in a plain tile.
        for (int step = 0; step < kRun; ++step) {
            if constexpr (KT == 1 && G == 4) {
                // The two common cases, each decided by one comparison of the four start bytes:
                // no group has anything to do, or all four take the whole token in one jump.
                const int k = wave * kRun + step;
                const int tl = (k & ~(kSortBlock - 1)) + (int)__builtin_amdgcn_readfirstlane(s_sorted[k]);
                const uint32_t n = __builtin_amdgcn_readfirstlane(s_len[tl]);
                const uint32_t w = __builtin_amdgcn_readfirstlane(s_clean[tl]);
                if (w == 0xFFFFFFFFu) continue;
                if (n <= (uint32_t)kJumpDepth && w == n * 0x01010101u) {
                    const ST* base = jt + (n - 1) * (uint32_t)q_stride;
                    uint32_t x[G];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        x[g] = SINK;
                        if (start[g] != SINK) x[g] = gather(base, start[g]);
                    }
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        if (x[g] != SINK) tile[(g * 64 + lane) * RS + tl] = (ST)x[g];
                    continue;
                }
            }
            uint32_t len[KT], off[KT], byte_lane[KT];
            int tls[KT];
            uint32_t v[KT][G];
            uint32_t cw[KT][Shape::CW];              // per group one byte: how many bytes of the token v[u][g] has taken
            uint32_t max_len = 0, first_step = 0xFFFFFFFFu;
#pragma unroll
            for (int u = 0; u < KT; ++u) {
                const int k = (wave * KT + u) * kRun + step;
                const int tl = (k & ~(kSortBlock - 1)) + (int)__builtin_amdgcn_readfirstlane(s_sorted[k]);
                tls[u] = tl;
                len[u] = __builtin_amdgcn_readfirstlane(s_len[tl]);
                off[u] = __builtin_amdgcn_readfirstlane(s_off[tl]);
#pragma unroll
                for (int j = 0; j < Shape::CW; ++j) cw[u][j] = __builtin_amdgcn_readfirstlane(s_clean[tl * Shape::CW + j]);
                max_len = max(max_len, len[u]);
                byte_lane[u] = (s_bytes[tl * kLdsWords + ((lane & (kNear - 1)) >> 2)] >> ((lane & 3) * 8)) & 0xFFu;
                const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane(byte_lane[u], 0);
                const ST* col1 = tt + b1 * (uint32_t)q_stride;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const uint32_t m = (cw[u][g >> 2] >> ((g & 3) * 8)) & 0xFFu;
                    const uint32_t live_below = m == 0xFFu ? 0u : SINK;            // 0xFF: nothing survives the first byte
                    const ST* base = m != 0 && m != 0xFFu ? jt + (m - 1) * (uint32_t)q_stride : col1;
                    v[u][g] = SINK;
                    if (start[g] < live_below) v[u][g] = gather(base, start[g]);
                    if (m == 0) cw[u][g >> 2] += 1u << ((g & 3) * 8);
                    const uint32_t p = max(m, 1u);
                    if (p < len[u]) first_step = min(first_step, p);
                }
            }
            for (uint32_t i = first_step; i < max_len; ++i) {
#pragma unroll
                for (int u = 0; u < KT; ++u) {
                    if (i < len[u]) {
                        const ST* col = tt + token_byte(byte_lane[u], off[u], i) * (uint32_t)q_stride;
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            const uint32_t p = (cw[u][g >> 2] >> ((g & 3) * 8)) & 0xFFu;
                            const uint32_t walking_below = i >= p ? SINK : 0u;       // 0: the group is still ahead of byte i
                            if (v[u][g] < walking_below) v[u][g] = gather(col, v[u][g]);
                        }
                    }
                }
                uint32_t lowest = SINK;
#pragma unroll
                for (int u = 0; u < KT; ++u) {
                    if (i + 1 < len[u]) {
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            const uint32_t p = (cw[u][g >> 2] >> ((g & 3) * 8)) & 0xFFu;
                            const uint32_t done_floor = p < len[u] ? 0u : SINK;   // a group that took the whole token is not waiting for bytes
                            lowest = min(lowest, max(v[u][g], done_floor));
                        }
                    }
                }
                if (__builtin_amdgcn_ballot_w64(lowest < SINK) == 0) break;
            }
#pragma unroll
            for (int u = 0; u < KT; ++u)
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (v[u][g] != SINK) tile[(g * 64 + lane) * RS + tls[u]] = (ST)v[u][g];
        }
    }
    __syncthreads();

    // ---- phase 2
    // Rows whose entries can be written 16 bytes at a time (row length a multiple of 4 tokens and
    // a 16-byte aligned table): a lane converts 4 consecutive entries and stores them at once,
    // T/4 lanes per row, 256/T rows per wavefront pass; the lane's 4 allowed bits are merged with
    // those of its 7 neighbours into one 32-bit word.  The memory pipeline handles a wavefront's
    // store instruction at a cost that hardly depends on its width, so this takes a quarter of
    // the store instructions of the entry-per-lane form below.
    if (wide_rows) {
        constexpr int LPR = T / 4;                   // lanes per row
        constexpr int RPW = 64 / LPR;                // rows per wavefront pass
        const int sub = lane / LPR, l = lane % LPR;
        const int t = t0 + 4 * l;
        // (32-bit operands, so that a row's address costs one multiply-add per buffer)
        const uint32_t out_row32 = (uint32_t)out_row, nt32 = (uint32_t)n_tokens, rw32 = (uint32_t)row_words;
        const uint32_t word = (uint32_t)(t0 >> 5) + (uint32_t)(l >> 3);
        const bool last_tile = tile_t == n_tiles_t - 1;
        const int lane_off = sub * RS + 4 * l;
        for (int r0 = wave * RPW; r0 < S; r0 += kTileWaves * RPW) {
            const int q = s_state[r0 + sub];
            uint32_t e[4];
            if (sizeof(ST) == 2) {
                const uint32_t* tw = reinterpret_cast<const uint32_t*>(tile + r0 * RS + lane_off);
                const uint32_t w0 = tw[0], w1 = tw[1];
                e[0] = w0 & 0xFFFFu, e[1] = w0 >> 16, e[2] = w1 & 0xFFFFu, e[3] = w1 >> 16;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) e[j] = tile[r0 * RS + lane_off + j];
            }
            int v[4];
            uint32_t bits = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[j] = e[j] == SINK ? TDFA_DEAD : (int)(e[j] / (uint32_t)sizeof(ST)) + state_base;
                bits |= (e[j] != SINK ? 1u : 0u) << j;
            }
            const bool row_ok = q >= 0;               // not an idle lane of a padded group, not past the last state
            const uint32_t grow = out_row32 + (uint32_t)q;
            if (row_ok && t < n_tokens) {
                // written once and not read again by this launch: a streaming store, so that the
                // table rows do not push the automaton's columns out of the L2
                typedef int i32x4 __attribute__((ext_vector_type(4)));
                const i32x4 pack = {v[0], v[1], v[2], v[3]};
                __builtin_nontemporal_store(pack, reinterpret_cast<i32x4*>(delta + ((uint64_t)grow * nt32 + (uint32_t)t)));
            }
            bits <<= 4 * (l & 7);
            // OR over the 8 lanes that share a word: neighbours in a quad, then the other quad
            bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
            bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
            bits |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bits, 0x141, 0xF, 0xF, true);   // row_half_mirror
            if (row_ok && (l & 7) == 0 && word < rw32) allow[(uint64_t)grow * rw32 + word] = bits;
            if (last_tile) {
                // a row is a multiple of 4 words: what lies past the last token tile is padding
                const uint32_t pad = (uint32_t)((t0 + T) >> 5) + (uint32_t)l;
                if (row_ok && l < 4 && pad < rw32) allow[(uint64_t)grow * rw32 + pad] = 0u;
            }
        }
        return;
    }
    for (int r = wave; r < S; r += kTileWaves) {
        const int q = __builtin_amdgcn_readfirstlane(s_state[r]);
        if (q < 0) continue;                          // idle lane of a padded group, or past the last state
        int32_t* drow = delta + (size_t)(out_row + q) * n_tokens;
        uint32_t* arow = allow + (size_t)(out_row + q) * row_words;
#pragma unroll
        for (int k = 0; k < T / 64; ++k) {
            const int tl = k * 64 + lane;
            const int t = t0 + tl;
            const uint32_t e = tile[r * RS + tl];
            const int v = e == SINK ? TDFA_DEAD : (int)(e / (uint32_t)sizeof(ST)) + state_base;
            if (t < n_tokens) drow[t] = v;
            const uint64_t m = __builtin_amdgcn_ballot_w64(v >= 0);
            const int64_t word = (int64_t)((t0 + k * 64) >> 5) + lane;
            if (lane < 2 && word < row_words) arow[word] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
        }
        // a row is a multiple of 4 words: what lies past the last token tile is padding
        const int64_t pad = (int64_t)((t0 + T) >> 5) + lane;
        if (tile_t == n_tiles_t - 1 && lane < 4 && pad < row_words) arow[pad] = 0u;
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

template <typename ST, int S, int T, int KT, bool HAS_JUMP, int kTileWaves = 16, bool STAGED = false>
int launch_tiles(const CompileArgs& a, const CompileEntry* e, int n, hipStream_t stream)
{
    size_t lds = TileShape<ST, S, T>::lds_bytes;
    if (STAGED) {
        size_t table = 0;
        for (int i = 0; i < n; ++i) table = std::max(table, (size_t)256 * e[i].q_stride * sizeof(ST));
        lds += table;
    }
    BatchDesc batch;
    batch.n = n;
    int64_t n_tiles_q = 0;
    bool share_columns = false;
    int max_q_tiles64 = 0, max_groups = 0;
    for (int i = 0; i < n; ++i) {
        DfaDesc& d = batch.d[i];
        d.trans = e[i].trans;
        d.tt = e[i].trans_t;
        d.order = e[i].order;
        d.plan = e[i].plan;
        d.start_bytes = e[i].start_bytes;
        d.n_states = e[i].n_states;
        d.q_stride = e[i].q_stride;
        d.tile_q_begin = (int32_t)n_tiles_q;
        d.out_row = e[i].out_row;
        d.state_base = e[i].state_base;
        d.n_order = e[i].n_order;
        n_tiles_q += (e[i].n_order + S - 1) / S;
        // a table that does not fit an XCD's 4 MB L2 (with room for the rest) gets the column-sharing order
        share_columns |= (size_t)256 * e[i].q_stride * sizeof(ST) > (size_t)3 << 20;
        max_q_tiles64 = std::max(max_q_tiles64, (e[i].q_stride + 63) / 64);
        max_groups = std::max(max_groups, (e[i].n_order + 63) / 64);
    }
    batch.n_tiles_q = (int32_t)n_tiles_q;
    transpose_kernel<ST><<<dim3(max_q_tiles64, 4, n), kThreads, 0, stream>>>(batch);
    TDFA_HIP(hipGetLastError());
    start_bytes_kernel<<<dim3((a.n_tokens + kThreads - 1) / kThreads, n, (max_groups + kStartChunk - 1) / kStartChunk), kThreads, 0,
                         stream>>>(batch, a.vprefix, a.vlen, a.n_tokens);
    TDFA_HIP(hipGetLastError());
    const int64_t n_tiles_t = (a.n_tokens + T - 1) / T;
    const int64_t n_groups = share_columns ? (n_tiles_t + kXcds - 1) / kXcds * kXcds * n_tiles_q : (n_tiles_t * n_tiles_q + 31) / 32 * 32;
    if (n_groups > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "table too large for one launch");
    const int wide_rows = a.n_tokens % 4 == 0 && reinterpret_cast<uintptr_t>(a.delta) % 16 == 0;
    auto kern = compile_tile_kernel<ST, S, T, KT, HAS_JUMP, kTileWaves, STAGED>;
    static size_t attr_set = 0;                    // the most LDS this instantiation has been allowed so far
    if (attr_set < lds) {
        TDFA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds));
        attr_set = lds;
    }
    kern<<<dim3((unsigned)n_groups), kTileWaves * 64, lds, stream>>>(batch, a.vwords, a.voff, a.vlen, a.vsorted, a.vprefix, a.n_tokens,
                                                                  (int)n_tiles_t, share_columns ? 1 : 0, wide_rows, a.delta, a.allow,
                                                                  a.row_words);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

}  // namespace

int launch_transpose(const CompileEntry* e, int n, hipStream_t stream)
{
    if (n <= 0) return TDFA_OK;
    if (n > kMaxBatch) return fail(TDFA_E_UNSUPPORTED, "too many automata for one launch");
    BatchDesc batch;
    batch.n = n;
    batch.n_tiles_q = 0;
    int max_q_tiles64 = 0;
    for (int i = 0; i < n; ++i) {
        DfaDesc& d = batch.d[i];
        d = DfaDesc();
        d.trans = e[i].trans;
        d.tt = e[i].trans_t;
        d.n_states = e[i].n_states;
        d.q_stride = e[i].q_stride;
        max_q_tiles64 = std::max(max_q_tiles64, (e[i].q_stride + 63) / 64);
    }
    if (e[0].narrow) transpose_kernel<uint16_t><<<dim3(max_q_tiles64, 4, n), kThreads, 0, stream>>>(batch);
    else transpose_kernel<uint32_t><<<dim3(max_q_tiles64, 4, n), kThreads, 0, stream>>>(batch);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
}

int launch_compile(const CompileArgs& a, hipStream_t stream)
{
    if (a.n_tokens <= 0) return TDFA_OK;
    // automata of one table width go together, up to kMaxBatch per launch, in the order given
    int i = 0;
    while (i < a.n) {
        if (a.entries[i].use_pairs) {
            const int prc = launch_compile_sweep(a, a.entries[i], stream);
            if (prc != TDFA_OK) return prc;
            ++i;
            continue;
        }
        int j = i + 1;
        while (j < a.n && j - i < kMaxBatch && a.entries[j].narrow == a.entries[i].narrow && a.entries[j].staged == a.entries[i].staged &&
               !a.entries[j].use_pairs)
            ++j;
        const CompileEntry* e = a.entries + i;
        const int n = j - i;
        bool jump = false;
        for (int k = 0; k < n; ++k) jump |= e[k].has_jump;
        // Measured: four workgroups of 512 threads per CU with 256 x 64 tiles (38 KB of LDS each)
        // beat two of 1,024 threads with 256 x 128 or 512 x 64 tiles on every workload: the set-up,
        // walk and flush phases of more independent workgroups overlap better.
        int rc;
        bool staged = e->narrow;
        for (int k = 0; k < n; ++k) staged = staged && e[k].staged;
        if (!e->narrow)
            rc = jump ? launch_tiles<uint32_t, 64, 256, 4, true>(a, e, n, stream)
                      : launch_tiles<uint32_t, 64, 256, 4, false>(a, e, n, stream);
        else if (staged)
            rc = jump ? launch_tiles<uint16_t, 256, 64, 1, true, 8, true>(a, e, n, stream)
                      : launch_tiles<uint16_t, 256, 64, 1, false, 8, true>(a, e, n, stream);
        else
            rc = jump ? launch_tiles<uint16_t, 256, 64, 1, true, 8>(a, e, n, stream)
                      : launch_tiles<uint16_t, 256, 64, 1, false, 8>(a, e, n, stream);
        if (rc != TDFA_OK) return rc;
        i = j;
    }
    return TDFA_OK;
}

namespace {

// Terminal labels (Section 2.5.1): one workgroup per 256 tokens of one state that has terminal
// edges.  An entry that is still DEAD takes the target of the first of the state's edges whose
// mask holds the token; the row's allowed words are rewritten from the entries.
__global__ void __launch_bounds__(kThreads)
apply_terminals_kernel(int32_t* __restrict__ delta, uint32_t* __restrict__ allow, int32_t n_tokens, int64_t row_words,
                       const int32_t* __restrict__ state_of, const int32_t* __restrict__ edge_begin,
                       const int32_t* __restrict__ edge_label, const int32_t* __restrict__ edge_target,
                       const uint32_t* __restrict__ masks)
{
    const int q = state_of[blockIdx.y];
    const int e_lo = edge_begin[blockIdx.y], e_hi = edge_begin[blockIdx.y + 1];
    const int t = blockIdx.x * kThreads + threadIdx.x;
    int32_t* row = delta + (size_t)q * n_tokens;
    int v = TDFA_DEAD;
    if (t < n_tokens) {
        v = row[t];
        if (v == TDFA_DEAD) {
            for (int e = e_lo; e < e_hi; ++e) {
                if ((masks[(size_t)edge_label[e] * row_words + (t >> 5)] >> (t & 31)) & 1u) {
                    v = edge_target[e];
                    row[t] = v;
                    break;
                }
            }
        }
    }
    const uint64_t m = __builtin_amdgcn_ballot_w64(v != TDFA_DEAD);
    const int lane = threadIdx.x & 63;
    const int64_t word = (int64_t)((t - lane) >> 5) + lane;
    if (lane < 2 && word < row_words) allow[(size_t)q * row_words + word] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
}

}  // namespace

int launch_apply_terminals(int32_t* delta, uint32_t* allow, int32_t n_tokens, int64_t row_words, int32_t n_states_with_edges,
                           const int32_t* state_of, const int32_t* edge_begin, const int32_t* edge_label,
                           const int32_t* edge_target, const uint32_t* masks, hipStream_t stream)
{
    if (n_states_with_edges <= 0 || n_tokens <= 0) return TDFA_OK;
    const unsigned bx = (unsigned)((row_words * 32 + kThreads - 1) / kThreads);
    apply_terminals_kernel<<<dim3(bx, (unsigned)n_states_with_edges), kThreads, 0, stream>>>(
        delta, allow, n_tokens, row_words, state_of, edge_begin, edge_label, edge_target, masks);
    TDFA_HIP(hipGetLastError());
    return TDFA_OK;
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
