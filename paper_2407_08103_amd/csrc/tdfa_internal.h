// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <functional>
#include <vector>

#include "tdfa.h"

namespace tdfa {

// Sets the thread-local message returned by tdfa_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define TDFA_HIP(expr)                                                                            \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return ::tdfa::fail(e_ == hipErrorOutOfMemory ? TDFA_E_OOM : TDFA_E_DEVICE,           \
                                "%s: %s", #expr, hipGetErrorString(e_));                          \
    } while (0)

constexpr int kVocabSortBlock = 64;
constexpr int kJumpDepth = 32;        // default-chain jump tables cover prefixes of 1 .. kJumpDepth bytes
constexpr int kMaxJumpClasses = 8;    // classes of states that get jump tables, per automaton
constexpr int kMinJumpClass = 24;     // a class smaller than this is not worth a 64-lane group of its own
constexpr size_t kStagedTableBytes = 96 * 1024;    // the largest transposed table the walk keeps in LDS beside its tile

// What the compile kernel needs to know about an automaton beyond its table (see plan.hip).
struct StatePlan {
    std::vector<int32_t> order;        // states in the order the lanes take them; -1 = idle lane
    std::vector<int8_t> group_class;   // per 64 entries of order: jump class of the group, or -1
    std::vector<uint32_t> group_live;  // [n_groups][8]: bit b set = some state of the group has a transition on byte b
    std::vector<uint32_t> clean_set;   // [n_classes][8]: bit b set = byte b is a clean byte of the class
    std::vector<int32_t> jump;         // [kJumpDepth][n_states]: state after m + 1 clean bytes (DEAD = -1);
                                       // empty if n_classes == 0
    int n_classes = 0;
    int64_t n_pairs = 0;               // (state, b1, b2) triples with delta*(state, b1 b2) defined
};
// Validates trans (every entry in [-1, n_states)) and fills *plan.
int make_state_plan(const int32_t* trans, int32_t n_states, StatePlan* plan);
// Calls task(0) .. task(n_tasks - 1) on the library's few host threads (the caller's among them) and
// returns when all are done.
void host_tasks(unsigned n_tasks, const std::function<void(unsigned)>& task);

// Layout of the plan as uploaded (one device blob per automaton):
//   bytes [0, kPlanSetBytes)            clean sets, kMaxJumpClasses x 8 words
//   bytes [kPlanSetBytes, + n_groups)   group_class (int8), n_groups = ceil(n_order / 64)
//   bytes [plan_live_offset(n_order), ..) group_live, n_groups x 8 words
//   bytes [plan_jump_offset(n_order), ..) jump tables [kJumpDepth][q_stride] in the offset form of the
//                                       transposed table (present only if the automaton has a class)
constexpr size_t kPlanSetBytes = (size_t)kMaxJumpClasses * 32;
__host__ __device__ inline size_t plan_live_offset(int32_t n_order) { return kPlanSetBytes + ((size_t)(n_order + 63) / 64 + 255) / 256 * 256; }
__host__ __device__ inline size_t plan_jump_offset(int32_t n_order)
{
    return plan_live_offset(n_order) + ((size_t)(n_order + 63) / 64 * 32 + 255) / 256 * 256;
}

// The device arrays of a vocabulary handle that other translation units read (api.hip owns the handle).
struct VocabView {
    const uint32_t* words;   // token bytes, each token padded to a multiple of 4 bytes
    const uint32_t* off;     // [n_tokens + 1] word offset of each token
    const uint32_t* len;     // [n_tokens] byte length
    int32_t n_tokens;
};
void vocab_view(const tdfa_vocab* vocab, VocabView* out);

inline int64_t allow_row_words(int64_t n_tokens) { return n_tokens <= 0 ? 0 : ((n_tokens + 31) / 32 + 3) / 4 * 4; }

// Launchers implemented in compile.hip / mask.hip.  All enqueue on `stream` and return a status.
struct CompileEntry {         // one character automaton of a compile launch
    const int32_t* trans;     // device [n_states][256], as uploaded
    void* trans_t;            // device workspace [256][q_stride], uint16 if narrow else uint32
    const int32_t* order;     // device [n_order]: states listed so that like states are neighbours, -1 = idle
    const unsigned char* plan;  // device blob: clean sets, group classes, jump tables (layout above)
    int32_t n_order;
    bool has_jump;            // the plan holds at least one jump class (and start_bytes is there)
    uint8_t* start_bytes;     // device workspace [ceil(n_order / 64)][n_tokens], or NULL: none (see compile.hip)
    bool narrow;              // byte offsets of all states (and the sink) fit in 16 bits
    int32_t n_states;
    int32_t q_stride;         // row stride of trans_t in elements (multiple of 64, > n_states)
    int32_t out_row;          // row of delta / allow where this automaton's rows start
    int32_t state_base;       // added to every live entry (row offset inside a stacked table)
    bool staged;              // the walk reads trans_t from a copy in LDS (it fits: kStagedTableBytes)
    // the level-by-level sweep over prefix lists (sweep.hip); use_pairs = compile this automaton that way
    bool use_pairs;
    const struct SweepWorkspace* sweep;
};
// Device workspace of the sweep (sweep.hip), owned by the automaton's handle.
struct SweepWorkspace {
    uint32_t* n1 = nullptr;       // [256]
    uint32_t* off1 = nullptr;     // [257]
    uint32_t* cnt2 = nullptr;     // [65536]
    uint32_t* err = nullptr;      // [1]
    uint32_t* list1 = nullptr;    // [off1[256]]
    uint32_t* list2 = nullptr;    // [256 * off1[256]]
    unsigned long long* chunk_sum = nullptr;   // [token_cap / 1024 + 2]
    uint32_t* need = nullptr;     // [token_cap + 1]
    uint32_t* cnt3 = nullptr;     // [token_cap]
    uint32_t* cntF = nullptr;     // [token_cap]
    uint32_t* buf_a = nullptr;    // [buf_cap]
    uint32_t* buf_b = nullptr;
    uint64_t buf_cap = 0;
    uint64_t list2_cap = 0;
    int32_t token_cap = 0;
    bool sized = false;           // list2 is allocated (its size depends on the automaton only)
    bool buffers_sized = false;   // buf_a / buf_b fit the vocabulary they were last sized for
    const void* sized_for = nullptr;   // that vocabulary
    // the launch that sized the buffers has left the lists of the first two levels and the tokens'
    // regions in place: the next launch for this automaton starts at the third byte
    mutable bool lists_ready = false;
};

struct CompileArgs {
    const CompileEntry* entries;
    int32_t n;
    const uint32_t* vwords;   // device: token bytes, each token padded to a multiple of 4 bytes
    const uint32_t* voff;     // device [n_tokens + 1]: word offset of each token in vwords
    const uint32_t* vlen;     // device [n_tokens]: byte length of each token
    const uint8_t* vsorted;   // device [n_tokens]: per block of kVocabSortBlock ids, the block-local token
                              // indices in byte-lexicographic order
    const uint32_t* vprefix;  // device [n_tokens][8]: the first 32 bytes of each token, zero padded
    int32_t n_tokens;
    const int32_t* group_tokens[2];   // tokens that have a third / fourth byte, grouped by that byte (sweep.hip)
    const int32_t* group_chunks[2];   // [n_group_chunks][3]: byte, first index into group_tokens, number of tokens
    int32_t n_group_chunks[2];
    const int32_t* tail_tokens;       // tokens of five or more bytes
    int32_t n_tail;
    int32_t* delta;           // device [rows][n_tokens]
    uint32_t* allow;          // device [rows][row_words]
    int64_t row_words;
};
int launch_compile(const CompileArgs& a, hipStream_t stream);
// The transposed offset-form tables of n automata of one width (compile.hip).
int launch_transpose(const CompileEntry* e, int n, hipStream_t stream);
// One narrow automaton by the level-by-level sweep (sweep.hip).  While the workspace is not fully
// sized (e.sweep->sized / buffers_sized) only the kernels whose results size it are launched.
int launch_compile_sweep(const CompileArgs& a, const CompileEntry& e, hipStream_t stream);

int launch_concat_part(const int32_t* src_delta, const uint32_t* src_allow, int64_t n_rows, int32_t n_tokens,
                       int64_t row_words, int64_t row_base, int32_t* dst_delta, uint32_t* dst_allow,
                       hipStream_t stream);

int launch_apply_terminals(int32_t* delta, uint32_t* allow, int32_t n_tokens, int64_t row_words, int32_t n_states_with_edges,
                           const int32_t* state_of, const int32_t* edge_begin, const int32_t* edge_label,
                           const int32_t* edge_target, const uint32_t* masks, hipStream_t stream);

// Token-level optimisation (optimize.hip): which old rows are the first rows of the classes that are
// kept, in the order of the new states, and the new state of every old state (TDFA_DEAD: dropped).
int minimize_table(const int32_t* delta, int64_t n_rows, int32_t n_tokens, const uint8_t* accept_host,
                   const int32_t* starts_host, int32_t n_starts, hipStream_t stream, std::vector<int32_t>* first_rows,
                   std::vector<int32_t>* map_out);
int launch_compact_rows(const int32_t* delta, int32_t n_tokens, int64_t row_words, const std::vector<int32_t>& first_rows,
                        const std::vector<int32_t>& map, int32_t* out_delta, uint32_t* out_allow, hipStream_t stream);

// out[q] = the tokens row q of `allow` allows (pack.hip).
int launch_row_allowed(const uint32_t* allow, int64_t n_rows, int32_t n_tokens, int64_t row_words, uint32_t* out, hipStream_t stream);

// Edge-list form of a table (pack.hip): the device arrays are allocated here and owned by the caller.
int pack_table(const int32_t* delta, const uint32_t* allow, int64_t n_rows, int32_t n_tokens, int64_t row_words,
               hipStream_t stream, uint32_t** dir_out, int64_t** row_begin_out, int32_t** targets_out, int64_t* n_edges_out);

struct MaskArgs {
    const int32_t* delta;               // dense rows, or NULL for a packed table: then the three arrays below.
                                        // Both delta and targets NULL: no table; the step chooses tokens only and
                                        // new_states receives the states unchanged
    const int32_t* targets;             // packed: targets of all edges, states in order, tokens in order
    const int64_t* row_begin;           // packed: [n_rows + 1] first edge of each state
    const uint32_t* dir;                // packed: [n_rows][row_words / 4] edges of the state below each 128-token block
    const uint32_t* allow;
    const uint32_t* row_allowed;        // [n_rows] tokens each state allows, or NULL if not known: a sequence in a state
                                        // that allows none (its text is complete) is done after two reads
    int64_t n_rows;
    int32_t n_tokens;
    int64_t row_words;
    const void* logits;
    int dtype;
    int32_t batch;
    int64_t row_stride;
    const int32_t* states;
    int32_t* tokens;
    int32_t* new_states;
    void* masked_out;
    unsigned long long* scratch_best;   // device [>= batch], all zero between launches
    unsigned int* scratch_count;        // device [>= batch], all zero between launches
    // The step of a push-down constraint (Section 3): when class_first is set there is no table (delta and
    // targets NULL), `states` are states of the push-down automaton, `allow` holds one row of allowed bits
    // per class of edges (the edges of a state that pop the same symbols; the classes of state q are rows
    // class_first[q] .. class_first[q + 1], at most 64), and the allowed set of a sequence is the OR of
    // the rows of its state's classes whose pops its stack ends with.
    struct Pda {
        const int32_t* class_first;     // [n_states + 1]
        const int32_t* class_n_pops;    // [rows]
        const int32_t* class_pops;      // [rows][kPdaPops], the symbol popped first (the top of the stack) first
        const int32_t* stacks;          // [batch][stack_cap]
        const int32_t* depths;          // [batch]
        int32_t stack_cap;
        int32_t n_states;
    } pda;
};
constexpr int kPdaPops = 12;            // symbols an edge of a push-down automaton may pop
int launch_mask_step(const MaskArgs& a, hipStream_t stream);
// Whether launch_mask_step takes `a` with a.pda set (16-bit logits, no masked row written, a vocabulary whose
// allowed bits fit the workgroup's LDS); otherwise the caller makes one row per sequence first.
bool mask_step_takes_pda(const MaskArgs& a);
// The per-device scratch of the step kernels for `batch` sequences (all zero between launches); grown
// outside stream capture only.
int step_scratch(int32_t batch, hipStream_t stream, unsigned long long** best, unsigned int** count);
// Whether launch_mask_step(a) splits rows over workgroups that meet through scratch_best / scratch_count.
bool mask_step_uses_scratch(const MaskArgs& a);
// best[0 .. n) <- 0, count[0 .. n) <- 0, by a kernel.
int launch_clear_scratch(unsigned long long* best, unsigned int* count, int32_t n, hipStream_t stream);
// cut_scratch: device [>= batch] words, written and read by the call when top_k > 0
// offset_dev: if not NULL, the kernel reads the offset from this device word instead of `offset`
int launch_sample_step(const MaskArgs& a, float inv_t, int32_t top_k, uint32_t* cut_scratch, uint64_t seed,
                       uint64_t offset, const uint64_t* offset_dev, hipStream_t stream);
int launch_sample_noise(int32_t batch, int32_t n_tokens, uint64_t seed, uint64_t offset, float* out, hipStream_t stream);
// The table fields of `table` are used (delta or the packed arrays, allow, n_rows, n_tokens, row_words).
int launch_advance_tokens(const MaskArgs& table, int32_t batch, int32_t k, const int32_t* states, const int32_t* tokens,
                          int32_t* history, int32_t* n_valid, hipStream_t stream);

}  // namespace tdfa
