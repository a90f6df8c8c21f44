// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

inline int64_t allow_row_words(int64_t n_tokens) { return n_tokens <= 0 ? 0 : ((n_tokens + 31) / 32 + 3) / 4 * 4; }

// Launchers implemented in compile.hip / mask.hip.  All enqueue on `stream` and return a status.
struct CompileEntry {         // one character automaton of a compile launch
    const int32_t* trans;     // device [n_states][256], as uploaded
    void* trans_t;            // device workspace [256][q_stride], uint16 if narrow else uint32
    const int32_t* order;     // device [n_states]: states listed so that like states are neighbours
    bool narrow;              // byte offsets of all states (and the sink) fit in 16 bits
    int32_t n_states;
    int32_t q_stride;         // row stride of trans_t in elements (multiple of 64, > n_states)
    int32_t out_row;          // row of delta / allow where this automaton's rows start
    int32_t state_base;       // added to every live entry (row offset inside a stacked table)
};
struct CompileArgs {
    const CompileEntry* entries;
    int32_t n;
    const uint32_t* vwords;   // device: token bytes, each token padded to a multiple of 4 bytes
    const uint32_t* voff;     // device [n_tokens + 1]: word offset of each token in vwords
    const uint32_t* vlen;     // device [n_tokens]: byte length of each token
    const uint8_t* vsorted;   // device [n_tokens]: per block of kVocabSortBlock ids, the block-local token
                              // indices in byte-lexicographic order
    int32_t n_tokens;
    int32_t* delta;           // device [rows][n_tokens]
    uint32_t* allow;          // device [rows][row_words]
    int64_t row_words;
};
int launch_compile(const CompileArgs& a, hipStream_t stream);

int launch_concat_part(const int32_t* src_delta, const uint32_t* src_allow, int64_t n_rows, int32_t n_tokens,
                       int64_t row_words, int64_t row_base, int32_t* dst_delta, uint32_t* dst_allow,
                       hipStream_t stream);

struct MaskArgs {
    const int32_t* delta;
    const uint32_t* allow;
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
};
int launch_mask_step(const MaskArgs& a, hipStream_t stream);

}  // namespace tdfa
