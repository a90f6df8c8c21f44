/*
 * tdfa.h - token-level constraint automata for language-model decoding on AMD CDNA4 (gfx950).
 *
 * C ABI of the library.  Two stages of "Automata-based constraints for language model
 * decoding" (arXiv 2407.08103) run as hand-written HIP kernels behind these calls:
 *
 *   compile   A character-level deterministic automaton A_R (Section 2.1) is lifted to the
 *             token-accepting automaton A_{R o V} = A_R o T_V (Sections 2.3-2.4, Algorithm 2,
 *             first three statements), materialised as a dense table
 *                 delta_T[q][t] = state reached from q by reading the bytes of token t,
 *                                 or TDFA_DEAD if some transition on the way is missing,
 *             which is what composing A_R with the detokenizing transducer T_V of Algorithm 1
 *             and removing its epsilon edges gives when A_R is deterministic (Theorems 1, 2).
 *   decode    The loop body of Algorithm 2 after ComputeLogits: the allowed set of each
 *             sequence's state, the -inf penalty on every other logit, the token choice
 *             (greedy argmax) and the traversal of the matching edge.
 *
 * Conventions
 *   - Every function returns an int status: TDFA_OK or a negative TDFA_E_* code; nothing
 *     throws or aborts.  tdfa_last_error() gives a thread-local message for the last failure.
 *   - "host" / "device" in a parameter comment says where the pointed-to memory lives.
 *     Device memory belongs to the GPU that is current when the call is made.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that take a
 *     stream only enqueue work on it and return; they do not synchronise with the host unless
 *     the comment says so.  Host arrays passed in may be freed as soon as the call returns.
 *   - States are int32 row indices of a table; alphabet = bytes (256 symbols).
 *   - Handles are not thread-safe; use one handle from one thread at a time.
 */
#ifndef TDFA_H_
#define TDFA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDFA_API __attribute__((visibility("default")))

enum {
    TDFA_OK = 0,
    TDFA_E_INVALID_ARG = -1,   /* null pointer, bad size, malformed automaton or vocabulary */
    TDFA_E_OOM = -2,           /* host or device allocation failed */
    TDFA_E_DEVICE = -3,        /* a HIP call failed; see tdfa_last_error() */
    TDFA_E_UNSUPPORTED = -4    /* valid request outside what the library handles */
};

enum { TDFA_F32 = 0, TDFA_BF16 = 1 };   /* element type of logits */

#define TDFA_DEAD     (-1)   /* table entry: no edge; state: outside the automaton */
#define TDFA_NO_TOKEN (-1)   /* tokens[] entry when no token is allowed */

typedef struct tdfa_vocab tdfa_vocab;   /* a vocabulary, packed on the device (the compact T_V) */
typedef struct tdfa_dfa   tdfa_dfa;     /* a character-level automaton, resident on the device */
typedef struct tdfa_table tdfa_table;   /* a token-level table delta_T plus its allowed-bit rows */

/* ---- library ------------------------------------------------------------------------------ */

/* Message for the last failing call on this thread ("" if none).  Never NULL. */
TDFA_API const char *tdfa_last_error(void);

/* Library version as major * 10000 + minor * 100 + patch. */
TDFA_API int tdfa_version(void);

/* ---- vocabulary (once per language model: Section 2.4, T_V does not depend on the constraint) -- */

/* Packs a vocabulary for the compile kernels.  Token t detokenizes to the bytes
 * bytes[offsets[t] .. offsets[t+1]) (Appendix B.1: d(v)); offsets has n_tokens + 1
 * non-decreasing entries.  This is the compact, prefix-merged form of Algorithm 1's T_V
 * (Section 2.3, last paragraph): the library stores the byte strings in a layout of its own in
 * which tokens that share a prefix sit together, plus the permutation back to token ids.
 * Tokens may repeat; a zero-length token has no cycle in T_V and is never allowed.
 *   bytes, offsets : host.   n_tokens : 0 .. 2^24.
 *   out            : receives a handle owned by the library; release with tdfa_vocab_destroy.
 * Blocks until the device copy is complete.  Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_vocab_create(const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens,
                      void *stream, tdfa_vocab **out);
TDFA_API int tdfa_vocab_destroy(tdfa_vocab *vocab);
TDFA_API int tdfa_vocab_info(const tdfa_vocab *vocab, int32_t *n_tokens, int64_t *n_bytes, int32_t *max_len);

/* ---- character automaton (once per constraint) --------------------------------------------- */

/* Uploads a deterministic character automaton (Section 2.1: no epsilon edges, at most one edge
 * per state and symbol).  trans[q * 256 + b] is the target of the edge of q labelled b, or
 * TDFA_DEAD.  The automaton should be trim (every state can reach a final state), so that a
 * non-DEAD table entry means the text is still a viable prefix; the library does not trim.
 *   trans  : host, int32 [n_states * 256], every entry in [-1, n_states).
 *   accept : host, uint8 [n_states], non-zero = final state; may be NULL (no final states
 *            recorded).  Passed through for the caller; the kernels do not read it.
 *   start  : the initial state I, in [0, n_states).   n_states : 1 .. 2^22 - 64.
 * Also prepares the automaton for the compile kernels, on a few host threads that the library
 * keeps for this: the range check, the order in which the kernel's lanes take the states, and for
 * counter-like classes of states the jump tables (delta* over runs of their clean bytes, see
 * tdfa_plan_describe), which the kernel copies into the table: about a millisecond per 5,000
 * states.  Blocks until the device copy is complete; the copies run on a stream of the library's
 * own, so the call does not wait for work queued on `stream` (which is not used).  Errors:
 * INVALID_ARG (names the bad entry), OOM, DEVICE. */
TDFA_API int tdfa_dfa_create(const int32_t *trans, const uint8_t *accept, int32_t n_states, int32_t start,
                    void *stream, tdfa_dfa **out);
/* Does not wait for the GPU: the automaton's device memory goes to a cache inside the library, with
 * an event recorded behind the last compile call that used the handle, and is handed to a later
 * tdfa_dfa_create once that event has completed (tdfa_trim gives the cache back to the device).  A
 * handle that a compile call used under stream capture, or that was compiled by the sweep (whose
 * lists are freed), waits for the device instead. */
TDFA_API int tdfa_dfa_destroy(tdfa_dfa *dfa);

/* Caps the device workspace that compile calls may allocate for this automaton beyond its tables
 * (one byte per 64 states and token, see tdfa_compile_token_dfa; 1 GiB unless set).  A compile
 * whose workspace would exceed the cap runs without it: the same table, computed by plain
 * byte-by-byte walks.  Errors: INVALID_ARG. */
TDFA_API int tdfa_dfa_workspace_limit(tdfa_dfa *dfa, int64_t max_bytes);

/* Which kernels compile this automaton.  The table is delta*(q, d(t)) of Section 2.4 whichever is
 * taken; the choice only changes how the kernels get there.
 *   TDFA_PATH_WALK  : every token is walked byte by byte from every state, 64 states per wavefront,
 *                     with jumps over runs of clean bytes for counter-like classes of states.
 *   TDFA_PATH_PAIRS : the vocabulary's prefix trie is swept level by level (the prefix sharing of the
 *                     compact T_V, Section 2.3).  For every two-byte prefix (b1, b2), at most 65,536
 *                     however large the vocabulary, the (state, target) pairs that survive it are
 *                     listed; every longer token filters its prefix's list through its third and
 *                     fourth byte, with that byte's column of the automaton held in LDS, and the
 *                     few pairs left are walked to the token's end; the lists are then expanded
 *                     into rows.  Needs device workspace: 1 KiB per edge of the automaton plus
 *                     8 bytes per token and pair of its prefix's list, sized by the first compile
 *                     call (which waits for the device twice) and again for another vocabulary.
 *                     Automata with more than 32,767 states or with counter-like classes are
 *                     compiled by TDFA_PATH_WALK all the same, and so is one whose workspace would
 *                     exceed 8 x the limit of tdfa_dfa_workspace_limit.
 *   TDFA_PATH_STAGED: TDFA_PATH_WALK with the automaton's whole table copied into the 160 KB of LDS of
 *                     each compute unit before the walk, so that the walk's lookups never leave it.
 *                     For automata of at most 191 states (the table beside the kernel's tile); larger
 *                     ones take TDFA_PATH_WALK all the same.
 *   TDFA_PATH_AUTO  : (default) TDFA_PATH_PAIRS for automata of 8,192 states or more that can take it,
 *                     else TDFA_PATH_WALK.
 * Errors: INVALID_ARG. */
enum { TDFA_PATH_AUTO = 0, TDFA_PATH_WALK = 1, TDFA_PATH_PAIRS = 2, TDFA_PATH_STAGED = 3 };
TDFA_API int tdfa_dfa_compile_path(tdfa_dfa *dfa, int path);

/* The four large workspace arrays of TDFA_PATH_PAIRS are kept when their automaton is destroyed (at
 * most eight blocks per process, the oldest freed first) and handed to the next automaton that needs
 * blocks of about their size: allocating them anew costs as much as a tenth of such a compile.
 * tdfa_trim() gives the kept blocks back to the device.  Errors: none. */
TDFA_API int tdfa_trim(void);

/* What is known about an uploaded automaton (any out-pointer may be NULL).
 *   compile_path    : TDFA_PATH_WALK, TDFA_PATH_PAIRS or TDFA_PATH_STAGED, the kernels the next compile call takes.
 *   workspace_bytes : device workspace of TDFA_PATH_PAIRS once a compile call has sized it; -1 before
 *                     that and for the walk (whose workspace is one byte per 64 states and token). */
TDFA_API int tdfa_dfa_info(const tdfa_dfa *dfa, int32_t *n_states, int32_t *start, int32_t *compile_path,
                  int64_t *workspace_bytes);

/* Disjoint union of n uploaded automata as one automaton (once per set of constraints): the
 * states of dfas[c] become states row_offsets_host[c] .. row_offsets_host[c + 1] - 1, edges stay
 * inside their automaton.  Compiling the union with tdfa_compile_token_dfa gives the stacked
 * multi-constraint table of tdfa_compile_stacked / tdfa_table_concat (states are global row ids)
 * in one piece: the lanes of the compile kernel are then filled across automata, and states of
 * the same kind from different automata share their jump tables.  A sequence bound to
 * constraint c starts in state row_offsets_host[c] + start_c; the union's own start state is
 * that of dfas[0].
 *   row_offsets_host : host, int64 [n + 1], written.
 * Reads the automata back from the device and blocks until the union is uploaded.
 * Errors: INVALID_ARG (also when the union has more than 2^22 - 64 states), OOM, DEVICE. */
TDFA_API int tdfa_dfa_union(const tdfa_dfa *const *dfas, int32_t n, void *stream, tdfa_dfa **out,
                   int64_t *row_offsets_host);

/* The same union made from automata that are still on the host, without uploading each one first:
 * one automaton is created, the union.
 *   trans    : host, n pointers to int32 [n_states[c] * 256], as for tdfa_dfa_create.
 *   accept   : host, n pointers to uint8 [n_states[c]], or NULL, or NULL entries (no final states).
 *   n_states : host, int32 [n].   start : the start state of automaton 0 (the union's own).
 *   row_offsets_host : host, int64 [n + 1], written.
 * Blocks until the union is uploaded.  Errors: as tdfa_dfa_create (a bad entry is named by its place
 * in the union) and tdfa_dfa_union. */
TDFA_API int tdfa_dfa_union_host(const int32_t *const *trans, const uint8_t *const *accept, const int32_t *n_states,
                        int32_t n, int32_t start, void *stream, tdfa_dfa **out, int64_t *row_offsets_host);

/* Host only, no device call: the preparation that tdfa_dfa_create derives from an automaton for
 * the compile kernels, for inspection and tests.  It does not change what is computed (the
 * table is delta*(q, d(t)) of Section 2.4 either way), only how the kernel gets there.
 *   order       : host, int32 [cap]: the states in the order the kernel's lanes take them, in
 *                 groups of 64; -1 = idle lane.  *n_order receives the length (a call with
 *                 cap too small fails with INVALID_ARG after setting *n_order).
 *   group_class : host, int8 [cap / 64 rounded up]: per group its jump class, or -1.
 *   clean_sets  : host, uint32 [8 * 8]: per class the 256-bit set of its clean bytes (bit b of
 *                 word b >> 5); a token whose first m bytes are clean bytes of the class takes
 *                 every state q of the class to jump[(m - 1) * n_states + q], m = 1 .. 32.
 *   jump        : host, int32 [32 * n_states] or NULL; entries of states outside a class are -1.
 *   n_classes   : receives the number of classes (0 .. 8).
 * Errors: INVALID_ARG (also for a malformed automaton), OOM. */
TDFA_API int tdfa_plan_describe(const int32_t *trans, int32_t n_states, int32_t *order, int32_t cap,
                       int32_t *n_order, int8_t *group_class, uint32_t *clean_sets, int32_t *jump,
                       int32_t *n_classes);

/* ---- compile: A_R o T_V as a dense table (Algorithm 2, statement 3) ------------------------- */

/* Number of 32-bit words in one allowed-bit row for a vocabulary of n_tokens (the row stride of
 * allow_bits): ceil(n_tokens / 32) rounded up to a multiple of 4.  Negative n_tokens gives 0. */
TDFA_API int64_t tdfa_allow_row_words(int32_t n_tokens);

/* Computes delta_T for every state of `dfa` and every token of `vocab`:
 *     delta[q * n_tokens + t]                     int32, state-major, columns in token-id order
 *     allow[q * row_words + (t >> 5)] bit (t & 31)  set iff delta[q][t] != TDFA_DEAD
 * (padding bits are zero).  All states get a row, also those that no token sequence reaches; the
 * result is not renumbered or minimised, so it is the unique table of the caller's state ids.
 *   delta_dev : device, caller's buffer of n_states * n_tokens int32, or NULL to let the
 *               library allocate it (then the table owns it).
 *   allow_dev : device, caller's buffer of n_states * tdfa_allow_row_words(n_tokens) uint32, or
 *               NULL to let the library allocate it.
 *   out       : receives a table handle; release with tdfa_table_destroy (which frees only what
 *               the library allocated).
 * Enqueues on `stream` and returns; the vocab and dfa handles must stay alive until that work
 * has finished.  A dfa handle carries device workspace that the compile kernels write (the
 * transposed table, one byte per 64 states and token): compile calls that use the same dfa
 * handle must not overlap in time, so enqueue them on one stream.  The workspace is sized by
 * the first call for a vocabulary size and again when a larger one comes (that call allocates
 * and waits for the device); later calls with the same sizes allocate nothing.
 * A table that the library has written (this call, tdfa_compile_stacked, tdfa_table_concat,
 * tdfa_table_minimize) also carries, in a small device array of its own, how many tokens each state
 * allows; a decode step is done after two reads with a sequence whose state allows none (a text that
 * is complete).  A caller that edits the allowed bits in its own buffers afterwards must wrap them
 * again (tdfa_table_wrap keeps no such counts); tdfa_table_apply_terminals recounts by itself.
 * Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_compile_token_dfa(const tdfa_vocab *vocab, const tdfa_dfa *dfa,
                           int32_t *delta_dev, uint32_t *allow_dev,
                           void *stream, tdfa_table **out);

/* The same computation for one constraint of a stacked multi-constraint table: the rows are
 * written to the caller's buffers as given (delta_dev / allow_dev point at the first row of this
 * constraint's slice; NULL lets the library allocate), and every live entry has row_base added,
 * so the slice is ready to be part of a table whose states are global row ids (see
 * tdfa_table_concat for the meaning; this call saves the copy).  row_base >= 0 and
 * row_base + n_states must fit int32.  The returned handle describes the slice only. */
TDFA_API int tdfa_compile_token_dfa_at(const tdfa_vocab *vocab, const tdfa_dfa *dfa, int64_t row_base,
                              int32_t *delta_dev, uint32_t *allow_dev,
                              void *stream, tdfa_table **out);

/* All constraints of a stacked multi-constraint table in one call: the n automata are compiled
 * against `vocab` into one table whose rows are those of dfas[0], then dfas[1], ... with states
 * as global row ids (row_offsets_host[c] is added to the live entries of constraint c, as in
 * tdfa_table_concat), by launches that cover many automata at once.  A sequence bound to
 * constraint c starts in state row_offsets_host[c] + start_c.
 *   dfas             : host array of n handles (n >= 1).
 *   delta_dev / allow_dev : device buffers for sum(n_states) rows, or NULL to let the library allocate.
 *   row_offsets_host : host, int64 [n + 1], written before the call returns.
 * Enqueues on `stream`; vocab and dfas must stay alive until that work has finished. */
TDFA_API int tdfa_compile_stacked(const tdfa_vocab *vocab, const tdfa_dfa *const *dfas, int32_t n,
                         int32_t *delta_dev, uint32_t *allow_dev, void *stream,
                         tdfa_table **out, int64_t *row_offsets_host);

/* Stacks n tables over the same vocabulary into one whose states are global row ids: table c
 * occupies rows row_offsets[c] .. row_offsets[c+1], and every non-DEAD entry of table c has
 * row_offsets[c] added, so a sequence bound to constraint c starts in state
 * row_offsets[c] + start_c and tdfa_mask_step needs no per-constraint argument.
 *   tables           : host array of n handles (n >= 1), all with the same n_tokens.
 *   row_offsets_host : host, int64 [n + 1], written before the call returns.
 *   delta_dev / allow_dev : as in tdfa_compile_token_dfa, sized for the sum of the rows.
 * Enqueues on `stream`.  The inputs may be destroyed once that work has finished. */
TDFA_API int tdfa_table_concat(const tdfa_table *const *tables, int32_t n,
                      int32_t *delta_dev, uint32_t *allow_dev, void *stream,
                      tdfa_table **out, int64_t *row_offsets_host);

/* Wraps caller-owned device buffers that already hold a table in the layout above (for
 * example a slice of a larger allocation).  Nothing is copied and nothing is checked on the
 * device. */
TDFA_API int tdfa_table_wrap(int32_t *delta_dev, uint32_t *allow_dev, int64_t n_rows, int32_t n_tokens,
                    tdfa_table **out);

/* Any out-pointer may be NULL.  delta_dev / allow_dev are device pointers. */
TDFA_API int tdfa_table_info(const tdfa_table *table, int64_t *n_rows, int32_t *n_tokens,
                    int32_t **delta_dev, uint32_t **allow_dev, int64_t *allow_row_words);
TDFA_API int tdfa_table_destroy(tdfa_table *table);

/* ---- edge-list form of a table (Section 2.5.1; Appendix C.2) --------------------------------- */

/* The paper keeps A_{R o V} as a list of edges, which is small for the many states that allow a
 * few tokens and costly for the few that allow nearly all (Section 2.5.1).  The dense table is the
 * other way round.  tdfa_table_pack makes the form that serves both: a new table with the same
 * allowed-bit rows (a copy) and, instead of the dense rows, only the targets of the edges:
 *     targets   : device, int32 [n_edges]; the edges of state q are row_begin[q] .. row_begin[q+1] - 1,
 *                 in token order (the token of an edge is not stored)
 *     row_begin : device, int64 [n_rows + 1]
 *     dir       : device, uint32 [n_rows][row_words / 4]; dir[q][k] = edges of q on tokens below 128 k
 * so that, for an allowed token t,
 *     delta_T[q][t] = targets[row_begin[q] + dir[q][t / 128] + (allowed tokens of q in [128 (t / 128), t))].
 * Size: 4 bytes per edge plus |V| (1/8 + 1/32) bytes per state.  tdfa_mask_step, tdfa_sample_step and
 * tdfa_advance_tokens take a packed table wherever they take a dense one, with the same results;
 * tdfa_table_info reports delta_dev = NULL for it.  Calls that edit a table (tdfa_table_concat,
 * tdfa_table_apply_terminals, tdfa_table_minimize) want the dense one: pack last, then the dense
 * table can be destroyed.  The allowed-bit rows of `table` must be 16-byte aligned (they are when
 * the library or torch allocated them).
 * A set-up call: allocates, enqueues on `stream` and waits for it.  Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_table_pack(const tdfa_table *table, void *stream, tdfa_table **out);

/* The arrays of a packed table (any out-pointer may be NULL); INVALID_ARG for a dense table. */
TDFA_API int tdfa_table_pack_info(const tdfa_table *table, int64_t *n_edges, int32_t **targets_dev,
                         int64_t **row_begin_dev, uint32_t **dir_dev, int64_t *dir_row_entries);

/* ---- decode step (Algorithm 2, loop body; Appendix B.2.2) ----------------------------------- */

/* One decoding step for `batch` sequences.  For sequence b in state q = states[b]:
 *     A        = { t : delta_T[q][t] != TDFA_DEAD }                 allowed next tokens
 *     masked   = logits[b][t] for t in A (bit for bit), -inf otherwise   (if masked_out != NULL)
 *     token    = the t in A with the largest logit; the lowest id wins ties; a NaN logit ranks as
 *                -inf, and an allowed token whose logit is -inf or NaN is still chosen when
 *                nothing better is allowed
 *     tokens[b] = token, new_states[b] = delta_T[q][token].
 * If A is empty: tokens[b] = TDFA_NO_TOKEN and new_states[b] = q (the caller checks whether q is
 * final).  If q is TDFA_DEAD or not a row of the table: tokens[b] = TDFA_NO_TOKEN,
 * new_states[b] = TDFA_DEAD, and the masked row is all -inf.  Data never makes a kernel trap.
 *   logits_dev     : device, [batch][row_stride] elements of `dtype` (float, or bf16 bit
 *                    patterns); the first n_tokens of each row are used.  Rows must be 16-byte
 *                    aligned (base pointer and row_stride * element size multiples of 16).
 *   row_stride     : elements between rows, >= n_tokens.
 *   states_dev     : device, int32 [batch].
 *   tokens_dev     : device, int32 [batch], written.
 *   new_states_dev : device, int32 [batch], written; may equal states_dev (in-place advance).
 *   masked_out_dev : device, same shape and type as logits, or NULL to skip the write-back; may
 *                    equal logits_dev.
 * Enqueues on `stream`; steps issued on one stream run in order, so states can be chained from
 * step to step without host synchronisation.  All steps on one device share a small reduction
 * scratch owned by the library, so steps must not overlap in time on different streams of one
 * device.  The scratch is allocated by the first call on a device (room for 4096 sequences) and
 * replaced by a larger one when a larger batch comes; such a call allocates and clears device
 * memory synchronously and therefore fails with UNSUPPORTED inside a stream capture: make one
 * step at the largest batch size before capturing.  Earlier scratch blocks stay allocated, so
 * graphs recorded with them remain valid.  Errors: INVALID_ARG, OOM, DEVICE, UNSUPPORTED. */
TDFA_API int tdfa_mask_step(const tdfa_table *table, const void *logits_dev, int dtype, int32_t batch,
                   int64_t row_stride, const int32_t *states_dev,
                   int32_t *tokens_dev, int32_t *new_states_dev,
                   void *masked_out_dev, void *stream);

/* tdfa_mask_step for callers that cannot allocate device memory or wait for the device: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * results, but the reduction scratch is a fixed array in the library's device image (48 KiB, held
 * by every GPU the library runs on until the process ends) instead of a buffer allocated on demand:
 * the call allocates nothing, frees nothing and does not synchronise.
 *   batch : at most 4096; a larger batch fails with TDFA_E_UNSUPPORTED and launches nothing.
 * All calls on one GPU share the array, which keeps what the last call left in it; each call
 * first clears the words it uses with a small kernel on `stream`.  Calls of this function that
 * overlap in time on one GPU (different streams, or graphs replayed side by side) therefore race;
 * issue them on one stream.  The first call on a GPU looks the array's address up, once; creating
 * any table on that GPU beforehand (every compile and tdfa_table_wrap does) has already done it.
 * Errors: INVALID_ARG, UNSUPPORTED, DEVICE. */
TDFA_API int tdfa_mask_step_noalloc(const tdfa_table *table, const void *logits_dev, int dtype, int32_t batch,
                           int64_t row_stride, const int32_t *states_dev,
                           int32_t *tokens_dev, int32_t *new_states_dev,
                           void *masked_out_dev, void *stream);

/* The same step with SampleNextToken (Algorithm 2) a random draw instead of the greedy choice:
 * the token is distributed as softmax(logits[b] / temperature) restricted to A.  The paper leaves
 * the sampler to the caller; this entry point fuses one into the pass that applies the mask, by
 * the Gumbel-max rule:  token = the t in A with the largest  fma(l_t, 1/temperature, g_t),  the
 * lowest id among equal scores (-0 equals +0), where l_t is the logit as binary32 (NaN counts as
 * -inf) and g_t is standard Gumbel noise.  An integer decided by floating point must be
 * reproducible, so the noise is defined exactly; every operation is one IEEE-754 binary32
 * operation, in this order:
 *     x  = word (t mod 4) of Philox4x32-10 [Salmon, Moraes, Dror, Shaw, SC'11] with
 *          counter = (t div 4, b, low word of offset, high word of offset),
 *          key     = (low word of seed, high word of seed)
 *     u  = fma(float(x >> 9), 2^-23, 2^-24)                      exact; 2^-24 <= u <= 1 - 2^-24
 *     g  = -ln32(-ln32(u))
 *     ln32(x), x positive and normal:  e = exponent of x, m = its significand in [1, 2); if the
 *          fraction field of x exceeds 0x3504F3 (that of sqrt 2): m = m / 2, e = e + 1;
 *          f = m - 1;  s = f / (2 + f);  z = s * s;
 *          p = fma(z, fma(z, fma(z, fma(z, 2/9, 2/7), 2/5), 2/3), 2)   (constants rounded to binary32)
 *          ln32 = fma(float(e), 0x1.62e43p-1 (ln 2), s * p)
 * ln32 is within 3 units in the last place of the logarithm; u has 23 random bits, so g lies in
 * about [-2.82, 16.64]: a tail of probability 2^-24 is cut off at either end.
 * The caller picks `seed` once and a fresh `offset` for every step (the step number, say): the
 * noise of sequence b at a step depends on (seed, offset, b, t) only, not on the batch around it.
 *   temperature : > 0, with a finite binary32 reciprocal; 1 / temperature is rounded once.
 *   top_k       : 0 draws from all of A.  k > 0 draws only from the t in A whose logit is at least
 *                 the k-th largest logit in A (counted with multiplicity, NaN as -inf, -0 = +0):
 *                 tokens tied with the k-th all stay, so more than k may remain; if A has fewer
 *                 than k tokens all stay.  The cut is part of the draw, not of the mask: the
 *                 masked row shows A.
 * Everything else (arguments, layouts, A empty, states that are no row, the masked row, stream
 * and scratch rules, errors) is as for tdfa_mask_step.  An allowed token whose logit is -inf or
 * NaN has probability zero, and is chosen only when no allowed token has a finite or +inf logit
 * (then the lowest allowed id is taken). */
TDFA_API int tdfa_sample_step(const tdfa_table *table, const void *logits_dev, int dtype, int32_t batch,
                     int64_t row_stride, const int32_t *states_dev,
                     float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                     int32_t *tokens_dev, int32_t *new_states_dev,
                     void *masked_out_dev, void *stream);

/* tdfa_sample_step with the offset read by the kernels from device memory (one uint64, 8-byte
 * aligned) when they run, not passed by value when the call is made.  For callers that record
 * their decode loop once and replay it (a HIP graph): the recorded launch keeps its arguments, so
 * a fresh offset per step has to come from memory that the loop itself advances (any kernel of
 * the caller's that adds one to the word between steps will do).  Everything else as above; the
 * result is that of tdfa_sample_step with offset = the word's value when the step runs. */
TDFA_API int tdfa_sample_step_at(const tdfa_table *table, const void *logits_dev, int dtype, int32_t batch,
                        int64_t row_stride, const int32_t *states_dev,
                        float temperature, int32_t top_k, uint64_t seed, const uint64_t *offset_dev,
                        int32_t *tokens_dev, int32_t *new_states_dev,
                        void *masked_out_dev, void *stream);

/* The noise tdfa_sample_step adds, on its own: noise[b][t] = g_t of sequence b for the given seed
 * and offset (definition above), so that a caller can reproduce or audit a draw.
 *   noise_dev : device, float [batch][n_tokens], written.
 * Enqueues on `stream`.  Errors: INVALID_ARG, DEVICE. */
TDFA_API int tdfa_sample_noise(int32_t batch, int32_t n_tokens, uint64_t seed, uint64_t offset,
                      float *noise_dev, void *stream);

/* ---- terminal labels (Section 2.5.1, wildcard matching) -------------------------------------- */

/* Applies terminal edges to a compiled table.  A terminal edge (state, label, target) stands for
 * one edge per token of the label's pre-computed mask; the paper keeps it as one edge because its
 * automata are edge lists.  In the dense table the same behaviour is reached once, here, and
 * the decode step needs nothing new: the whole mask is applied at once because its tokens are
 * simply allowed in the state's row, and a chosen token that lies in the mask takes the
 * terminal edge because its entry holds the edge's target.
 * Where a normal token edge and a terminal edge both match, the normal edge is kept; among
 * terminal edges the one listed first wins (the paper's precedence order).  So, for the edges
 * in the order given: every token of the mask whose entry in the state's row is still
 * TDFA_DEAD gets the edge's target, and its allowed bit is set.
 *   edge_state_host / edge_label_host / edge_target_host : host, int32 [n_edges]; states and
 *                targets are rows of the table (global row ids in a stacked table).
 *   masks_dev  : device, uint32 [n_labels][tdfa_allow_row_words(n_tokens)], bit t & 31 of word
 *                t >> 5 set = token t is in the mask (the layout of the allowed-bit rows).
 * Blocks until the table is updated.  Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_table_apply_terminals(tdfa_table *table, int32_t n_edges, const int32_t *edge_state_host,
                               const int32_t *edge_label_host, const int32_t *edge_target_host,
                               int32_t n_labels, const uint32_t *masks_dev, void *stream);

/* ---- token-level optimisation (Appendix C.2, fourth compile operation) ------------------------ */

/* A smaller table with the same behaviour.  The paper lists the optimisation of the composed
 * automaton as the last compile operation without naming it; this call does the classical one
 * for a deterministic automaton, seen from the given start states:
 *   - states that no token sequence reaches are dropped;
 *   - states from which no final state can be reached are dropped, and edges into them become
 *     TDFA_DEAD (decoding can then never walk into a dead end);
 *   - states that accept the same set of token sequences are merged.
 * The result is the minimal deterministic token automaton of the same language for every start
 * state; its states are numbered by the smallest old state of each class, so the table is unique.
 *   accept_host       : host, uint8 [n_rows], non-zero = final state.
 *   start_states_host : host, int32 [n_starts], rows of the table (one per constraint).
 *   out               : receives the new table (owned by the library); it may have no rows.
 *   state_map_host    : host, int32 [n_rows], written: the new state of every old state, or
 *                       TDFA_DEAD if it was dropped.  A sequence in old state q continues in
 *                       state_map[q].
 *   accept_out_host   : host, uint8 [n_rows] or NULL; the first (new number of rows) entries
 *                       are written.
 * A set-up call: it allocates and frees device memory of its own (a few bytes per distinct target
 * of every row), reads the table twice, waits for a counter after every round of refinement, and
 * blocks until the new table is complete; not to be called under stream capture.  A table whose rows
 * have thousands of distinct targets each takes a slower route that streams the rows in every
 * round.  Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_table_minimize(const tdfa_table *table, const uint8_t *accept_host,
                        const int32_t *start_states_host, int32_t n_starts, void *stream,
                        tdfa_table **out, int32_t *state_map_host, uint8_t *accept_out_host);

/* ---- speculated runs (Section 5.3) ----------------------------------------------------------- */

/* The constraint over a run of k speculated tokens per sequence, with the full history of
 * states, so that the caller can rewind to any prefix when the target model rejects the rest
 * (the paper keeps every state passed through, not only the last).  For sequence b:
 *     history[b][0]     = states[b], or TDFA_DEAD if that is not a row of the table
 *     history[b][i + 1] = delta_T[history[b][i]][tokens[b][i]]; TDFA_DEAD if that edge does not
 *                         exist or tokens[b][i] is not a token id, and TDFA_DEAD from there on
 *     n_valid[b]        = number of leading tokens the constraint accepts (history[b][1 ..
 *                         n_valid[b]] are live, the rest is TDFA_DEAD).
 * The penalties for the target model are those of the history states: one tdfa_mask_step call
 * over batch * (k + 1) rows with states_dev = history_dev masks the target's logits at every
 * position (and the allowed-bit row of state q is row q of allow_dev, see tdfa_table_info), so
 * nothing is evaluated twice.
 *   states_dev  : device, int32 [batch].
 *   tokens_dev  : device, int32 [batch * k], the run of sequence b at b * k.
 *   history_dev : device, int32 [batch * (k + 1)], written.
 *   n_valid_dev : device, int32 [batch], written; may be NULL.
 * batch >= 0, k >= 0.  Enqueues on `stream`.  Errors: INVALID_ARG, DEVICE. */
TDFA_API int tdfa_advance_tokens(const tdfa_table *table, int32_t batch, int32_t k, const int32_t *states_dev,
                        const int32_t *tokens_dev, int32_t *history_dev, int32_t *n_valid_dev,
                        void *stream);

/* ---- push-down constraints (Section 3; Algorithm 3) ------------------------------------------- */

/* A character-level push-down automaton P_G (Section 3.1) and the token-accepting automaton
 * P_{G o V} = P_G o T_V made from it (Section 3.2).  Stack strings are written bottom to top: a
 * stack "ends with" the pops of an edge when its topmost symbols are those, in that order.  How
 * P_G is made from a grammar is the caller's business (Algorithm 3, BuildGrammarPDA). */
typedef struct tdfa_pda    tdfa_pda;      /* P_G, resident on the device */
typedef struct tdfa_ptable tdfa_ptable;   /* the token edges of P_{G o V} */

#define TDFA_PDA_STRING 12   /* most symbols an edge, of P_G or of P_{G o V}, may pop or push */

/* Uploads P_G.  Edge e is (src[e], input[e], pops, dst[e], pushes) with
 * pops = pop_syms[pop_begin[e] .. pop_begin[e+1]) and pushes = push_syms[push_begin[e] ..
 * push_begin[e+1]); it can be taken in state src[e] when the input is input[e] and the stack ends
 * with pops, which are then removed and pushes appended.
 *   src, input, dst       : host, int32 [n_edges], sorted by src; input is a byte 0 .. 255 or -1 (epsilon).
 *   pop_begin, push_begin : host, int32 [n_edges + 1], starting at 0; at most TDFA_PDA_STRING symbols per edge.
 *   pop_syms, push_syms   : host, int32, symbols >= 0.
 *   accept                : host, uint8 [n_states] or NULL; kept for the caller, not read by the kernels.
 * The automaton must be deterministic (Section 3.1: a non-deterministic one is an error, there is
 * no way to determinize it): of two edges of one state whose inputs can meet (equal, or one of
 * them epsilon) neither's pops may be a suffix of the other's.  The check is made here; the error
 * message names the two edges.  Blocks until the device copy is complete.
 * Errors: INVALID_ARG, OOM, DEVICE. */
TDFA_API int tdfa_pda_create(int32_t n_states, int32_t start, const uint8_t *accept, int32_t n_edges,
                    const int32_t *src, const int32_t *input, const int32_t *dst,
                    const int32_t *pop_begin, const int32_t *pop_syms,
                    const int32_t *push_begin, const int32_t *push_syms, void *stream, tdfa_pda **out);
TDFA_API int tdfa_pda_destroy(tdfa_pda *pda);

/* Algorithm 3, third statement: the token edges of P_G o T_V.  For state q and token t there is one
 * token edge per run of P_G from q over the bytes of t; epsilon edges are taken with the byte that
 * follows them and a token edge ends with the token's last byte, so whether a configuration accepts
 * is asked after the epsilon edges that can still be taken (the caller's check, as with final
 * states of tables).  The stack edits on the way are concatenated: the edge's pops are what the
 * stack must end with for the whole run, its pushes what the run leaves in their place; a token
 * that crosses the boundary of a non-terminal pops or pushes several symbols (Fig. 7).  The states
 * of P_{G o V} are those of P_G.  The edges are stored sorted by (state, token):
 *     edge_first : device, int64 [n_states + 1]; state q owns edges edge_first[q] .. edge_first[q+1] - 1
 *     token, dst, n_pops, n_push : device, int32 [n_edges]
 *     pops, pushes               : device, int32 [n_edges][TDFA_PDA_STRING], unused places -1
 * A set-up call: runs its kernels on `stream` and waits for them (the number of edges sizes the
 * arrays).  Errors: INVALID_ARG, OOM, DEVICE; UNSUPPORTED when a token edge would pop or push more
 * than TDFA_PDA_STRING symbols, a run takes more than 64 epsilon edges in a row, or one state and
 * token have more than 8 runs open at once. */
TDFA_API int tdfa_compile_token_pda(const tdfa_vocab *vocab, const tdfa_pda *pda, void *stream, tdfa_ptable **out);
TDFA_API int tdfa_ptable_info(const tdfa_ptable *table, int32_t *n_states, int32_t *n_tokens, int64_t *n_edges,
                     int64_t **edge_first_dev, int32_t **token_dev, int32_t **dst_dev, int32_t **n_pops_dev,
                     int32_t **pops_dev, int32_t **n_push_dev, int32_t **pushes_dev);
TDFA_API int tdfa_ptable_destroy(tdfa_ptable *table);

/* The loop body of Algorithm 3 for `batch` sequences.  For sequence b in state q = states[b] with
 * stack s = stacks[b][0 .. depths[b]) (bottom to top):
 *     A      = { token(e) : e leaves q and s ends with pops(e) }
 *     masked = logits[b][t] for t in A, -inf otherwise                       (if masked_out != NULL)
 *     token  = the t in A with the largest logit (ties, NaN, -0: as tdfa_mask_step)
 *     e      = the edge of q with that token whose pops s ends with
 *     new_states[b] = dst(e);  s loses pops(e) and gains pushes(e);  depths[b] follows.
 * A empty: tokens[b] = TDFA_NO_TOKEN, state and stack stay.  q no state of the table, or depths[b]
 * outside [0, stack_cap]: TDFA_NO_TOKEN, new state TDFA_DEAD, masked row all -inf.  If the chosen
 * edge would leave more than stack_cap symbols on the stack: TDFA_NO_TOKEN, TDFA_DEAD, stack left
 * as it was.
 *   logits_dev, dtype, row_stride, tokens_dev, new_states_dev : as tdfa_mask_step (no alignment demanded;
 *                 with rows that are 16-byte aligned the step runs the kernels of tdfa_mask_step: on
 *                 16-bit logits without masked_out the kernel itself ORs the rows of allowed bits of the
 *                 state's edges that the stack matches, otherwise one such row per sequence is made
 *                 first; with other rows it scans the edges of each sequence's state).
 *   stacks_dev  : device, int32 [batch][stack_cap], updated in place.
 *   depths_dev  : device, int32 [batch], updated in place.
 *   masked_out_dev : device or NULL; must not be logits_dev.
 * new_states_dev may equal states_dev.  Enqueues on `stream`.  The table keeps the per-sequence rows of
 * allowed bits (batch x |V| / 8 bytes) and allocates them on the first step at a larger batch than any
 * before: make that call before capturing the stream into a graph (under capture it is refused with
 * UNSUPPORTED); steps on one table that overlap in time share those rows and race.
 * Errors: INVALID_ARG, DEVICE, OOM, UNSUPPORTED. */
TDFA_API int tdfa_pda_step(const tdfa_ptable *table, const void *logits_dev, int dtype, int32_t batch,
                  int64_t row_stride, const int32_t *states_dev, int32_t *stacks_dev, int32_t *depths_dev,
                  int32_t stack_cap, int32_t *tokens_dev, int32_t *new_states_dev, void *masked_out_dev,
                  void *stream);

/* tdfa_pda_step with the token drawn instead of taken greedily (Algorithm 3 calls the language
 * model's sampler for its token as Algorithm 2 does; Section 3.2): the allowed set A as there,
 * the token drawn from softmax(logits / temperature) over A by the rule of tdfa_sample_step
 * (temperature, top_k, seed, offset as there; sequence b and token t use the noise of (seed, offset,
 * b, t)), then the edge of that token is traversed.  Same results as tdfa_pda_step for every other
 * case (A empty, states that are no state, a stack that would outgrow stack_cap).
 * Runs on one row of allowed bits per sequence (made from the table's rows per class of edges, or
 * edge by edge for a table with more than 64 classes in a state): the rows of logits must be
 * 16-byte aligned, else UNSUPPORTED.  Allocation and capture as tdfa_pda_step.
 * Errors: INVALID_ARG, DEVICE, OOM, UNSUPPORTED. */
TDFA_API int tdfa_pda_sample_step(const tdfa_ptable *table, const void *logits_dev, int dtype, int32_t batch,
                         int64_t row_stride, const int32_t *states_dev, int32_t *stacks_dev, int32_t *depths_dev,
                         int32_t stack_cap, float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                         int32_t *tokens_dev, int32_t *new_states_dev, void *masked_out_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TDFA_H_ */
