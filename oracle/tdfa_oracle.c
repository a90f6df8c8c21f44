/*
 * CPU oracle for token-level constraint automata and the constrained decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the tests,
 * the smoke check and the benchmark's CPU-baseline leg compare the GPU library
 * against.  It shares no code with the GPU library and the library never calls it.
 *
 * What it follows (arXiv 2407.08103):
 *   - Algorithm 1 (Section 2.3): the detokenizing transducer T_V, built in its
 *     original chain form, one private cycle through the root per token.
 *   - Section 2.2 (composition of an FST with an FSA) and Section 2.4 / Algorithm 2,
 *     third statement: A_{R o V} = Determinize(A_R o T_V).  The composition is done
 *     explicitly over pair states; epsilon-input edges are then removed by closure.
 *   - Algorithm 2, decoding loop (allowed set, -inf penalty, token choice, edge
 *     traversal) and Appendix B.2.2 (unmasked logits are left untouched).
 *
 * Readings of points the paper leaves open (the same list is in the design notes):
 *   - alphabet = bytes; DEAD / "no token" = -1; all states of A_R get a row, also
 *     those no token sequence reaches; no renumbering or minimisation of the result;
 *   - a zero-length token has no cycle in T_V (Algorithm 1's closing edge needs a
 *     last character), so it is never allowed;
 *   - SampleNextToken = greedy argmax (orc_mask_step) or a draw from softmax(l / T)
 *     over the allowed set by the Gumbel-max rule (orc_sample_step, defined operation
 *     by operation above it); ties go to the lowest token id; a NaN logit ranks as
 *     -inf; an allowed token whose logit is -inf or NaN can still be chosen when
 *     nothing better is allowed;
 *   - a live state with no allowed token yields token -1 and keeps its state; a DEAD
 *     or out-of-range state yields token -1 and state DEAD.
 *
 * Every function here is pinned by tests/test_oracle_*.py (the paper's worked
 * examples, brute force against an independent regex engine, Theorem 1, invariants,
 * closed forms).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_DEAD (-1)
#define ORC_EPS  (-1)            /* epsilon label on either side of an FST edge */
#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_MEM (-2)
#define ORC_E_NONDET (-3)        /* two different targets for one (state, token) */
#define ORC_E_STRUCT (-4)        /* composed automaton does not have the expected shape */

/* ------------------------------------------------------------------ FST T_V (Algorithm 1) */

typedef struct { int32_t src, in, out, dst; } orc_fst_edge;

typedef struct {
    int32_t n_states;            /* |Q_V| */
    int32_t root;                /* q_r = I_V, F_V = {q_r} */
    int64_t n_edges;
    orc_fst_edge *edges;         /* E_V, in construction order */
} orc_fst;

void orc_fst_free(orc_fst *t) { if (t) { free(t->edges); t->edges = NULL; t->n_edges = 0; } }

/* The detokenizing transducer T_V of Section 2.3 (the one Algorithm 1 constructs), written out
 * from what it is: one root state, initial and final; every token v with bytes b_0 .. b_{n-1}
 * is a cycle of n edges from the root back to the root whose outputs spell b_0 .. b_{n-1}, whose
 * last edge reads v and whose other edges read nothing.  The cycles share only the root, so
 * token v owns n - 1 inner states; they are numbered after the root in token order, which makes
 * the first inner state of v the sum of (len - 1) over the tokens before it, plus one.  A token
 * without bytes has no last edge to read it on and gets no cycle.
 * Token v = bytes[offsets[v] .. offsets[v+1]).  Input labels are token ids, output labels bytes. */
int orc_build_detok_fst(const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens, orc_fst *out)
{
    if (!offsets || !out || n_tokens < 0) return ORC_E_ARG;
    int64_t total = 0;
    for (int32_t v = 0; v < n_tokens; ++v) {
        if (offsets[v + 1] < offsets[v]) return ORC_E_ARG;
        total += (int64_t)(offsets[v + 1] - offsets[v]);
    }
    if (total > 0 && !bytes) return ORC_E_ARG;
    out->edges = (orc_fst_edge *)malloc(sizeof(orc_fst_edge) * (size_t)(total > 0 ? total : 1));
    if (!out->edges) return ORC_E_MEM;
    out->root = 0;
    int64_t inner_before = 0;                       /* inner states of the tokens before v */
    for (int32_t v = 0; v < n_tokens; ++v) {
        const int64_t n = (int64_t)(offsets[v + 1] - offsets[v]);
        const int64_t first_inner = 1 + inner_before;
        /* the edge that outputs byte k of v is edge offsets[v] + k of the transducer */
        for (int64_t k = 0; k < n; ++k) {
            orc_fst_edge *e = &out->edges[(int64_t)offsets[v] - (int64_t)offsets[0] + k];
            e->src = k == 0 ? out->root : (int32_t)(first_inner + k - 1);
            e->dst = k == n - 1 ? out->root : (int32_t)(first_inner + k);
            e->in = k == n - 1 ? v : ORC_EPS;
            e->out = (int32_t)bytes[offsets[v] + (uint64_t)k];
        }
        if (n > 0) inner_before += n - 1;
    }
    out->n_states = (int32_t)(1 + inner_before);
    out->n_edges = total;
    return ORC_OK;
}

/* Transduce a token sequence with T_V by exhaustive search over edge paths (Section 2.2:
 * a path from I to F whose input labels spell x; its output labels spell the result).
 * Returns the output length, -1 if no path accepts, -2 if two paths give different
 * outputs, -3 if out_cap is too small.  Meant for small cases (Theorem 1 checks). */
typedef struct { int32_t state; int32_t pos; int64_t next_edge; int32_t out_len; } orc_frame;

int64_t orc_fst_transduce(const orc_fst *t, const int32_t *x, int32_t n, uint8_t *out, int64_t out_cap)
{
    /* out-edges by source state */
    int64_t *first = (int64_t *)calloc((size_t)t->n_states + 1, sizeof(int64_t));
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)(t->n_edges ? t->n_edges : 1));
    for (int64_t e = 0; e < t->n_edges; ++e) first[t->edges[e].src + 1]++;
    for (int32_t s = 0; s < t->n_states; ++s) first[s + 1] += first[s];
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * ((size_t)t->n_states + 1));
    memcpy(fill, first, sizeof(int64_t) * ((size_t)t->n_states + 1));
    for (int64_t e = 0; e < t->n_edges; ++e) order[fill[t->edges[e].src]++] = e;
    free(fill);

    int64_t cap = 64, depth = 0, found = -1;
    orc_frame *st = (orc_frame *)malloc(sizeof(orc_frame) * (size_t)cap);
    uint8_t *cur = (uint8_t *)malloc((size_t)(out_cap > 0 ? out_cap : 1) + 1);
    uint8_t *best = (uint8_t *)malloc((size_t)(out_cap > 0 ? out_cap : 1) + 1);
    int64_t rc = -1;
    st[depth++] = (orc_frame){ t->root, 0, first[t->root], 0 };
    while (depth > 0) {
        orc_frame *f = &st[depth - 1];
        if (f->next_edge == first[f->state]) {     /* first visit of this configuration */
            if (f->state == t->root && f->pos == n) {
                if (found < 0) { found = f->out_len; memcpy(best, cur, (size_t)found); }
                else if (found != f->out_len || memcmp(best, cur, (size_t)found)) { rc = -2; goto done; }
            }
        }
        if (f->next_edge >= first[f->state + 1]) { depth--; continue; }
        const orc_fst_edge *e = &t->edges[order[f->next_edge++]];
        int32_t pos = f->pos, out_len = f->out_len;
        if (e->in != ORC_EPS) {
            if (pos >= n || x[pos] != e->in) continue;
            pos++;
        }
        if (e->out != ORC_EPS) {
            if (out_len >= out_cap) { rc = -3; goto done; }
            cur[out_len++] = (uint8_t)e->out;
        }
        if (depth == cap) { cap *= 2; st = (orc_frame *)realloc(st, sizeof(orc_frame) * (size_t)cap); }
        st[depth++] = (orc_frame){ e->dst, pos, first[e->dst], out_len };
    }
    rc = found;
    if (found >= 0) memcpy(out, best, (size_t)found);
done:
    free(st); free(cur); free(best); free(first); free(order);
    return rc;
}

/* ------------------------------------------------------------------ FSA view of the char DFA */

typedef struct { int32_t src, label, dst; } orc_fsa_edge;

typedef struct {
    int32_t n_states;
    int64_t n_edges;
    orc_fsa_edge *edges;         /* E of A_R: one per defined (state, byte) */
    int64_t *by_src_label;       /* [n_states*256] edge id or -1: lookup index over E */
} orc_fsa;

static void orc_fsa_free(orc_fsa *a) { free(a->edges); free(a->by_src_label); a->edges = NULL; a->by_src_label = NULL; }

static int orc_fsa_from_table(const int32_t *trans, int32_t n_states, orc_fsa *a)
{
    if (!trans || n_states <= 0) return ORC_E_ARG;
    int64_t ne = 0;
    for (int64_t i = 0; i < (int64_t)n_states * 256; ++i) {
        if (trans[i] < ORC_DEAD || trans[i] >= n_states) return ORC_E_ARG;
        if (trans[i] != ORC_DEAD) ne++;
    }
    a->n_states = n_states;
    a->n_edges = ne;
    a->edges = (orc_fsa_edge *)malloc(sizeof(orc_fsa_edge) * (size_t)(ne ? ne : 1));
    a->by_src_label = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_states * 256);
    if (!a->edges || !a->by_src_label) { orc_fsa_free(a); return ORC_E_MEM; }
    ne = 0;
    for (int32_t q = 0; q < n_states; ++q)
        for (int32_t b = 0; b < 256; ++b) {
            int32_t d = trans[(int64_t)q * 256 + b];
            a->by_src_label[(int64_t)q * 256 + b] = -1;
            if (d != ORC_DEAD) {
                a->edges[ne] = (orc_fsa_edge){ q, b, d };
                a->by_src_label[(int64_t)q * 256 + b] = ne++;
            }
        }
    return ORC_OK;
}

/* ------------------------------------------------------------------ composition A_R o T_V */

/* Composed automaton over pair states (a, u), a in Q of A_R, u in Q_V.  Pairs are numbered
 * in discovery order; the out-edges of pair p are edges[first_edge[p] .. first_edge[p+1]). */
typedef struct {
    int64_t n_pairs, cap_pairs;
    int32_t *pa, *pu;
    int64_t *first_edge;         /* [n_pairs + 1] once expanded */
    int64_t n_edges, cap_edges;
    int32_t *e_in;               /* token id or ORC_EPS */
    int64_t *e_dst;              /* pair id */
    /* visited set: open addressing on key = a * |Q_V| + u */
    uint64_t *h_key; int64_t *h_val; uint64_t h_cap, h_used;
} orc_comp;

static void orc_comp_free(orc_comp *c)
{
    free(c->pa); free(c->pu); free(c->first_edge); free(c->e_in); free(c->e_dst);
    free(c->h_key); free(c->h_val);
    memset(c, 0, sizeof(*c));
}

static uint64_t orc_hash64(uint64_t k) { k ^= k >> 33; k *= 0xff51afd7ed558ccdULL; k ^= k >> 33; k *= 0xc4ceb9fe1a85ec53ULL; k ^= k >> 33; return k; }

static int orc_comp_rehash(orc_comp *c, uint64_t new_cap)
{
    uint64_t *nk = (uint64_t *)malloc(sizeof(uint64_t) * new_cap);
    int64_t *nv = (int64_t *)malloc(sizeof(int64_t) * new_cap);
    if (!nk || !nv) { free(nk); free(nv); return ORC_E_MEM; }
    for (uint64_t i = 0; i < new_cap; ++i) nv[i] = -1;
    for (uint64_t i = 0; i < c->h_cap; ++i)
        if (c->h_val[i] >= 0) {
            uint64_t j = orc_hash64(c->h_key[i]) & (new_cap - 1);
            while (nv[j] >= 0) j = (j + 1) & (new_cap - 1);
            nk[j] = c->h_key[i]; nv[j] = c->h_val[i];
        }
    free(c->h_key); free(c->h_val);
    c->h_key = nk; c->h_val = nv; c->h_cap = new_cap;
    return ORC_OK;
}

/* id of pair (a, u), adding it to the state set if new; < 0 on allocation failure */
static int64_t orc_comp_pair(orc_comp *c, int32_t a, int32_t u, uint64_t n_fst_states)
{
    uint64_t key = (uint64_t)a * n_fst_states + (uint64_t)u;
    if (c->h_cap == 0 || (c->h_used + 1) * 10 > c->h_cap * 6)
        if (orc_comp_rehash(c, c->h_cap ? c->h_cap * 2 : 1024) != ORC_OK) return ORC_E_MEM;
    uint64_t j = orc_hash64(key) & (c->h_cap - 1);
    while (c->h_val[j] >= 0) {
        if (c->h_key[j] == key) return c->h_val[j];
        j = (j + 1) & (c->h_cap - 1);
    }
    if (c->n_pairs == c->cap_pairs) {
        int64_t nc = c->cap_pairs ? c->cap_pairs * 2 : 1024;
        int32_t *npa = (int32_t *)realloc(c->pa, sizeof(int32_t) * (size_t)nc);
        if (!npa) return ORC_E_MEM;
        c->pa = npa;
        int32_t *npu = (int32_t *)realloc(c->pu, sizeof(int32_t) * (size_t)nc);
        if (!npu) return ORC_E_MEM;
        c->pu = npu;
        int64_t *nfe = (int64_t *)realloc(c->first_edge, sizeof(int64_t) * (size_t)(nc + 1));
        if (!nfe) return ORC_E_MEM;
        c->first_edge = nfe;
        c->cap_pairs = nc;
    }
    int64_t id = c->n_pairs++;
    c->pa[id] = a; c->pu[id] = u;
    c->h_key[j] = key; c->h_val[j] = id; c->h_used++;
    return id;
}

/* Section 2.2: A' = A o T.  For every FST edge (u, in, out, u') and FSA edge (a, out, a')
 * with the same symbol, A' has the edge ((a,u), in, (a',u')); an FST edge with no output
 * leaves the FSA where it is.  Pairs are built from the seeds (q, q_r), q in [q_lo, q_hi), in
 * discovery order (worklist).  A pair (a, q_r) that is not one of this block's seeds is kept
 * as an edge target but not expanded: its out-edges are the row of state a, which belongs to
 * the block that seeds a.  The union over blocks is the whole composed automaton. */
static int orc_compose(const orc_fsa *A, const orc_fst *T, const int64_t *fst_first,
                       const int64_t *fst_order, int32_t q_lo, int32_t q_hi, orc_comp *c)
{
    memset(c, 0, sizeof(*c));
    for (int32_t q = q_lo; q < q_hi; ++q)
        if (orc_comp_pair(c, q, T->root, (uint64_t)T->n_states) < 0) return ORC_E_MEM;
    const int64_t n_seeds = c->n_pairs;
    for (int64_t p = 0; p < c->n_pairs; ++p) {           /* c->n_pairs grows as we go */
        int32_t a = c->pa[p], u = c->pu[p];
        c->first_edge[p] = c->n_edges;
        if (u == T->root && p >= n_seeds) continue;       /* another block's seed */
        for (int64_t k = fst_first[u]; k < fst_first[u + 1]; ++k) {
            const orc_fst_edge *te = &T->edges[fst_order[k]];
            int32_t a2;
            if (te->out == ORC_EPS) a2 = a;
            else {
                int64_t ae = A->by_src_label[(int64_t)a * 256 + te->out];
                if (ae < 0) continue;                     /* no FSA edge reads this symbol */
                a2 = A->edges[ae].dst;
            }
            int64_t d = orc_comp_pair(c, a2, te->dst, (uint64_t)T->n_states);
            if (d < 0) return ORC_E_MEM;
            if (c->n_edges == c->cap_edges) {
                int64_t nc = c->cap_edges ? c->cap_edges * 2 : 4096;
                int32_t *ni = (int32_t *)realloc(c->e_in, sizeof(int32_t) * (size_t)nc);
                if (!ni) return ORC_E_MEM;
                c->e_in = ni;
                int64_t *nd = (int64_t *)realloc(c->e_dst, sizeof(int64_t) * (size_t)nc);
                if (!nd) return ORC_E_MEM;
                c->e_dst = nd;
                c->cap_edges = nc;
            }
            c->e_in[c->n_edges] = te->in;
            c->e_dst[c->n_edges] = d;
            c->n_edges++;
        }
    }
    c->first_edge[c->n_pairs] = c->n_edges;
    return ORC_OK;
}

/* Epsilon removal (the Determinize of Algorithm 2 when A_R is already deterministic):
 * from (q, q_r) follow epsilon-input edges; every token-labelled edge met on the way must
 * lead back to some (q', q_r) and gives delta_T[q][token] = q'.  A second, different
 * target for the same (q, token) would need subset construction: reported as an error. */
static int orc_close_rows(const orc_comp *c, const orc_fst *T, int32_t q_lo, int32_t q_hi,
                          int32_t n_tokens, int32_t *rows /* [(q_hi-q_lo) * n_tokens], pre-filled DEAD */)
{
    int64_t cap = 1024, top;
    int64_t *stack = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
    if (!stack) return ORC_E_MEM;
    int rc = ORC_OK;
    for (int32_t q = q_lo; q < q_hi && rc == ORC_OK; ++q) {
        int32_t *row = rows + (int64_t)(q - q_lo) * n_tokens;
        top = 0;
        stack[top++] = (int64_t)(q - q_lo);               /* seeds were numbered first, in order */
        if (c->pa[q - q_lo] != q || c->pu[q - q_lo] != T->root) { rc = ORC_E_STRUCT; break; }
        while (top > 0) {
            int64_t p = stack[--top];
            for (int64_t e = c->first_edge[p]; e < c->first_edge[p + 1]; ++e) {
                int64_t d = c->e_dst[e];
                if (c->e_in[e] == ORC_EPS) {
                    if (top == cap) {
                        cap *= 2;
                        int64_t *ns = (int64_t *)realloc(stack, sizeof(int64_t) * (size_t)cap);
                        if (!ns) { rc = ORC_E_MEM; goto out; }
                        stack = ns;
                    }
                    stack[top++] = d;
                } else {
                    int32_t tok = c->e_in[e];
                    if (tok < 0 || tok >= n_tokens || c->pu[d] != T->root) { rc = ORC_E_STRUCT; goto out; }
                    if (row[tok] != ORC_DEAD && row[tok] != c->pa[d]) { rc = ORC_E_NONDET; goto out; }
                    row[tok] = c->pa[d];
                }
            }
        }
    }
out:
    free(stack);
    return rc;
}

/* delta_T rows [q_lo, q_hi) by the paper's construction: T_V (Algorithm 1), composition,
 * epsilon removal.  `out` is [(q_hi - q_lo) * n_tokens] int32.  Source states are handled
 * in blocks of `block` (each block composes only what its seeds reach, so memory stays
 * bounded); blocks are spread over `n_threads` threads.  Returns ORC_OK or an error. */
int orc_compile_compose(const int32_t *trans, int32_t n_states,
                        const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens,
                        int32_t q_lo, int32_t q_hi, int32_t block, int32_t n_threads, int32_t *out)
{
    if (!out || q_lo < 0 || q_hi > n_states || q_lo > q_hi || block <= 0) return ORC_E_ARG;
    orc_fsa A; memset(&A, 0, sizeof(A));
    orc_fst T; memset(&T, 0, sizeof(T));
    int rc = orc_fsa_from_table(trans, n_states, &A);
    if (rc != ORC_OK) return rc;
    rc = orc_build_detok_fst(bytes, offsets, n_tokens, &T);
    if (rc != ORC_OK) { orc_fsa_free(&A); return rc; }

    int64_t *first = (int64_t *)calloc((size_t)T.n_states + 1, sizeof(int64_t));
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)(T.n_edges ? T.n_edges : 1));
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * ((size_t)T.n_states + 1));
    if (!first || !order || !fill) { free(first); free(order); free(fill); orc_fsa_free(&A); orc_fst_free(&T); return ORC_E_MEM; }
    for (int64_t e = 0; e < T.n_edges; ++e) first[T.edges[e].src + 1]++;
    for (int32_t s = 0; s < T.n_states; ++s) first[s + 1] += first[s];
    memcpy(fill, first, sizeof(int64_t) * ((size_t)T.n_states + 1));
    for (int64_t e = 0; e < T.n_edges; ++e) order[fill[T.edges[e].src]++] = e;
    free(fill);

    for (int64_t i = 0; i < (int64_t)(q_hi - q_lo) * n_tokens; ++i) out[i] = ORC_DEAD;
    int32_t n_blocks = (q_hi - q_lo + block - 1) / block;
    int err = ORC_OK;
    if (n_threads < 1) n_threads = 1;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int32_t b = 0; b < n_blocks; ++b) {
        int32_t lo = q_lo + b * block, hi = lo + block < q_hi ? lo + block : q_hi;
        orc_comp c;
        int r = orc_compose(&A, &T, first, order, lo, hi, &c);
        if (r == ORC_OK) r = orc_close_rows(&c, &T, lo, hi, n_tokens, out + (int64_t)(lo - q_lo) * n_tokens);
        orc_comp_free(&c);
        if (r != ORC_OK) {
#ifdef _OPENMP
#pragma omp critical
#endif
            err = r;
        }
    }
    free(first); free(order);
    orc_fsa_free(&A); orc_fst_free(&T);
    return err;
}

/* Closed form of the same table (what the composition must equal by Theorems 1 and 2):
 * delta_T[q][t] = delta*(q, d(t)), DEAD at the first missing transition; a zero-length
 * token is DEAD everywhere.  A second, independent route to the table. */
int orc_compile_walk(const int32_t *trans, int32_t n_states,
                     const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens,
                     int32_t q_lo, int32_t q_hi, int32_t n_threads, int32_t *out)
{
    if (!trans || !offsets || !out || q_lo < 0 || q_hi > n_states || q_lo > q_hi) return ORC_E_ARG;
    if (n_threads < 1) n_threads = 1;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(n_threads)
#endif
    for (int32_t q = q_lo; q < q_hi; ++q) {
        int32_t *row = out + (int64_t)(q - q_lo) * n_tokens;
        for (int32_t t = 0; t < n_tokens; ++t) {
            int32_t s = q;
            uint64_t lo = offsets[t], hi = offsets[t + 1];
            if (lo == hi) s = ORC_DEAD;
            for (uint64_t i = lo; i < hi && s != ORC_DEAD; ++i) s = trans[(int64_t)s * 256 + bytes[i]];
            row[t] = s;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ decode step (Algorithm 2) */

#define ORC_F32 0
#define ORC_BF16 1

static double orc_logit(const void *logits, int dtype, int64_t i)
{
    float f;
    if (dtype == ORC_F32) f = ((const float *)logits)[i];
    else { uint32_t w = (uint32_t)((const uint16_t *)logits)[i] << 16; memcpy(&f, &w, 4); }
    return isnan(f) ? -INFINITY : (double)f;
}

/* One decoding step for `batch` sequences (loop body of Algorithm 2 after ComputeLogits):
 *   A = tokens with an edge out of the current state  (table[state][t] != DEAD)
 *   l_t <- -inf for t not in A; the others are left bit-for-bit
 *   token = argmax over A (lowest id on ties), new state = table[state][token].
 * table is [n_rows * n_tokens]; logits row b starts at element b * row_stride.
 * masked_out (may be NULL) has the same layout and element type as logits.  Sequences are
 * independent; n_threads > 1 only spreads them over threads. */
int orc_mask_step(const int32_t *table, int64_t n_rows, int32_t n_tokens,
                  const void *logits, int dtype, int32_t batch, int64_t row_stride,
                  const int32_t *states, int32_t *tokens, int32_t *new_states, void *masked_out,
                  int32_t n_threads)
{
    if (!table || !logits || !states || !tokens || !new_states || batch < 0 || n_tokens < 0) return ORC_E_ARG;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return ORC_E_ARG;
    if (n_threads < 1) n_threads = 1;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(n_threads)
#endif
    for (int32_t b = 0; b < batch; ++b) {
        int32_t q = states[b];
        int valid = (q >= 0 && (int64_t)q < n_rows);
        const int32_t *row = valid ? table + (int64_t)q * n_tokens : NULL;
        int32_t best = -1;
        double best_v = 0.0;
        for (int32_t t = 0; t < n_tokens; ++t) {
            int64_t i = (int64_t)b * row_stride + t;
            int allowed = valid && row[t] != ORC_DEAD;
            if (masked_out) {
                if (dtype == ORC_F32) ((uint32_t *)masked_out)[i] = allowed ? ((const uint32_t *)logits)[i] : 0xFF800000u;
                else ((uint16_t *)masked_out)[i] = allowed ? ((const uint16_t *)logits)[i] : (uint16_t)0xFF80u;
            }
            if (!allowed) continue;
            double v = orc_logit(logits, dtype, i);
            if (best < 0 || v > best_v) { best = t; best_v = v; }
        }
        tokens[b] = best;
        new_states[b] = !valid ? ORC_DEAD : (best < 0 ? q : row[best]);
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * SampleNextToken of Algorithm 2 as a draw from softmax(l / T) over the allowed set.
 *
 * The paper leaves the sampler open.  The reading taken here is the Gumbel-max rule: with
 * independent standard Gumbel variates g_t, argmax_t (l_t / T + g_t) over the allowed tokens is
 * distributed as softmax(l / T) restricted to them.  Because the result is an integer decided by
 * floating point, every operation below is a single IEEE-754 binary32 operation (add, multiply,
 * divide, fused multiply-add), in this order, so that any conforming implementation chooses the
 * same token:
 *
 *   x      = word (t mod 4) of Philox4x32-10(counter = (t div 4, b, offset_lo, offset_hi),
 *                                            key = (seed_lo, seed_hi))            [Salmon et al. 2011]
 *   u      = ((x >> 9) + 1/2) * 2^-23            exact; 2^-24 <= u <= 1 - 2^-24
 *   g      = -ln32(-ln32(u))
 *   score  = fma(l_t, 1 / T, g)                  1 / T rounded once; NaN logits count as -inf
 *   token  = allowed token of largest score, lowest id among equals (-0 equals +0)
 *
 * ln32(x), x positive and normal:  x = 2^e * m with m in (sqrt(1/2), sqrt(2)]  (m is taken from
 * the significand, halved when its fraction field exceeds that of sqrt(2));  f = m - 1 (exact);
 * s = f / (2 + f);  z = s * s;  ln m = 2 atanh(s) = s * (2 + z (2/3 + z (2/5 + z (2/7 + z 2/9))))
 * by Horner's rule in fused multiply-adds;  ln32 = fma(e, ln 2, ln m).
 * ------------------------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

float orc_ln32(float x)
{
    uint32_t i;
    memcpy(&i, &x, 4);
    int32_t e = (int32_t)(i >> 23) - 127;
    uint32_t frac = i & 0x7FFFFFu, mi = frac | 0x3F800000u;
    float m;
    memcpy(&m, &mi, 4);
    if (frac > 0x3504F3u) { m = m * 0.5f; e += 1; }          /* 0x3504F3: fraction field of sqrt(2) */
    float f = m - 1.0f;
    float s = f / (2.0f + f);
    float z = s * s;
    float p = fmaf(z, 2.0f / 9.0f, 2.0f / 7.0f);
    p = fmaf(z, p, 2.0f / 5.0f);
    p = fmaf(z, p, 2.0f / 3.0f);
    p = fmaf(z, p, 2.0f);
    return fmaf((float)e, 0.693147180559945309f, s * p);
}

float orc_uniform(uint64_t seed, uint64_t offset, int32_t b, int32_t t)
{
    uint32_t ctr[4] = {(uint32_t)t >> 2, (uint32_t)b, (uint32_t)offset, (uint32_t)(offset >> 32)};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)}, w[4];
    orc_philox4x32_10(ctr, key, w);
    return fmaf((float)(w[t & 3] >> 9), 0x1p-23f, 0x1p-24f);
}

float orc_gumbel(uint64_t seed, uint64_t offset, int32_t b, int32_t t)
{
    return -orc_ln32(-orc_ln32(orc_uniform(seed, offset, b, t)));
}

/* g as a function of the generator word, for words x[0 .. n). */
int orc_gumbel_of_words(const uint32_t *x, int64_t n, float *out)
{
    if (n < 0 || (n > 0 && (!x || !out))) return ORC_E_ARG;
    for (int64_t i = 0; i < n; ++i) {
        float u = fmaf((float)(x[i] >> 9), 0x1p-23f, 0x1p-24f);
        out[i] = -orc_ln32(-orc_ln32(u));
    }
    return ORC_OK;
}

/* g for every token of every sequence: out[b][t]. */
int orc_sample_noise(int32_t batch, int32_t n_tokens, uint64_t seed, uint64_t offset, float *out)
{
    if (batch < 0 || n_tokens < 0 || (!out && batch > 0 && n_tokens > 0)) return ORC_E_ARG;
    for (int32_t b = 0; b < batch; ++b)
        for (int32_t t = 0; t < n_tokens; ++t) out[(int64_t)b * n_tokens + t] = orc_gumbel(seed, offset, b, t);
    return ORC_OK;
}

static int orc_float_desc(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return x > y ? -1 : (x < y ? 1 : 0);
}

/* One decoding step as orc_mask_step, with the token drawn instead of taken greedily.
 * temperature must be positive with a finite reciprocal.  top_k > 0 restricts the draw to the
 * allowed tokens whose logit is at least the k-th largest allowed logit (counted with
 * multiplicity, NaN as -inf; tokens tied with the k-th are all kept, so more than k may remain;
 * fewer than k allowed tokens: all remain); top_k = 0 draws from all allowed tokens.  The masked
 * row shows the constraint only, not the cut.  A sequence whose state has no row, or whose
 * allowed set is empty, is handled as in orc_mask_step. */
int orc_sample_step(const int32_t *table, int64_t n_rows, int32_t n_tokens,
                    const void *logits, int dtype, int32_t batch, int64_t row_stride,
                    const int32_t *states, float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                    int32_t *tokens, int32_t *new_states, void *masked_out, int32_t n_threads)
{
    if (!table || !logits || !states || !tokens || !new_states || batch < 0 || n_tokens < 0) return ORC_E_ARG;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return ORC_E_ARG;
    if (!(temperature > 0.0f) || top_k < 0) return ORC_E_ARG;
    const float inv_t = 1.0f / temperature;
    if (!isfinite(inv_t) || !(inv_t > 0.0f)) return ORC_E_ARG;
    if (n_threads < 1) n_threads = 1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(n_threads)
#endif
    for (int32_t b = 0; b < batch; ++b) {
        int32_t q = states[b];
        int valid = (q >= 0 && (int64_t)q < n_rows);
        const int32_t *row = valid ? table + (int64_t)q * n_tokens : NULL;
        /* the cut: the k-th largest allowed logit */
        float cut = -INFINITY;
        if (valid && top_k > 0) {
            float *vals = (float *)malloc(sizeof(float) * (size_t)(n_tokens > 0 ? n_tokens : 1));
            if (!vals) { failed = 1; continue; }
            int32_t n = 0;
            for (int32_t t = 0; t < n_tokens; ++t)
                if (row[t] != ORC_DEAD) vals[n++] = (float)orc_logit(logits, dtype, (int64_t)b * row_stride + t);
            qsort(vals, (size_t)n, sizeof(float), orc_float_desc);
            if (n > 0) cut = vals[(top_k < n ? top_k : n) - 1];
            free(vals);
        }
        int32_t best = -1;
        float best_v = 0.0f;
        for (int32_t t = 0; t < n_tokens; ++t) {
            int64_t i = (int64_t)b * row_stride + t;
            int allowed = valid && row[t] != ORC_DEAD;
            if (masked_out) {
                if (dtype == ORC_F32) ((uint32_t *)masked_out)[i] = allowed ? ((const uint32_t *)logits)[i] : 0xFF800000u;
                else ((uint16_t *)masked_out)[i] = allowed ? ((const uint16_t *)logits)[i] : (uint16_t)0xFF80u;
            }
            if (!allowed) continue;
            float l = (float)orc_logit(logits, dtype, i);            /* fp32 or bf16: exact in float */
            if (l < cut) continue;
            float v = fmaf(l, inv_t, orc_gumbel(seed, offset, b, t));
            if (best < 0 || v > best_v) { best = t; best_v = v; }
        }
        tokens[b] = best;
        new_states[b] = !valid ? ORC_DEAD : (best < 0 ? q : row[best]);
    }
    return failed ? ORC_E_MEM : ORC_OK;
}

/* A run of k speculated tokens per sequence under the constraint, with the full history of
 * states (Section 5.3: the constraint must be rewindable, which the paper gets by keeping every
 * state passed through, not only the last).  history[b][0] is the sequence's state (DEAD if it is outside the
 * table); history[b][i + 1] = table[history[b][i]][tokens[b][i]], DEAD once a token has no edge
 * (or is not a token id), and DEAD from there on.  n_valid[b] = number of leading tokens the
 * constraint accepts, i.e. the longest prefix the caller may keep. */
int orc_advance_tokens(const int32_t *table, int64_t n_rows, int32_t n_tokens, int32_t batch, int32_t k,
                       const int32_t *states, const int32_t *tokens, int32_t *history, int32_t *n_valid)
{
    if (!table || !states || !history || batch < 0 || k < 0 || (k > 0 && !tokens)) return ORC_E_ARG;
    for (int32_t b = 0; b < batch; ++b) {
        int32_t *h = history + (int64_t)b * (k + 1);
        int32_t s = states[b];
        if (s < 0 || s >= n_rows) s = ORC_DEAD;
        h[0] = s;
        int32_t ok = 0;
        for (int32_t i = 0; i < k; ++i) {
            const int32_t t = tokens[(int64_t)b * k + i];
            if (s != ORC_DEAD && t >= 0 && t < n_tokens) s = table[(int64_t)s * n_tokens + t];
            else s = ORC_DEAD;
            h[i + 1] = s;
            if (s != ORC_DEAD && ok == i) ok = i + 1;
        }
        if (n_valid) n_valid[b] = ok;
    }
    return ORC_OK;
}

/* Terminal labels (Section 2.5.1, wildcard matching): a terminal edge (state, label, target)
 * stands for one edge per token of the label's pre-computed mask: all tokens of the mask are
 * allowed at once when the logits are penalised, and a chosen token that lies in the mask takes
 * the terminal edge; where both a normal token edge and a terminal
 * edge match, the normal edge is preferred, and among terminal edges the one that comes first in
 * the given (precedence) order.  On a dense table this is: for the edges in order, every token of
 * the mask whose entry in the state's row is still DEAD gets the edge's target.
 * masks is [n_labels][n_tokens], one byte per token (non-zero = in the mask). */
int orc_apply_terminals(int32_t *table, int64_t n_rows, int32_t n_tokens, int32_t n_edges,
                        const int32_t *edge_state, const int32_t *edge_label, const int32_t *edge_target,
                        int32_t n_labels, const uint8_t *masks)
{
    if (!table || n_edges < 0 || (n_edges > 0 && (!edge_state || !edge_label || !edge_target || !masks))) return ORC_E_ARG;
    for (int32_t e = 0; e < n_edges; ++e) {
        const int32_t q = edge_state[e], l = edge_label[e], to = edge_target[e];
        if (q < 0 || q >= n_rows || to < 0 || to >= n_rows || l < 0 || l >= n_labels) return ORC_E_ARG;
    }
    for (int32_t e = 0; e < n_edges; ++e) {
        int32_t *row = table + (int64_t)edge_state[e] * n_tokens;
        const uint8_t *mask = masks + (int64_t)edge_label[e] * n_tokens;
        for (int32_t t = 0; t < n_tokens; ++t)
            if (mask[t] && row[t] == ORC_DEAD) row[t] = edge_target[e];
    }
    return ORC_OK;
}

/* Token-level optimisation of a compiled table (Appendix C.2, fourth compile operation,
 * the optimisation of the composed automaton; the paper does not say which optimisation, the reading taken is
 * the classical one): drop the states that no token sequence reaches from the given start states
 * and those from which no final state can be reached (edges into them become DEAD: they accept
 * nothing, like DEAD), and merge the states that accept the same set of token sequences (Moore's partition
 * refinement: start from {final, not final}, split classes whose members disagree on the class
 * of some token's target, DEAD counting as a class of its own, until nothing splits).  The
 * result is the unique minimal deterministic token automaton of the same language per start
 * state; its states are numbered by the smallest old state of each class, which makes the table
 * unique too.
 *   map[q]   : new state of old state q, DEAD if q is not reachable
 *   out      : [*n_new * n_tokens], caller provides room for n_rows * n_tokens
 *   out_acc  : [*n_new] (may be NULL) */
typedef struct { const int32_t *sig; int64_t width; } orc_sig_ctx;
static orc_sig_ctx g_sig_ctx;
static int orc_sig_cmp(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    const int c = memcmp(g_sig_ctx.sig + (int64_t)x * g_sig_ctx.width, g_sig_ctx.sig + (int64_t)y * g_sig_ctx.width,
                         (size_t)g_sig_ctx.width * sizeof(int32_t));
    return c ? c : (x > y) - (x < y);
}

int orc_minimize(const int32_t *table, int64_t n_rows, int32_t n_tokens, const uint8_t *accept,
                 const int32_t *starts, int32_t n_starts, int32_t *map, int64_t *n_new, int32_t *out, uint8_t *out_acc)
{
    if (!table || !accept || !starts || !map || !n_new || !out || n_rows <= 0 || n_tokens < 0 || n_starts < 0) return ORC_E_ARG;
    const int64_t width = (int64_t)n_tokens + 1;
    int32_t *cls = malloc((size_t)n_rows * sizeof(int32_t));
    int32_t *next = malloc((size_t)n_rows * sizeof(int32_t));
    int32_t *stack = malloc((size_t)n_rows * sizeof(int32_t));
    int32_t *idx = malloc((size_t)n_rows * sizeof(int32_t));
    int32_t *sig = malloc((size_t)n_rows * (size_t)width * sizeof(int32_t));
    if (!cls || !next || !stack || !idx || !sig) { free(cls); free(next); free(stack); free(idx); free(sig); return ORC_E_MEM; }
    /* reachable states */
    for (int64_t q = 0; q < n_rows; ++q) cls[q] = ORC_DEAD;
    int64_t top = 0;
    for (int32_t i = 0; i < n_starts; ++i) {
        const int32_t q = starts[i];
        if (q < 0 || q >= n_rows) { free(cls); free(next); free(stack); free(idx); free(sig); return ORC_E_ARG; }
        if (cls[q] == ORC_DEAD) { cls[q] = accept[q] ? 1 : 0; stack[top++] = q; }
    }
    while (top > 0) {
        const int32_t q = stack[--top];
        for (int32_t t = 0; t < n_tokens; ++t) {
            const int32_t r = table[(int64_t)q * n_tokens + t];
            if (r != ORC_DEAD && cls[r] == ORC_DEAD) { cls[r] = accept[r] ? 1 : 0; stack[top++] = r; }
        }
    }
    /* of those, the states that can reach a final state (next[] as the flag); the others go */
    for (int64_t q = 0; q < n_rows; ++q) next[q] = cls[q] != ORC_DEAD && accept[q];
    for (int changed = 1; changed;) {
        changed = 0;
        for (int64_t q = 0; q < n_rows; ++q) {
            if (cls[q] == ORC_DEAD || next[q]) continue;
            for (int32_t t = 0; t < n_tokens; ++t) {
                const int32_t r = table[(int64_t)q * n_tokens + t];
                if (r != ORC_DEAD && next[r]) { next[q] = 1; changed = 1; break; }
            }
        }
    }
    for (int64_t q = 0; q < n_rows; ++q)
        if (!next[q]) cls[q] = ORC_DEAD;
    int64_t n_reach = 0;
    for (int64_t q = 0; q < n_rows; ++q)
        if (cls[q] != ORC_DEAD) idx[n_reach++] = (int32_t)q;
    /* refinement: signature = (own class, class of every token's target) */
    int64_t n_cls = 0, prev = -1;
    while (1) {
        for (int64_t i = 0; i < n_reach; ++i) {
            const int32_t q = idx[i];
            int32_t *s = sig + (int64_t)q * width;
            s[0] = cls[q];
            for (int32_t t = 0; t < n_tokens; ++t) {
                const int32_t r = table[(int64_t)q * n_tokens + t];
                s[t + 1] = r == ORC_DEAD ? ORC_DEAD : cls[r];      /* a dropped state has class DEAD */
            }
        }
        memcpy(stack, idx, (size_t)n_reach * sizeof(int32_t));
        g_sig_ctx.sig = sig; g_sig_ctx.width = width;
        qsort(stack, (size_t)n_reach, sizeof(int32_t), orc_sig_cmp);
        n_cls = 0;
        for (int64_t i = 0; i < n_reach; ++i) {
            if (i == 0 || memcmp(sig + (int64_t)stack[i] * width, sig + (int64_t)stack[i - 1] * width, (size_t)width * sizeof(int32_t)) != 0)
                ++n_cls;
            next[stack[i]] = (int32_t)(n_cls - 1);
        }
        for (int64_t i = 0; i < n_reach; ++i) cls[idx[i]] = next[idx[i]];
        if (n_cls == prev) break;
        prev = n_cls;
    }
    /* number the classes by their smallest member */
    for (int64_t c = 0; c < n_cls; ++c) next[c] = ORC_DEAD;      /* class -> new id */
    int64_t k = 0;
    for (int64_t i = 0; i < n_reach; ++i) {                       /* idx is ascending */
        const int32_t q = idx[i];
        if (next[cls[q]] == ORC_DEAD) {
            next[cls[q]] = (int32_t)k;
            stack[k] = q;                                         /* representative */
            ++k;
        }
    }
    for (int64_t q = 0; q < n_rows; ++q) map[q] = cls[q] == ORC_DEAD ? ORC_DEAD : next[cls[q]];
    for (int64_t c = 0; c < k; ++c) {
        const int32_t rep = stack[c];
        for (int32_t t = 0; t < n_tokens; ++t) {
            const int32_t r = table[(int64_t)rep * n_tokens + t];
            out[c * n_tokens + t] = r == ORC_DEAD ? ORC_DEAD : map[r];
        }
        if (out_acc) out_acc[c] = accept[rep] ? 1 : 0;
    }
    *n_new = k;
    free(cls); free(next); free(stack); free(idx); free(sig);
    return ORC_OK;
}

/* Stack per-constraint tables into one table whose states are global row ids: table c's
 * rows start at row_offsets[c]; every non-DEAD entry gets row_offsets[c] added. */
int orc_concat_tables(const int32_t *const *tables, const int32_t *n_rows, int32_t n, int32_t n_tokens,
                      int32_t *out, int64_t *row_offsets /* [n+1] */)
{
    if (!tables || !n_rows || !out || !row_offsets || n < 0) return ORC_E_ARG;
    int64_t base = 0;
    for (int32_t c = 0; c < n; ++c) {
        row_offsets[c] = base;
        for (int64_t i = 0; i < (int64_t)n_rows[c] * n_tokens; ++i) {
            int32_t v = tables[c][i];
            out[base * n_tokens + i] = v == ORC_DEAD ? ORC_DEAD : (int32_t)(v + base);
        }
        base += n_rows[c];
    }
    row_offsets[n] = base;
    return ORC_OK;
}

/* Edge-list form of a token-level table (the paper keeps A_{R o V} as a list of edges; Section
 * 2.5.1 remarks on the cost of states with many of them).  The edges of a state are kept in token
 * order, so the token of an edge need not be stored: it is the position of the edge among the
 * state's allowed tokens.
 *   row_begin[q]  : number of edges of the states before q        (n_rows + 1 entries)
 *   targets[i]    : target of edge i; the edges of state q are row_begin[q] .. row_begin[q+1] - 1
 * First call with targets == NULL to size it (row_begin is written). */
int orc_compact(const int32_t *table, int64_t n_rows, int32_t n_tokens, int64_t *row_begin, int32_t *targets)
{
    if (!table || !row_begin || n_rows < 0 || n_tokens < 0) return ORC_E_ARG;
    int64_t n = 0;
    for (int64_t q = 0; q < n_rows; ++q) {
        row_begin[q] = n;
        for (int32_t t = 0; t < n_tokens; ++t) {
            int32_t v = table[q * n_tokens + t];
            if (v == ORC_DEAD) continue;
            if (targets) targets[n] = v;
            ++n;
        }
    }
    row_begin[n_rows] = n;
    return ORC_OK;
}

/* The table an edge list stands for: allowed[q][t] (one byte each) says which tokens have an
 * edge; the k-th allowed token of state q takes targets[row_begin[q] + k]. */
int orc_expand(const uint8_t *allowed, int64_t n_rows, int32_t n_tokens, const int64_t *row_begin,
               const int32_t *targets, int32_t *table)
{
    if (!allowed || !row_begin || !targets || !table || n_rows < 0 || n_tokens < 0) return ORC_E_ARG;
    for (int64_t q = 0; q < n_rows; ++q) {
        int64_t k = row_begin[q];
        for (int32_t t = 0; t < n_tokens; ++t) {
            if (allowed[q * n_tokens + t]) {
                if (k >= row_begin[q + 1]) return ORC_E_ARG;
                table[q * n_tokens + t] = targets[k++];
            } else {
                table[q * n_tokens + t] = ORC_DEAD;
            }
        }
        if (k != row_begin[q + 1]) return ORC_E_ARG;
    }
    return ORC_OK;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
