/*
 * CPU oracle for push-down constraints (Section 3 of arXiv 2407.08103).
 *
 * TEST INFRASTRUCTURE ONLY, like tdfa_oracle.c, with which it is linked into one library: the
 * tests, the smoke check and the benchmark's CPU-baseline leg compare the GPU library against
 * it; it shares no code with the GPU library and the library never calls it.
 *
 * What it follows:
 *   - Section 3.1: a push-down automaton P = (Sigma, Pi, S, Q, I, F, E); an edge is
 *     (source, input, pops, target, pushes) with the input a byte or epsilon and pops / pushes
 *     strings of stack symbols; an edge can be taken when the stack ends with its pops, which
 *     are then removed and its pushes appended.  Non-deterministic automata are an error.
 *   - Section 3.2 / Algorithm 3, third statement: P_{G o V} = P_G o T_V.  The composition is
 *     done explicitly over pair states (state of P_G, state of T_V), with T_V the chain
 *     transducer of Algorithm 1 (built by tdfa_oracle.c); edges whose input is epsilon are then
 *     removed by following every path from (q, root) to the token-labelled edge that closes the
 *     token's cycle, concatenating the stack edits on the way.
 *   - Algorithm 3, decoding loop: the allowed set {input(e) : source(e) = q, s ends with
 *     pops(e)}, the -inf penalty, the token choice, the matching edge and its traversal
 *     (q <- target, pops removed, pushes appended).
 *
 * Readings of points the paper leaves open:
 *   - stack strings are written bottom to top (the last symbol is the top), as in "s ends with
 *     pops";
 *   - epsilon edges of P_G belong to the token edge of the byte that FOLLOWS them: a token edge
 *     ends with its last byte (it is the closing edge of T_V's cycle that carries the token
 *     label, so nothing follows it inside the cycle).  Whether a configuration is accepting
 *     is therefore asked after a last closure over epsilon edges (orc_pda_accepting);
 *   - concatenating stack edits: an edit (pops p, pushes u) followed by (p', u') is
 *     (p, u[..|u|-|p'|] u') if u ends with p', and (r p, u') if p' = r u; anything else cannot
 *     be taken.  A token edge therefore may pop and push several symbols (caption of Fig. 7);
 *   - determinism: two edges of one state whose inputs can meet (equal, or one of them
 *     epsilon) must have pops of which neither is a suffix of the other; the same holds for
 *     the token edges of one (state, token).  Violations are reported, not resolved;
 *   - token choice, ties, NaN, -0, states that are no state: as in tdfa_oracle.c; a sequence
 *     whose stack would outgrow its buffer gets token -1 and state DEAD;
 *   - Algorithm 3 takes its token from the language model's sampler like Algorithm 2 does:
 *     orc_pda_sample_step draws it from softmax(l / T) over the allowed set by the rule of
 *     orc_sample_step (the allowed token with the largest fma(l, 1/T, g), g the Gumbel variate of
 *     (seed, offset, sequence, token); top_k as there), then traverses the matching edge.
 *
 * Pinned by tests/test_oracle_pda.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_DEAD (-1)
#define ORC_EPS  (-1)
#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_MEM (-2)
#define ORC_E_NONDET (-3)
#define ORC_E_STRUCT (-4)
#define ORC_E_LIMIT (-5)         /* a stack string, an epsilon run or an output buffer outgrew its limit */

#define ORC_PDA_STR 12           /* longest pops / pushes string of a token edge */
#define ORC_PDA_EPS_RUN 64       /* longest run of epsilon edges inside one token edge */

typedef struct { int32_t src, in, out, dst; } orc_fst_edge;
typedef struct { int32_t n_states, root; int64_t n_edges; orc_fst_edge *edges; } orc_fst;
int orc_build_detok_fst(const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens, orc_fst *out);
void orc_fst_free(orc_fst *t);
float orc_gumbel(uint64_t seed, uint64_t offset, int32_t b, int32_t t);      /* tdfa_oracle.c: the noise of a draw */

/* P_G as arrays: edge e = (src[e], input[e], pop_syms[pop_begin[e] .. pop_begin[e+1]), dst[e],
 * push_syms[push_begin[e] .. push_begin[e+1])), input -1 = epsilon. */
typedef struct {
    int32_t n_states, n_edges;
    const int32_t *src, *input, *dst, *pop_begin, *pop_syms, *push_begin, *push_syms;
} orc_pda;

static int is_suffix(const int32_t *a, int na, const int32_t *b, int nb)   /* a is a suffix of b */
{
    if (na > nb) return 0;
    return memcmp(a, b + (nb - na), sizeof(int32_t) * (size_t)na) == 0;
}

static int pda_args_ok(const orc_pda *p)
{
    if (p->n_states <= 0 || p->n_edges < 0) return 0;
    for (int32_t e = 0; e < p->n_edges; ++e) {
        if (p->src[e] < 0 || p->src[e] >= p->n_states || p->dst[e] < 0 || p->dst[e] >= p->n_states) return 0;
        if (p->input[e] < -1 || p->input[e] > 255) return 0;
        if (p->pop_begin[e + 1] < p->pop_begin[e] || p->push_begin[e + 1] < p->push_begin[e]) return 0;
    }
    return 1;
}

/* Section 3.1, last paragraph: 0 if no two edges of a state can both be taken in some
 * configuration; else 1 + the index of the first edge that has such a rival. */
int orc_pda_check_deterministic(int32_t n_states, int32_t n_edges, const int32_t *src, const int32_t *input,
                                const int32_t *dst, const int32_t *pop_begin, const int32_t *pop_syms,
                                const int32_t *push_begin, const int32_t *push_syms)
{
    orc_pda p = {n_states, n_edges, src, input, dst, pop_begin, pop_syms, push_begin, push_syms};
    if (!pda_args_ok(&p)) return ORC_E_ARG;
    for (int32_t e = 0; e < n_edges; ++e)
        for (int32_t f = e + 1; f < n_edges; ++f) {
            if (src[e] != src[f]) continue;
            if (input[e] != input[f] && input[e] != ORC_EPS && input[f] != ORC_EPS) continue;
            const int32_t *pe = pop_syms + pop_begin[e], *pf = pop_syms + pop_begin[f];
            const int ne = pop_begin[e + 1] - pop_begin[e], nf = pop_begin[f + 1] - pop_begin[f];
            if (is_suffix(pe, ne, pf, nf) || is_suffix(pf, nf, pe, ne)) return 1 + e;
        }
    return 0;
}

/* The stack edit of a path so far: the original stack must end with req[0 .. n_req) (which is
 * removed), then top[0 .. n_top) is appended. */
typedef struct { int32_t req[ORC_PDA_STR], top[ORC_PDA_STR]; int n_req, n_top; } orc_edit;

/* edit followed by edge e of p: 1 = can be taken (out written), 0 = cannot, <0 = error */
static int edit_then_edge(const orc_edit *ed, const orc_pda *p, int32_t e, orc_edit *out)
{
    const int32_t *pops = p->pop_syms + p->pop_begin[e];
    const int n_pops = p->pop_begin[e + 1] - p->pop_begin[e];
    const int32_t *pushes = p->push_syms + p->push_begin[e];
    const int n_push = p->push_begin[e + 1] - p->push_begin[e];
    *out = *ed;
    if (n_pops <= ed->n_top) {
        if (!is_suffix(pops, n_pops, ed->top, ed->n_top)) return 0;
        out->n_top = ed->n_top - n_pops;
    } else {
        /* pops = r top: the known top must be the end of pops, r comes from below it */
        if (!is_suffix(ed->top, ed->n_top, pops, n_pops)) return 0;
        const int n_r = n_pops - ed->n_top;
        if (n_r + ed->n_req > ORC_PDA_STR) return ORC_E_LIMIT;
        memmove(out->req + n_r, ed->req, sizeof(int32_t) * (size_t)ed->n_req);
        memcpy(out->req, pops, sizeof(int32_t) * (size_t)n_r);
        out->n_req = ed->n_req + n_r;
        out->n_top = 0;
    }
    if (out->n_top + n_push > ORC_PDA_STR) return ORC_E_LIMIT;
    memcpy(out->top + out->n_top, pushes, sizeof(int32_t) * (size_t)n_push);
    out->n_top += n_push;
    return 1;
}

/* Token edges of P_{G o V} as they are found. */
typedef struct {
    int64_t cap, n;
    int32_t *src, *token, *dst, *n_pops, *pops, *n_push, *pushes;   /* pops / pushes: ORC_PDA_STR per edge */
} orc_tedges;

typedef struct {
    const orc_pda *p;
    const int32_t *pda_first;      /* edges of P_G by source state (edges sorted by the caller) */
    const orc_fst *t;
    const int64_t *fst_first;      /* edges of T_V by source state */
    const int64_t *fst_order;
    orc_tedges *out;
    int32_t q;                     /* the source state of the token edges being collected */
} orc_pctx;

/* Depth-first over the composed automaton from pair state (a, u): epsilon-input edges are
 * followed, a token-labelled edge ends the path and is recorded. */
static int explore(const orc_pctx *c, int32_t a, int32_t u, const orc_edit *ed, int n_eps)
{
    const orc_pda *p = c->p;
    /* (i) an epsilon edge of P_G, T_V stays where it is */
    for (int32_t e = c->pda_first[a]; e < c->pda_first[a + 1]; ++e) {
        if (p->input[e] != ORC_EPS) continue;
        orc_edit nx;
        const int ok = edit_then_edge(ed, p, e, &nx);
        if (ok < 0) return ok;
        if (!ok) continue;
        if (n_eps + 1 > ORC_PDA_EPS_RUN) return ORC_E_LIMIT;
        const int rc = explore(c, p->dst[e], u, &nx, n_eps + 1);
        if (rc != ORC_OK) return rc;
    }
    /* (ii) an edge of T_V that emits byte x, matched with an edge of P_G that reads x */
    for (int64_t k = c->fst_first[u]; k < c->fst_first[u + 1]; ++k) {
        const orc_fst_edge *fe = &c->t->edges[c->fst_order[k]];
        for (int32_t e = c->pda_first[a]; e < c->pda_first[a + 1]; ++e) {
            if (p->input[e] != fe->out) continue;
            orc_edit nx;
            const int ok = edit_then_edge(ed, p, e, &nx);
            if (ok < 0) return ok;
            if (!ok) continue;
            if (fe->in == ORC_EPS) {
                const int rc = explore(c, p->dst[e], fe->dst, &nx, 0);
                if (rc != ORC_OK) return rc;
                continue;
            }
            /* the closing edge of the token's cycle: back at the root of T_V */
            if (fe->dst != c->t->root) return ORC_E_STRUCT;
            orc_tedges *o = c->out;
            /* a second edge for this (state, token) must not be able to fire together with this one */
            for (int64_t j = o->n - 1; j >= 0 && o->src[j] == c->q; --j) {
                if (o->token[j] != fe->in) continue;
                const int32_t *pj = o->pops + j * ORC_PDA_STR;
                if (is_suffix(pj, o->n_pops[j], nx.req, nx.n_req) || is_suffix(nx.req, nx.n_req, pj, o->n_pops[j]))
                    return ORC_E_NONDET;
            }
            if (o->n >= o->cap) return ORC_E_LIMIT;
            const int64_t i = o->n++;
            o->src[i] = c->q;
            o->token[i] = fe->in;
            o->dst[i] = p->dst[e];
            o->n_pops[i] = nx.n_req;
            o->n_push[i] = nx.n_top;
            memset(o->pops + i * ORC_PDA_STR, 0xFF, sizeof(int32_t) * ORC_PDA_STR);
            memset(o->pushes + i * ORC_PDA_STR, 0xFF, sizeof(int32_t) * ORC_PDA_STR);
            memcpy(o->pops + i * ORC_PDA_STR, nx.req, sizeof(int32_t) * (size_t)nx.n_req);
            memcpy(o->pushes + i * ORC_PDA_STR, nx.top, sizeof(int32_t) * (size_t)nx.n_top);
        }
    }
    return ORC_OK;
}

/* Algorithm 3, third statement: the token edges of P_G o T_V that leave the states q_lo .. q_hi - 1,
 * in the order (state, order of discovery).  The edges of P_G must be sorted by source state.
 * pops / pushes hold ORC_PDA_STR symbols per edge, unused places -1.  *n_out receives the number
 * of edges; ORC_E_LIMIT if they do not fit in cap. */
int orc_pda_compile(int32_t n_states, int32_t n_edges, const int32_t *src, const int32_t *input, const int32_t *dst,
                    const int32_t *pop_begin, const int32_t *pop_syms, const int32_t *push_begin, const int32_t *push_syms,
                    const uint8_t *bytes, const uint64_t *offsets, int32_t n_tokens, int32_t q_lo, int32_t q_hi,
                    int64_t cap, int32_t *e_src, int32_t *e_token, int32_t *e_dst, int32_t *e_n_pops, int32_t *e_pops,
                    int32_t *e_n_push, int32_t *e_pushes, int64_t *n_out)
{
    orc_pda p = {n_states, n_edges, src, input, dst, pop_begin, pop_syms, push_begin, push_syms};
    if (!n_out || !pda_args_ok(&p) || q_lo < 0 || q_hi > n_states || q_lo > q_hi) return ORC_E_ARG;
    for (int32_t e = 1; e < n_edges; ++e)
        if (src[e] < src[e - 1]) return ORC_E_ARG;
    const int det = orc_pda_check_deterministic(n_states, n_edges, src, input, dst, pop_begin, pop_syms, push_begin, push_syms);
    if (det != 0) return det < 0 ? det : ORC_E_NONDET;
    int32_t *pda_first = (int32_t *)calloc((size_t)n_states + 1, sizeof(int32_t));
    if (!pda_first) return ORC_E_MEM;
    for (int32_t e = 0; e < n_edges; ++e) ++pda_first[src[e] + 1];
    for (int32_t s = 0; s < n_states; ++s) pda_first[s + 1] += pda_first[s];

    orc_fst t;
    int rc = orc_build_detok_fst(bytes, offsets, n_tokens, &t);
    if (rc != ORC_OK) { free(pda_first); return rc; }
    int64_t *fst_first = (int64_t *)calloc((size_t)t.n_states + 1, sizeof(int64_t));
    int64_t *fst_order = (int64_t *)malloc(sizeof(int64_t) * (size_t)(t.n_edges > 0 ? t.n_edges : 1));
    int64_t *fill = (int64_t *)calloc((size_t)t.n_states + 1, sizeof(int64_t));
    if (!fst_first || !fst_order || !fill) { rc = ORC_E_MEM; goto done; }
    for (int64_t k = 0; k < t.n_edges; ++k) ++fst_first[t.edges[k].src + 1];
    for (int32_t s = 0; s < t.n_states; ++s) fst_first[s + 1] += fst_first[s];
    for (int64_t k = 0; k < t.n_edges; ++k) fst_order[fst_first[t.edges[k].src] + fill[t.edges[k].src]++] = k;
    {
        orc_tedges out = {cap, 0, e_src, e_token, e_dst, e_n_pops, e_pops, e_n_push, e_pushes};
        orc_pctx c = {&p, pda_first, &t, fst_first, fst_order, &out, 0};
        for (int32_t q = q_lo; q < q_hi && rc == ORC_OK; ++q) {
            orc_edit ed;
            memset(&ed, 0, sizeof(ed));
            c.q = q;
            rc = explore(&c, q, t.root, &ed, 0);
        }
        *n_out = out.n;
    }
done:
    free(fill);
    free(fst_order);
    free(fst_first);
    free(pda_first);
    orc_fst_free(&t);
    return rc;
}

/* Whether configuration (q, stack) accepts with nothing more to read: q is final, or a run of
 * epsilon edges of P_G leads to a final state (deterministic automaton: at most one can be taken
 * at a time).  stack is bottom to top.  Returns 1 / 0, or a negative code. */
int orc_pda_accepting(int32_t n_states, int32_t n_edges, const int32_t *src, const int32_t *input, const int32_t *dst,
                      const int32_t *pop_begin, const int32_t *pop_syms, const int32_t *push_begin, const int32_t *push_syms,
                      const uint8_t *accept, int32_t q, const int32_t *stack, int32_t depth)
{
    orc_pda p = {n_states, n_edges, src, input, dst, pop_begin, pop_syms, push_begin, push_syms};
    if (!pda_args_ok(&p) || !accept || q < 0 || q >= n_states || depth < 0) return ORC_E_ARG;
    int32_t cap = depth + 4 * ORC_PDA_EPS_RUN * ORC_PDA_STR + 8;
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    if (!s) return ORC_E_MEM;
    memcpy(s, stack, sizeof(int32_t) * (size_t)depth);
    int32_t n = depth, result = 0;
    for (int step = 0; step <= ORC_PDA_EPS_RUN; ++step) {
        if (accept[q]) { result = 1; break; }
        int32_t take = -1;
        for (int32_t e = 0; e < n_edges; ++e) {
            if (src[e] != q || input[e] != ORC_EPS) continue;
            if (is_suffix(pop_syms + pop_begin[e], pop_begin[e + 1] - pop_begin[e], s, n)) { take = e; break; }
        }
        if (take < 0) break;
        n -= pop_begin[take + 1] - pop_begin[take];
        const int np = push_begin[take + 1] - push_begin[take];
        if (n + np > cap) { result = ORC_E_LIMIT; break; }
        memcpy(s + n, push_syms + push_begin[take], sizeof(int32_t) * (size_t)np);
        n += np;
        q = dst[take];
    }
    free(s);
    return result;
}

static double pda_logit(const void *logits, int dtype, int64_t i)
{
    if (dtype == 0) return (double)((const float *)logits)[i];
    const uint32_t w = (uint32_t)((const uint16_t *)logits)[i] << 16;
    float f;
    memcpy(&f, &w, sizeof(f));
    return (double)f;
}

/* Algorithm 3, loop body, for `batch` sequences.  Token edges sorted by source state:
 * edge_first[q] .. edge_first[q + 1] are those of state q.  stacks: [batch][stack_cap], bottom to
 * top, depths[b] symbols in use; both are updated in place, states -> new_states.
 * dtype 0 = float32, 1 = bfloat16 bit patterns; masked (may be NULL) receives the penalised logits. */
int orc_pda_step(int32_t n_states, int32_t n_tokens, const int64_t *edge_first, const int32_t *e_token, const int32_t *e_dst,
                 const int32_t *e_n_pops, const int32_t *e_pops, const int32_t *e_n_push, const int32_t *e_pushes,
                 const void *logits, int dtype, int32_t batch, int64_t row_stride, const int32_t *states,
                 int32_t *stacks, int32_t *depths, int32_t stack_cap, int32_t *tokens, int32_t *new_states, void *masked)
{
    if (n_states <= 0 || n_tokens < 0 || batch < 0 || row_stride < n_tokens || stack_cap < 0 || (dtype != 0 && dtype != 1))
        return ORC_E_ARG;
    uint8_t *allowed = (uint8_t *)malloc((size_t)(n_tokens > 0 ? n_tokens : 1));
    int64_t *edge_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_tokens > 0 ? n_tokens : 1));
    if (!allowed || !edge_of) { free(allowed); free(edge_of); return ORC_E_MEM; }
    int rc = ORC_OK;
    for (int32_t b = 0; b < batch && rc == ORC_OK; ++b) {
        const int32_t q = states[b];
        int32_t *s = stacks + (int64_t)b * stack_cap;
        const int32_t n = depths[b];
        const int valid = q >= 0 && q < n_states && n >= 0 && n <= stack_cap;
        memset(allowed, 0, (size_t)n_tokens);
        /* A = { input(e) : source(e) = q and s ends with pops(e) } */
        if (valid)
            for (int64_t e = edge_first[q]; e < edge_first[q + 1]; ++e)
                if (is_suffix(e_pops + e * ORC_PDA_STR, e_n_pops[e], s, n)) {
                    if (allowed[e_token[e]]) { rc = ORC_E_NONDET; break; }
                    allowed[e_token[e]] = 1;
                    edge_of[e_token[e]] = e;
                }
        if (rc != ORC_OK) break;
        int32_t best = -1;
        double best_v = 0.0;
        for (int32_t t = 0; t < n_tokens; ++t) {
            const int64_t i = (int64_t)b * row_stride + t;
            if (!allowed[t]) {
                if (masked) {
                    if (dtype == 0) ((uint32_t *)masked)[i] = 0xFF800000u;
                    else ((uint16_t *)masked)[i] = 0xFF80u;
                }
                continue;
            }
            double v = pda_logit(logits, dtype, i);
            if (isnan(v)) v = -INFINITY;
            if (best < 0 || v > best_v) { best = t; best_v = v; }
        }
        tokens[b] = best;
        if (best < 0) {
            new_states[b] = valid ? q : ORC_DEAD;
            continue;
        }
        /* the matching edge: q <- target, pops off, pushes on */
        const int64_t e = edge_of[best];
        const int32_t m = n - e_n_pops[e];
        if (m + e_n_push[e] > stack_cap) {           /* the stack would outgrow its buffer */
            tokens[b] = -1;
            new_states[b] = ORC_DEAD;
            continue;
        }
        memcpy(s + m, e_pushes + e * ORC_PDA_STR, sizeof(int32_t) * (size_t)e_n_push[e]);
        depths[b] = m + e_n_push[e];
        new_states[b] = e_dst[e];
    }
    free(allowed);
    free(edge_of);
    return rc;
}

static int float_desc(const void *a, const void *b)
{
    const float x = *(const float *)a, y = *(const float *)b;
    return x > y ? -1 : (x < y ? 1 : 0);
}

/* Algorithm 3, loop body, with the token drawn instead of taken greedily: the allowed set as in
 * orc_pda_step, the draw as in orc_sample_step (temperature > 0 with a finite reciprocal; top_k > 0
 * keeps the allowed tokens whose logit is at least the k-th largest allowed logit, NaN as -inf,
 * ties with the k-th all kept; 0 keeps all), then the traversal of the drawn token's edge.  The
 * penalised row shows the constraint only, not the cut. */
int orc_pda_sample_step(int32_t n_states, int32_t n_tokens, const int64_t *edge_first, const int32_t *e_token, const int32_t *e_dst,
                        const int32_t *e_n_pops, const int32_t *e_pops, const int32_t *e_n_push, const int32_t *e_pushes,
                        const void *logits, int dtype, int32_t batch, int64_t row_stride, const int32_t *states,
                        int32_t *stacks, int32_t *depths, int32_t stack_cap, float temperature, int32_t top_k,
                        uint64_t seed, uint64_t offset, int32_t *tokens, int32_t *new_states, void *masked)
{
    if (n_states <= 0 || n_tokens < 0 || batch < 0 || row_stride < n_tokens || stack_cap < 0 || (dtype != 0 && dtype != 1))
        return ORC_E_ARG;
    if (!(temperature > 0.0f) || top_k < 0) return ORC_E_ARG;
    const float inv_t = 1.0f / temperature;
    if (!isfinite(inv_t) || !(inv_t > 0.0f)) return ORC_E_ARG;
    const size_t room = (size_t)(n_tokens > 0 ? n_tokens : 1);
    uint8_t *allowed = (uint8_t *)malloc(room);
    int64_t *edge_of = (int64_t *)malloc(sizeof(int64_t) * room);
    float *vals = (float *)malloc(sizeof(float) * room);
    if (!allowed || !edge_of || !vals) { free(allowed); free(edge_of); free(vals); return ORC_E_MEM; }
    int rc = ORC_OK;
    for (int32_t b = 0; b < batch && rc == ORC_OK; ++b) {
        const int32_t q = states[b];
        int32_t *s = stacks + (int64_t)b * stack_cap;
        const int32_t n = depths[b];
        const int valid = q >= 0 && q < n_states && n >= 0 && n <= stack_cap;
        memset(allowed, 0, (size_t)n_tokens);
        /* A = { input(e) : source(e) = q and s ends with pops(e) } */
        if (valid)
            for (int64_t e = edge_first[q]; e < edge_first[q + 1]; ++e)
                if (is_suffix(e_pops + e * ORC_PDA_STR, e_n_pops[e], s, n)) {
                    if (allowed[e_token[e]]) { rc = ORC_E_NONDET; break; }
                    allowed[e_token[e]] = 1;
                    edge_of[e_token[e]] = e;
                }
        if (rc != ORC_OK) break;
        /* the cut: the k-th largest allowed logit */
        float cut = -INFINITY;
        if (top_k > 0) {
            int32_t k = 0;
            for (int32_t t = 0; t < n_tokens; ++t)
                if (allowed[t]) {
                    float l = (float)pda_logit(logits, dtype, (int64_t)b * row_stride + t);
                    vals[k++] = isnan(l) ? -INFINITY : l;
                }
            qsort(vals, (size_t)k, sizeof(float), float_desc);
            if (k > 0) cut = vals[(top_k < k ? top_k : k) - 1];
        }
        int32_t best = -1;
        float best_v = 0.0f;
        for (int32_t t = 0; t < n_tokens; ++t) {
            const int64_t i = (int64_t)b * row_stride + t;
            if (!allowed[t]) {
                if (masked) {
                    if (dtype == 0) ((uint32_t *)masked)[i] = 0xFF800000u;
                    else ((uint16_t *)masked)[i] = 0xFF80u;
                }
                continue;
            }
            float l = (float)pda_logit(logits, dtype, i);           /* fp32 or bf16: exact in float */
            if (isnan(l)) l = -INFINITY;
            if (l < cut) continue;
            const float v = fmaf(l, inv_t, orc_gumbel(seed, offset, b, t));
            if (best < 0 || v > best_v) { best = t; best_v = v; }
        }
        tokens[b] = best;
        if (best < 0) {
            new_states[b] = valid ? q : ORC_DEAD;
            continue;
        }
        /* the matching edge: q <- target, pops off, pushes on */
        const int64_t e = edge_of[best];
        const int32_t m = n - e_n_pops[e];
        if (m + e_n_push[e] > stack_cap) {           /* the stack would outgrow its buffer */
            tokens[b] = -1;
            new_states[b] = ORC_DEAD;
            continue;
        }
        memcpy(s + m, e_pushes + e * ORC_PDA_STR, sizeof(int32_t) * (size_t)e_n_push[e]);
        depths[b] = m + e_n_push[e];
        new_states[b] = e_dst[e];
    }
    free(allowed);
    free(edge_of);
    free(vals);
    return rc;
}
