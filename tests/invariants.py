"""Properties every token-level table must have, whoever computed it (numpy only).

Used on oracle tables (CPU tests) and on GPU tables at sizes where a full oracle table
would be slow.  Each follows from A_{R o V}(x) = A_R(D(x)) (Theorems 1 and 2, Appendix B).
"""
from __future__ import annotations

import numpy as np

DEAD = -1


def check_singletons(table, trans, vocab, rows=None):
    """A one-byte token t = b has delta_T[q][t] == delta[q][b]: restricted to singletons
    the table is the character automaton itself."""
    lens = np.diff(vocab.offsets.astype(np.int64))
    ids = np.nonzero(lens == 1)[0]
    bs = vocab.data[vocab.offsets[ids].astype(np.int64)]
    rows = np.arange(table.shape[0]) if rows is None else np.asarray(rows)
    assert np.array_equal(table[:, ids], trans[rows][:, bs])
    return len(ids)


def check_concatenation(table_full, vocab, rng, n_triples=2000):
    """If d(u) = d(t1) d(t2) then delta_T[q][u] == delta_T[delta_T[q][t1]][t2] (DEAD absorbing).
    table_full must hold all rows.  Returns the number of triples checked."""
    toks = vocab.tokens()
    index = {}
    for i, s in enumerate(toks):
        index.setdefault(s, i)
    cand = [i for i, s in enumerate(toks) if len(s) >= 2]
    rng.shuffle(cand)
    done = 0
    for u in cand:
        s = toks[u]
        k = int(rng.integers(1, len(s)))
        t1, t2 = index.get(s[:k]), index.get(s[k:])
        if t1 is None or t2 is None:
            continue
        mid = table_full[:, t1]
        via = np.where(mid >= 0, table_full[np.clip(mid, 0, None), t2], DEAD)
        assert np.array_equal(table_full[:, u], via), (u, t1, t2)
        done += 1
        if done >= n_triples:
            break
    return done


def token_reachable(table_full, start):
    """States reachable from `start` through tokens."""
    seen = np.zeros(table_full.shape[0], dtype=bool)
    seen[start] = True
    frontier = [start]
    while frontier:
        nxt = np.unique(table_full[frontier].ravel())
        nxt = nxt[nxt >= 0]
        new = nxt[~seen[nxt]]
        seen[new] = True
        frontier = new.tolist()
    return np.nonzero(seen)[0]


def check_liveness(table_full, accept, start):
    """Every state reachable through tokens is accepting or has at least one live token
    (holds for a trim DFA whose alphabet bytes are all one-byte tokens, Section 2.4)."""
    reach = token_reachable(table_full, start)
    live = (table_full[reach] >= 0).any(axis=1)
    bad = reach[~(live | accept[reach].astype(bool))]
    assert len(bad) == 0, bad[:10]
    return len(reach)


def check_range(table, n_states):
    assert table.dtype == np.int32
    assert table.min() >= DEAD and table.max() < n_states
