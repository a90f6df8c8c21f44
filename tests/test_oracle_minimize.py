"""Pins for the oracle's token-level optimisation (reachable states only, equivalent states merged):
the worked example of Figures 3/4 (states that cannot reach a final state count as DEAD), language preservation by brute force, minimality by a search
for distinguishing sequences, idempotence, and agreement with character-level minimality."""
import itertools

import numpy as np
import pytest

from workloads import vocab as V
from workloads.regex_dfa import compile_regex

DEAD = -1


def _accepts(table, accept, q, seq):
    for t in seq:
        if q == DEAD:
            return False
        q = int(table[q, t])
    return q != DEAD and bool(accept[q])


def _distinguishable(table, accept, a, b):
    """Is there a token sequence accepted from exactly one of a, b?  Search over pairs."""
    seen = {(a, b)}
    todo = [(a, b)]
    while todo:
        x, y = todo.pop()
        ax = x != DEAD and bool(accept[x])
        ay = y != DEAD and bool(accept[y])
        if ax != ay:
            return True
        for t in range(table.shape[1]):
            nx = DEAD if x == DEAD else int(table[x, t])
            ny = DEAD if y == DEAD else int(table[y, t])
            if nx == ny or (nx, ny) in seen:
                continue
            seen.add((nx, ny))
            todo.append((nx, ny))
    return False


def test_fig4_example(oracle):
    """(foo)+d over {f, oo, foo, for, food}: 'fo' (s2) is reached by no token sequence, and s0 and s3
    (before the first and after a complete 'foo') differ: only s3 may be followed by d... through
    'food' both reach the end, so their rows are equal and they merge."""
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    assert table.tolist() == [[1, -1, 3, -1, 4], [-1, 3, -1, -1, -1], [-1] * 5, [1, -1, 3, -1, 4], [-1] * 5]
    new, acc, mp = oracle.minimize(table, d.accept, [d.start])
    assert mp.tolist() == [0, 1, DEAD, 0, 2]
    assert new.tolist() == [[1, -1, 0, -1, 2], [-1, 0, -1, -1, -1], [-1] * 5]
    assert acc.tolist() == [0, 0, 1]


@pytest.mark.parametrize("seed", range(8))
def test_language_kept_and_minimal(oracle, seed):
    rng = np.random.default_rng(seed)
    n, v = int(rng.integers(2, 9)), int(rng.integers(1, 5))
    table = rng.integers(0, n, size=(n, v), dtype=np.int32)
    table[rng.random((n, v)) < 0.35] = DEAD
    # plant duplicates of a state so that there is something to merge
    table[n - 1] = table[0]
    accept = (rng.random(n) < 0.4).astype(np.uint8)
    accept[n - 1] = accept[0]
    starts = sorted(set(rng.integers(0, n, size=2).tolist()))
    new, acc, mp = oracle.minimize(table, accept, starts)
    for s in starts:
        for k in range(0, 6):
            for seq in itertools.product(range(v), repeat=k):
                assert _accepts(table, accept, s, seq) == _accepts(new, acc, int(mp[s]), seq)
    # every new state is reached and can reach a final state, and no two of them are equivalent
    reach = set(int(mp[s]) for s in starts if mp[s] != DEAD)
    todo = list(reach)
    while todo:
        q = todo.pop()
        for t in range(v):
            r = int(new[q, t])
            if r != DEAD and r not in reach:
                reach.add(r)
                todo.append(r)
    assert reach == set(range(len(new)))
    for a in range(len(new)):
        assert _distinguishable(new, acc, a, DEAD)            # it accepts something
        for b in range(a + 1, len(new)):
            assert _distinguishable(new, acc, a, b)
    # numbering: by the smallest old state of each class; the map is consistent with the table
    firsts = [int(np.nonzero(mp == c)[0][0]) for c in range(len(new))]
    assert firsts == sorted(firsts)
    for q in range(n):
        if mp[q] != DEAD:
            for t in range(v):
                r = table[q, t]
                assert new[mp[q], t] == (DEAD if r == DEAD else mp[r])
    # idempotent
    if len(new) == 0:
        return
    again, acc2, mp2 = oracle.minimize(new, acc, [int(mp[s]) for s in starts if mp[s] != DEAD])
    assert np.array_equal(again, new) and np.array_equal(acc2, acc) and mp2.tolist() == list(range(len(new)))


def test_singleton_vocabulary_keeps_a_minimal_automaton(oracle):
    """With every byte of the alphabet as a token, token-level equivalence is character-level
    equivalence: a minimal trim character automaton loses no state."""
    d = compile_regex(r"(ab|cd)*e?f{1,3}")
    toks = [bytes([b]) for b in b"abcdef"] + [b"ab", b"cdab", b"ff"]
    vocab = V.from_tokens(toks)
    table = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    new, acc, mp = oracle.minimize(table, d.accept, [d.start])
    assert len(new) == d.n_states and sorted(mp.tolist()) == list(range(d.n_states))
