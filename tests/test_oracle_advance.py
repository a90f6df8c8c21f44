"""Pins for the oracle's speculated-run function (Section 5.3: a rewindable constraint keeps the
full history of states): the worked example of Figures 3/4, agreement with Python's `re` on the
detokenized text, and the relation to single decode steps."""
import re

import numpy as np

from workloads import vocab as V
from workloads.regex_dfa import compile_regex

DEAD = -1


def test_fig4_runs(oracle):
    """(foo)+d over {f, oo, foo, for, food}: table derived by hand in tests/golden."""
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    F, OO, FOO, FOR, FOOD = range(5)
    runs = np.array([[F, OO, FOOD],        # f.oo.food : foofood, accepted by (foo)+d
                     [FOO, FOO, F],        # foo.foo.f : still a viable prefix
                     [FOO, FOR, FOO],      # 'for' has no edge anywhere: rejected at position 1
                     [OO, F, FOO],         # 'oo' first: rejected at position 0
                     [FOOD, F, F]],        # complete after one token, nothing may follow
                    dtype=np.int32)
    hist, n_valid = oracle.advance_tokens(table, np.full(5, d.start, np.int32), runs)
    assert n_valid.tolist() == [3, 3, 1, 0, 1]
    assert hist[0].tolist() == [0, 1, 3, 4] and d.accept[hist[0, 3]]
    assert hist[1].tolist() == [0, 3, 3, 1]
    assert hist[2].tolist() == [0, 3, DEAD, DEAD]          # DEAD is absorbing
    assert hist[3].tolist() == [0, DEAD, DEAD, DEAD]
    assert hist[4].tolist() == [0, 4, DEAD, DEAD]


def test_runs_against_re(oracle):
    """A prefix of a run is kept iff the text it spells can still be completed to a member of
    the language; the history state is accepting iff the text is a member."""
    pattern = r"(ab|cd)*e?"
    d = compile_regex(pattern)
    toks = [b"a", b"b", b"ab", b"cd", b"e", b"abc", b"d", b"c", b"abab", b"de"]
    vocab = V.from_tokens(toks)
    table = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    rng = np.random.default_rng(0)
    B, k = 400, 5
    runs = rng.integers(0, len(toks), size=(B, k), dtype=np.int32)
    hist, n_valid = oracle.advance_tokens(table, np.full(B, d.start, np.int32), runs)
    full = re.compile(pattern)

    def viable(text: bytes) -> bool:       # can be completed: try all short continuations over the alphabet
        frontier = {text}
        for _ in range(3):
            if any(full.fullmatch(x.decode()) for x in frontier):
                return True
            frontier = {x + c for x in frontier for c in (b"a", b"b", b"c", b"d", b"e")}
        return any(full.fullmatch(x.decode()) for x in frontier)

    for b in range(B):
        text = b""
        alive = True
        for i in range(k):
            text += toks[runs[b, i]]
            alive = alive and viable(text)
            assert (hist[b, i + 1] != DEAD) == alive, (b, i, text)
            if alive:
                assert bool(d.accept[hist[b, i + 1]]) == bool(full.fullmatch(text.decode()))
        assert n_valid[b] == sum(1 for i in range(k) if hist[b, i + 1] != DEAD)
        assert (hist[b, 1:n_valid[b] + 1] != DEAD).all() and (hist[b, n_valid[b] + 1:] == DEAD).all()


def test_runs_equal_chained_single_steps(oracle):
    """history[i + 1] is what a decode step that chose tokens[i] would have advanced to."""
    rng = np.random.default_rng(1)
    n_rows, n_tok = 9, 50
    table = rng.integers(0, n_rows, size=(n_rows, n_tok), dtype=np.int32)
    table[rng.random((n_rows, n_tok)) < 0.5] = DEAD
    states = np.array([0, 3, 8, DEAD, n_rows, 5], dtype=np.int32)
    runs = rng.integers(-1, n_tok + 1, size=(len(states), 7), dtype=np.int32)   # includes -1 and n_tok: not token ids
    hist, n_valid = oracle.advance_tokens(table, states, runs)
    for b, s in enumerate(states):
        s = int(s) if 0 <= s < n_rows else DEAD
        assert hist[b, 0] == s
        for i, t in enumerate(runs[b]):
            s = int(table[s, t]) if s != DEAD and 0 <= t < n_tok else DEAD
            assert hist[b, i + 1] == s
    h0, n0 = oracle.advance_tokens(table, states, np.zeros((len(states), 0), np.int32))
    assert h0.shape == (len(states), 1) and (n0 == 0).all()
