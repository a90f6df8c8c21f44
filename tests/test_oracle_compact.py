"""Pins for the oracle's edge-list form of a table (the paper's own representation of A_{R o V} is
a list of edges; Section 2.5.1): the seven edges of the worked example of Figures 3/4 written out
by hand, the lookup rule of edges kept in token order, and the round trip through the expansion,
which is written separately."""
import numpy as np

from workloads import vocab as V
from workloads.regex_dfa import compile_regex

DEAD = -1


def test_fig4_edge_list(oracle):
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    row_begin, targets = oracle.compact(table)
    # s0: f->s1, foo->s3, food->s4 | s1: oo->s3 | s2: none | s3: as s0 | s4: none
    assert row_begin.tolist() == [0, 3, 4, 4, 7, 7]
    assert targets.tolist() == [1, 3, 4, 3, 1, 3, 4]


def test_lookup_and_round_trip(oracle):
    rng = np.random.default_rng(3)
    for n_rows, n_tokens, p_live in [(1, 1, 1.0), (7, 127, 0.5), (9, 128, 0.02), (6, 129, 0.9), (11, 1000, 0.3),
                                     (4, 5000, 0.0), (3, 640, 1.0)]:
        t = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
        t[rng.random((n_rows, n_tokens)) >= p_live] = DEAD
        row_begin, targets = oracle.compact(t)
        live = t >= 0
        assert row_begin[0] == 0 and np.array_equal(np.diff(row_begin), live.sum(1))
        assert np.array_equal(targets, t[live])                      # row-major order of the live entries
        # the lookup rule of the form, entry by entry, on a sample: the edge of an allowed token is
        # the one at its rank among the state's allowed tokens
        for _ in range(200):
            q, tok = int(rng.integers(n_rows)), int(rng.integers(n_tokens))
            if live[q, tok]:
                assert targets[row_begin[q] + live[q, :tok].sum()] == t[q, tok]
        assert np.array_equal(oracle.expand(live, row_begin, targets), t)


def test_expand_rejects_inconsistent_lists(oracle):
    import pytest
    allowed = np.array([[1, 0, 1], [0, 1, 0]], dtype=bool)
    with pytest.raises(RuntimeError):
        oracle.expand(allowed, [0, 1, 2], [5, 6, 7])                 # row 0 has two allowed tokens, one edge
    assert oracle.expand(allowed, [0, 2, 3], [5, 6, 7]).tolist() == [[5, -1, 6], [-1, 7, -1]]
