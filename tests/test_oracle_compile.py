"""Pins for the oracle's compile half: the paper's worked examples, brute force against
Python's `re` (an independent regex engine), Theorem 1, and table invariants."""
import itertools
import os
import re

import numpy as np
import pytest

from workloads import configs, vocab as V
from workloads.regex_dfa import compile_regex
import invariants as inv

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DEAD = -1


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.rstrip("\n") for ln in f if not ln.startswith("#") and ln.strip()]


def _hand_dfa(n, edges, accept):
    trans = np.full((n, 256), DEAD, dtype=np.int32)
    for s, ch, d in edges:
        trans[s, ord(ch)] = d
    acc = np.zeros(n, dtype=np.uint8)
    acc[list(accept)] = 1
    return trans, acc


def _both(oracle, trans, vocab):
    a = oracle.compile_compose(trans, vocab.data, vocab.offsets, block=3)
    b = oracle.compile_walk(trans, vocab.data, vocab.offsets)
    assert np.array_equal(a, b)
    return a


def _run(table, start, ids):
    q = start
    for t in ids:
        if q < 0:
            return DEAD
        q = int(table[q, t])
    return q


# ---------------------------------------------------------------- Figure 3 / Figure 4
def test_fig4_table(oracle):
    trans, acc = _hand_dfa(5, [(0, "f", 1), (1, "o", 2), (2, "o", 3), (3, "f", 1), (3, "d", 4)], {4})
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    golden = np.array([[int(x) for x in ln.split()] for ln in _lines("fig4_foo_table.txt")], dtype=np.int32)
    assert golden.shape == (5, 5)
    assert np.array_equal(_both(oracle, trans, vocab), golden)
    # caption of Figure 4: foo and f+oo are both accepted paths; food crosses into d
    t = golden
    assert _run(t, 0, [2]) == _run(t, 0, [0, 1]) == 3
    assert acc[_run(t, 0, [4])] and acc[_run(t, 0, [2, 4])] and acc[_run(t, 0, [0, 1, 0, 1, 4])]
    assert (t[:, 3] == DEAD).all()          # "for" never fits
    # the regex compiler (input tooling) gives the same automaton with the same numbering
    d = compile_regex(r"(foo)+d")
    assert np.array_equal(d.trans, trans) and np.array_equal(d.accept, acc) and d.start == 0


# ---------------------------------------------------------------- Appendix A
def test_appendixA_tokenizations(oracle):
    seqs = [ln.split(" ") for ln in _lines("appendixA_tokenizations.txt")]
    pieces = []
    for s in seqs:
        for p in s:
            if p not in pieces:
                pieces.append(p)
    assert len(pieces) == 14
    d = compile_regex(r"foo\(123\)|bar\(456\)")
    vocab = V.from_tokens([p.encode() for p in pieces])
    table = _both(oracle, d.trans, vocab)
    for s in seqs:
        ids = [pieces.index(p) for p in s]
        assert "".join(s) in ("foo(123)", "bar(456)")
        q = _run(table, d.start, ids)
        assert q >= 0 and d.accept[q], s
        assert _run(table, d.start, ids[::-1]) == DEAD
        assert not d.accept[_run(table, d.start, ids[:-1])]
    # mixing the calls is rejected: fo o(1 then 5
    assert _run(table, d.start, [pieces.index("fo"), pieces.index("o(1"), pieces.index("5")]) == DEAD


# ---------------------------------------------------------------- Figure 7 vocabulary
def test_fig7_vocab_bounded(oracle):
    toks = _lines("fig7_vocab.txt")
    assert toks == ["a", "b", "bb", "aaab"]
    d = compile_regex(r"ab|aabb|aaabbb")
    table = _both(oracle, d.trans, V.from_tokens([t.encode() for t in toks]))
    a, b, bb, aaab = 0, 1, 2, 3
    assert d.accept[_run(table, 0, [aaab, bb])]
    assert d.accept[_run(table, 0, [a, a, a, b, b, b])]
    q = _run(table, 0, [aaab, b])
    assert q >= 0 and not d.accept[q]
    assert _run(table, 0, [aaab, bb, b]) == DEAD


# ---------------------------------------------------------------- Theorem 2 by brute force
BRUTE = [
    (r"(ab)*c", [b"a", b"b", b"c", b"ab", b"ba", b"bc", b"abc", b"cab", b"abab", b"", b"ab"], "abc", 2),
    (r"a{1,3}b?|ba", [b"a", b"b", b"aa", b"ab", b"ba", b"aab", b"aaa", b"bab", b"aaab"], "ab", 2),
    (r"(foo)+d", [b"f", b"oo", b"foo", b"for", b"food", b"o", b"d", b"od", b"of"], "fodr", 4),
    (r"x(y|zz)*x?", [b"x", b"y", b"z", b"zz", b"xy", b"yz", b"zx", b"xx", b"zzx", b"yzz"], "xyz", 1),
]


@pytest.mark.parametrize("pattern,toks,alphabet,k_complete", BRUTE)
def test_theorem2_bruteforce(oracle, pattern, toks, alphabet, k_complete):
    """All token sequences up to length 4: accepting <=> re.fullmatch(D(x)); alive <=> D(x) can
    still be completed to a match (completion searched by brute force over the alphabet)."""
    d = compile_regex(pattern)
    vocab = V.from_tokens(toks)
    table = _both(oracle, d.trans, vocab)
    cre = re.compile(pattern.encode())
    exts = [b""]
    for k in range(1, k_complete + 1):
        exts += [bytes(p) for p in itertools.product(alphabet.encode(), repeat=k)]
    viable_cache = {}

    def viable(text):
        v = viable_cache.get(text)
        if v is None:
            v = any(cre.fullmatch(text + e) for e in exts)
            viable_cache[text] = v
        return v

    n = len(toks)
    checked = 0
    for L in range(0, 5):
        for ids in itertools.product(range(n), repeat=L):
            if any(len(toks[i]) == 0 for i in ids):
                assert _run(table, d.start, ids) == DEAD     # a zero-length token is never allowed
                continue
            text = b"".join(toks[i] for i in ids)
            q = _run(table, d.start, ids)
            assert (q >= 0 and bool(d.accept[q])) == (cre.fullmatch(text) is not None), ids
            assert (q >= 0) == viable(text), (ids, text)
            checked += 1
    assert checked > 5000


# ---------------------------------------------------------------- Theorem 1
def test_theorem1_transducer(oracle):
    rng = np.random.default_rng(7)
    for toks in ([b"f", b"oo", b"foo", b"for", b"food"], [b"a", b"b", b"bb", b"aaab"],
                 configs.small(1, n_tokens=40).vocab.tokens()):
        vocab = V.from_tokens(toks)
        fst = oracle.build_detok_fst(vocab.data, vocab.offsets)
        lens = [len(t) for t in toks]
        # structure stated in Appendix B.1.1: one cycle per token through the root
        assert fst.n_states == 1 + sum(max(n - 1, 0) for n in lens)
        assert len(fst.edges) == sum(lens)
        e = fst.edges
        for t, n in enumerate(lens):
            closing = e[e[:, 1] == t]
            assert len(closing) == (1 if n else 0)
            if n:
                assert closing[0, 3] == fst.root and closing[0, 2] == toks[t][-1]
        assert (e[e[:, 1] == -1][:, 3] != fst.root).all()      # epsilon-input edges go down a chain
        for _ in range(200):
            ids = rng.integers(0, len(toks), size=int(rng.integers(0, 7)))
            ids = [int(i) for i in ids if lens[int(i)] > 0]
            assert oracle.fst_transduce(fst, ids) == b"".join(toks[i] for i in ids)
    # a zero-length token has no cycle, so a sequence holding it is outside the domain
    vocab = V.from_tokens([b"a", b"", b"bc"])
    fst = oracle.build_detok_fst(vocab.data, vocab.offsets)
    assert oracle.fst_transduce(fst, [0, 1]) is None
    assert oracle.fst_transduce(fst, [0, 2, 0]) == b"abca"


# ---------------------------------------------------------------- two routes, invariants
@pytest.mark.parametrize("seed", range(6))
def test_compose_equals_walk_small(oracle, seed):
    w = configs.small(seed)
    d = w.dfas[0]
    table = _both(oracle, d.trans, w.vocab)
    inv.check_range(table, d.n_states)
    assert inv.check_singletons(table, d.trans, w.vocab) >= 3
    assert inv.check_concatenation(table, w.vocab, np.random.default_rng(seed), 300) > 20
    inv.check_liveness(table, d.accept, d.start)
    # blocks and threads do not change the result
    again = oracle.compile_compose(d.trans, w.vocab.data, w.vocab.offsets, block=5, n_threads=3)
    assert np.array_equal(again, table)
    part = oracle.compile_compose(d.trans, w.vocab.data, w.vocab.offsets, q_lo=2, q_hi=5, block=2)
    assert np.array_equal(part, table[2:5])


def test_c1_full(oracle):
    w = configs.get("c1")
    d = w.dfas[0]
    table = _both(oracle, d.trans, w.vocab)
    assert table.shape == (d.n_states, 512)
    assert inv.check_singletons(table, d.trans, w.vocab) == 95
    assert inv.check_concatenation(table, w.vocab, np.random.default_rng(1), 500) > 50
    assert inv.check_liveness(table, d.accept, d.start) > 5
    # tokens are matched against Python's re on detokenized text along random token walks
    cre = re.compile(w.patterns[0].encode())
    toks = w.vocab.tokens()
    rng = np.random.default_rng(2)
    accepted = 0
    for _ in range(300):
        q, text = d.start, b""
        for _ in range(12):
            live = np.nonzero(table[q] >= 0)[0]
            if len(live) == 0:
                break
            t = int(rng.choice(live))
            q, text = int(table[q, t]), text + toks[t]
            ok = cre.fullmatch(text) is not None
            assert ok == bool(d.accept[q])
            accepted += ok
    assert accepted > 0


def test_c2_rows_compose_equals_walk(oracle):
    w = configs.get("c2")
    d = w.dfas[0]
    walk = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=4)
    rows = oracle.compile_compose(d.trans, w.vocab.data, w.vocab.offsets, q_lo=40, q_hi=72, block=8,
                                  n_threads=4)
    assert np.array_equal(rows, walk[40:72])
    assert inv.check_singletons(walk, d.trans, w.vocab) == 256
    assert inv.check_concatenation(walk, w.vocab, np.random.default_rng(3), 500) > 100
    inv.check_liveness(walk, d.accept, d.start)


def test_duplicate_and_empty_tokens(oracle):
    d = compile_regex(r"(ab)*c")
    vocab = V.from_tokens([b"ab", b"", b"ab", b"c", b""])
    table = _both(oracle, d.trans, vocab)
    assert np.array_equal(table[:, 0], table[:, 2])
    assert (table[:, 1] == DEAD).all() and (table[:, 4] == DEAD).all()
    assert table[0, 0] == 0 or table[0, 0] >= 0


def test_bad_arguments(oracle):
    trans = np.full((2, 256), 5, dtype=np.int32)          # target outside [ -1, n )
    vocab = V.from_tokens([b"a"])
    with pytest.raises(RuntimeError):
        oracle.compile_compose(trans, vocab.data, vocab.offsets)
