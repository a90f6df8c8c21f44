"""Pins for the oracle's terminal labels (Section 2.5.1): a hand-derived example with both kinds
of ambiguity the paper names, an independent per-entry evaluation of the rule, and soundness
against Python's `re` on a bulleted-list constraint of the kind the paper describes."""
import itertools
import re

import numpy as np

from workloads import vocab as V
from terminals_util import dfa_with_terminals

DEAD = -1
T1, T2 = 0xFE, 0xFF          # placeholder bytes for two terminal labels


def _walk(trans, q, data):
    for b in data:
        if q < 0:
            return DEAD
        q = int(trans[q, b])
    return q


def test_hand_example(oracle):
    """a (T)+ b with T = {x, ab, b}: 'b' after the first T is both a normal edge and in the mask."""
    d, edges = dfa_with_terminals(b"a\xff+b", {T2: 0})
    toks = [b"a", b"b", b"x", b"ab", b"bb"]
    vocab = V.from_tokens(toks)
    base = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    s0 = d.start
    s1 = int(d.trans[s0, ord("a")])
    assert (base[s1] == DEAD).all()                              # s1 has only the terminal edge
    assert [tuple(e) for e in edges if e[0] == s1] == [(s1, 0, edges[0][2])]
    s2 = int(edges[edges[:, 0] == s1][0][2])
    s3 = int(d.trans[s2, ord("b")])
    assert d.accept[s3] and edges.tolist() == [[s1, 0, s2], [s2, 0, s2]] or edges.tolist() == [[s2, 0, s2], [s1, 0, s2]]
    mask = np.array([[0, 1, 1, 1, 0]], dtype=np.uint8)           # T = {b, x, ab}
    got = oracle.apply_terminals(base, edges, mask)
    A, B, X, AB, BB = range(5)
    assert got[s0].tolist() == base[s0].tolist()                 # no terminal edge leaves s0
    assert got[s1].tolist() == [DEAD, s2, s2, s2, DEAD]          # b, x, ab through the terminal edge
    assert got[s2].tolist() == [DEAD, s3, s2, s2, DEAD]          # b: the normal edge wins over the terminal
    assert base[s2].tolist() == [DEAD, s3, DEAD, DEAD, DEAD]


def test_precedence_of_terminals(oracle):
    """Two terminal edges out of one state whose masks overlap: the first in the order wins."""
    table = np.full((3, 4), DEAD, dtype=np.int32)
    table[0, 3] = 0
    masks = np.array([[1, 1, 0, 1], [0, 1, 1, 1]], dtype=np.uint8)
    got = oracle.apply_terminals(table, [(0, 0, 1), (0, 1, 2)], masks)
    assert got[0].tolist() == [1, 1, 2, 0]
    got = oracle.apply_terminals(table, [(0, 1, 2), (0, 0, 1)], masks)
    assert got[0].tolist() == [1, 2, 2, 0]
    assert (got[1:] == DEAD).all()
    assert np.array_equal(oracle.apply_terminals(table, np.zeros((0, 3), np.int32), masks), table)


def test_rule_entry_by_entry(oracle):
    """The rule evaluated separately for every (state, token): the normal edge if the bytes of the
    token can be walked, else the first terminal edge of the state whose mask holds the token."""
    rng = np.random.default_rng(0)
    d, edges = dfa_with_terminals(b"(k\xfe*;|v\xff{1,3}[.;]|k\xff\xfe)+", {T1: 0, T2: 1})
    alphabet = b"kv;.ab"
    toks = sorted({bytes(rng.choice(list(alphabet), size=rng.integers(1, 4)).tolist()) for _ in range(120)})
    vocab = V.from_tokens(toks)
    masks = (rng.random((2, len(toks))) < 0.4).astype(np.uint8)
    base = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    got = oracle.apply_terminals(base, edges, masks)
    assert len(edges) >= 4
    for q in range(d.n_states):
        for t, tok in enumerate(toks):
            want = _walk(d.trans, q, tok)
            if want == DEAD:
                for (s, l, to) in edges:
                    if s == q and masks[l, t]:
                        want = int(to)
                        break
            assert got[q, t] == want, (q, tok)


def test_bulleted_list_sound_against_re(oracle):
    """A heading followed by one or two bullets of newline-free tokens.  Every token sequence the
    table accepts spells a text of the language in which the terminal stands for any one token
    of its mask; and bullets made of mask tokens are accepted."""
    d, edges = dfa_with_terminals(b"S:(\n\\* \xff+){1,2}", {T2: 0})
    toks = [b"S:", b"S", b":", b"\n", b"* ", b"\n* ", b"a", b"bc", b"d\ne", b"*", b" "]
    vocab = V.from_tokens(toks)
    mask = np.array([[0 if b"\n" in t else 1 for t in toks]], dtype=np.uint8)       # tokens with no newline
    table = oracle.apply_terminals(oracle.compile_walk(d.trans, vocab.data, vocab.offsets), edges, mask)
    tok_alt = "|".join(re.escape(t.decode()) for t, m in zip(toks, mask[0]) if m)
    text_re = re.compile(rf"S:(?:\n\* (?:{tok_alt})+){{1,2}}")
    n_accept = 0
    for k in range(1, 6):
        for seq in itertools.product(range(len(toks)), repeat=k):
            q = d.start
            for t in seq:
                q = int(table[q, t]) if q != DEAD else DEAD
                if q == DEAD:
                    break
            if q != DEAD and d.accept[q]:
                n_accept += 1
                text = b"".join(toks[t] for t in seq).decode()
                assert text_re.fullmatch(text), seq
    assert n_accept > 50
    for seq in ([0, 5, 6], [0, 3, 4, 7, 6], [1, 2, 5, 6, 7], [0, 5, 6, 5, 7]):
        q = d.start
        for t in seq:
            q = int(table[q, t])
        assert q != DEAD and d.accept[q], seq
