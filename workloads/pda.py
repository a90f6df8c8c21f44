"""Character-level push-down automata used as inputs (Section 3.1 of the paper): a container and a
few hand-built deterministic automata.  Input tooling only: nothing here computes a token edge.

An edge is (source, input, pops, target, pushes): input a byte value or EPS, pops / pushes
tuples of stack symbols written bottom to top.  By convention here symbol 0 is the initial stack
symbol S, and a run starts in `start` with the stack (0,).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

EPS = -1
S0 = 0          # the initial stack symbol


@dataclass
class CharPDA:
    n_states: int
    start: int
    accept: np.ndarray        # uint8 [n_states]
    src: np.ndarray           # int32 [n_edges], sorted
    input: np.ndarray         # int32 [n_edges], byte or EPS
    dst: np.ndarray
    pop_begin: np.ndarray     # int32 [n_edges + 1]
    pop_syms: np.ndarray
    push_begin: np.ndarray
    push_syms: np.ndarray

    @property
    def n_edges(self) -> int:
        return len(self.src)

    def edges(self):
        for e in range(self.n_edges):
            yield (int(self.src[e]), int(self.input[e]), tuple(self.pop_syms[self.pop_begin[e]:self.pop_begin[e + 1]].tolist()),
                   int(self.dst[e]), tuple(self.push_syms[self.push_begin[e]:self.push_begin[e + 1]].tolist()))


def make_pda(n_states: int, start: int, accept_states, edges) -> CharPDA:
    """edges: iterable of (src, input, pops, dst, pushes); input may be a one-byte bytes/str, an int or EPS."""
    norm = []
    for (s, a, pops, d, pushes) in edges:
        if isinstance(a, str):
            a = a.encode("latin-1")
        if isinstance(a, (bytes, bytearray)):
            assert len(a) == 1
            a = a[0]
        norm.append((int(s), int(a), tuple(pops), int(d), tuple(pushes)))
    norm.sort(key=lambda e: e[0])            # stable: the given order is kept inside a state
    acc = np.zeros(n_states, dtype=np.uint8)
    acc[list(accept_states)] = 1
    pop_begin, push_begin, pop_syms, push_syms = [0], [0], [], []
    for e in norm:
        pop_syms += list(e[2])
        push_syms += list(e[4])
        pop_begin.append(len(pop_syms))
        push_begin.append(len(push_syms))
    i32 = lambda x: np.array(x, dtype=np.int32)
    return CharPDA(n_states, start, acc, i32([e[0] for e in norm]), i32([e[1] for e in norm]), i32([e[3] for e in norm]),
                   i32(pop_begin), i32(pop_syms), i32(push_begin), i32(push_syms))


def anbn() -> CharPDA:
    """The language a^n b^n, n >= 1, of the grammar S -> ab | a S b (Fig. 6), with the inner S entered on its
    first `a` and a return symbol R per nesting level; the run ends by popping the initial symbol."""
    R = 1
    return make_pda(5, 0, [4], [
        (0, "a", (), 1, ()),
        (1, "a", (), 1, (R,)),            # the a of an inner S: remember to come back
        (1, "b", (), 2, ()),              # S -> ab complete
        (2, EPS, (R,), 3, ()),            # return into S -> a S . b
        (3, "b", (), 2, ()),
        (2, EPS, (S0,), 4, ()),           # the outermost S is complete
    ])


def dyck2() -> CharPDA:
    """Balanced strings over () and [] (the empty string included).  State 0 = nothing open (final),
    state 1 = something open; a closing bracket looks at the symbol below the one it pops."""
    P, B = 1, 2
    edges = [(0, "(", (), 1, (P,)), (0, "[", (), 1, (B,)), (1, "(", (), 1, (P,)), (1, "[", (), 1, (B,))]
    for close, sym in ((")", P), ("]", B)):
        edges.append((1, close, (S0, sym), 0, (S0,)))
        edges.append((1, close, (P, sym), 1, (P,)))
        edges.append((1, close, (B, sym), 1, (B,)))
    return make_pda(2, 0, [0], edges)


def call_grammar() -> CharPDA:
    """S -> Function "(" Number ")", Function -> "foo" | "bar", Number -> "123" | "456" (Appendix A.2), with
    the two non-terminals entered and left through epsilon edges that push and pop return symbols."""
    R1, R2 = 1, 2
    e = [(0, EPS, (), 1, (R1,))]                                  # call Function
    e += [(1, "f", (), 2, ()), (2, "o", (), 3, ()), (3, "o", (), 7, ()),
          (1, "b", (), 4, ()), (4, "a", (), 5, ()), (5, "r", (), 7, ())]
    e += [(7, EPS, (R1,), 8, ()), (8, "(", (), 9, ()), (9, EPS, (), 10, (R2,))]   # return, "(", call Number
    e += [(10, "1", (), 11, ()), (11, "2", (), 12, ()), (12, "3", (), 16, ()),
          (10, "4", (), 13, ()), (13, "5", (), 14, ()), (14, "6", (), 16, ())]
    e += [(16, EPS, (R2,), 17, ()), (17, ")", (), 18, ())]
    return make_pda(19, 0, [18], e)


def int_lists() -> CharPDA:
    """value := digits | "[" "]" | "[" value ("," value)* "]", nested to any depth.
    States: 0 expect the top-level value; 6 top-level number (final); 7 top-level list closed (final);
    1 just after "["; 2 inside a nested number; 3 after a nested value; 4 after ","."""
    L = 1
    e = []
    for dch in "0123456789":
        e += [(0, dch, (), 6, ()), (6, dch, (), 6, ()), (1, dch, (), 2, ()), (2, dch, (), 2, ()), (4, dch, (), 2, ())]
    for s in (0, 1, 4):
        e.append((s, "[", (), 1, (L,)))
    for s in (1, 2, 3):                                           # "]" closes a list: the outermost one ends the value
        e.append((s, "]", (S0, L), 7, (S0,)))
        e.append((s, "]", (L, L), 3, (L,)))
    for s in (2, 3):
        e.append((s, ",", (L,), 4, (L,)))
    return make_pda(8, 0, [6, 7], e)


def dfa_as_pda(trans: np.ndarray, accept: np.ndarray, start: int) -> CharPDA:
    """A finite automaton as a push-down automaton that never touches its stack."""
    edges = [(q, b, (), int(trans[q, b]), ()) for q in range(trans.shape[0]) for b in range(256) if trans[q, b] >= 0]
    return make_pda(trans.shape[0], start, np.nonzero(accept)[0].tolist(), edges)


def run_chars(pda: CharPDA, text: bytes, stack=(S0,)):
    """Direct simulation of the character-level automaton (deterministic: the first edge that can be taken is
    the only one): returns (state, stack) after `text` and the epsilon edges that precede each byte, or None."""
    by_src: dict[int, list] = {}
    for ed in pda.edges():
        by_src.setdefault(ed[0], []).append(ed)
    q, st = pda.start, list(stack)

    def take(sym):
        nonlocal q, st
        for (_, a, pops, d, pushes) in by_src.get(q, []):
            if a == sym and (len(pops) == 0 or tuple(st[len(st) - len(pops):]) == pops) and len(pops) <= len(st):
                del st[len(st) - len(pops):]
                st += list(pushes)
                q = d
                return True
        return False

    for ch in text:
        guard = 0
        while not any(a == ch and len(p) <= len(st) and (len(p) == 0 or tuple(st[len(st) - len(p):]) == p)
                      for (_, a, p, _, _) in by_src.get(q, [])):
            if not take(EPS):
                return None
            guard += 1
            if guard > 64:
                return None
        take(ch)
    return q, tuple(st)


def json_like() -> CharPDA:
    """Nested JSON without white space, escapes or fractions: the top-level value is an array or an object;
    values are arrays, objects, strings over [a-z0-9_ ], integers (no leading zeros), true, false, null.
    The stack holds one symbol per open container (A array, O object) above the initial symbol."""
    A, O = 1, 2
    names = ["V0", "DONE", "EVA", "EV", "EKO", "EK", "KS", "KE", "S", "N", "N0", "NM", "AV",
             "t1", "t2", "t3", "f1", "f2", "f3", "f4", "n1", "n2", "n3"]
    st = {n: i for i, n in enumerate(names)}
    e = []
    add = lambda s, ch, pops, d, pushes: e.append((st[s], ch, pops, st[d], pushes))
    add("V0", "[", (), "EVA", (A,))
    add("V0", "{", (), "EKO", (O,))
    for s in ("EVA", "EV"):                                      # a value starts
        add(s, "[", (), "EVA", (A,))
        add(s, "{", (), "EKO", (O,))
        add(s, '"', (), "S", ())
        add(s, "-", (), "NM", ())
        add(s, "0", (), "N0", ())
        for dch in "123456789":
            add(s, dch, (), "N", ())
        add(s, "t", (), "t1", ())
        add(s, "f", (), "f1", ())
        add(s, "n", (), "n1", ())
    add("NM", "0", (), "N0", ())
    for dch in "123456789":
        add("NM", dch, (), "N", ())
    for dch in "0123456789":
        add("N", dch, (), "N", ())
    for a, b, ch in (("t1", "t2", "r"), ("t2", "t3", "u"), ("t3", "AV", "e"), ("f1", "f2", "a"), ("f2", "f3", "l"), ("f3", "f4", "s"),
                     ("f4", "AV", "e"), ("n1", "n2", "u"), ("n2", "n3", "l"), ("n3", "AV", "l")):
        add(a, ch, (), b, ())
    for ch in "abcdefghijklmnopqrstuvwxyz0123456789_ ":
        add("S", ch, (), "S", ())
        add("KS", ch, (), "KS", ())
    add("S", '"', (), "AV", ())
    add("KS", '"', (), "KE", ())
    add("KE", ":", (), "EV", ())
    add("EKO", '"', (), "KS", ())
    add("EK", '"', (), "KS", ())
    for s in ("AV", "N", "N0"):                                  # after a value
        add(s, ",", (A,), "EV", (A,))
        add(s, ",", (O,), "EK", (O,))
    for s, close, sym in [(x, "]", A) for x in ("EVA", "AV", "N", "N0")] + [(x, "}", O) for x in ("EKO", "AV", "N", "N0")]:
        add(s, close, (S0, sym), "DONE", (S0,))
        add(s, close, (A, sym), "AV", (A,))
        add(s, close, (O, sym), "AV", (O,))
    return make_pda(len(names), st["V0"], [st["DONE"]], e)
