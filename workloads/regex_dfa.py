"""Regular expression -> minimal, trim, byte-level DFA (input tooling only).

This module only *makes inputs*: it turns a regular expression (mathematical
regexes, no backreferences) into the deterministic character-level automaton
A_R that the constrained-decoding method takes as given (Section 2.1: FSAs,
determinism; Section 2.4, Algorithm 2: BuildRegexFSA).  It holds none of the
method's own arithmetic (no vocabulary, no composition, no masking).

Pipeline: parse -> Thompson NFA over byte sets -> subset construction over
byte equivalence classes -> Moore/Hopcroft-style partition refinement ->
removal of states that cannot reach an accepting state (trim) -> breadth-first
renumbering from the start state (start = 0).

Supported syntax (bytes, ASCII patterns): literals, escapes (\\n \\t \\r \\\\ and
any escaped punctuation, \\d \\w \\s), classes [a-z0-9_], negated classes
[^"\\\\] (complement over all 256 byte values), '.', groups ( ) and (?: ),
alternation |, quantifiers * + ? {m} {m,} {m,n}.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass

import numpy as np

DEAD = -1
ALL_BYTES = (1 << 256) - 1


@dataclass
class CharDFA:
    """Deterministic byte automaton: trans[q, b] is the next state or DEAD."""
    trans: np.ndarray    # int32 [n_states, 256], DEAD = -1
    accept: np.ndarray   # uint8 [n_states], 1 = final state
    start: int

    @property
    def n_states(self) -> int:
        return int(self.trans.shape[0])

    def run(self, data: bytes, state: int | None = None) -> int:
        q = self.start if state is None else state
        for b in data:
            if q < 0:
                return DEAD
            q = int(self.trans[q, b])
        return q

    def accepts(self, data: bytes) -> bool:
        q = self.run(data)
        return q >= 0 and bool(self.accept[q])


# --------------------------------------------------------------------------- parser
def _set(*bs: int) -> int:
    m = 0
    for b in bs:
        m |= 1 << b
    return m


def _range(lo: int, hi: int) -> int:
    return ((1 << (hi + 1)) - 1) & ~((1 << lo) - 1)


_DIGIT = _range(0x30, 0x39)
_WORD = _DIGIT | _range(0x41, 0x5A) | _range(0x61, 0x7A) | _set(0x5F)
_SPACE = _set(0x20, 0x09, 0x0A, 0x0D, 0x0B, 0x0C)
_ESC_SINGLE = {ord("n"): 0x0A, ord("t"): 0x09, ord("r"): 0x0D, ord("f"): 0x0C, ord("v"): 0x0B,
               ord("0"): 0x00}
_ESC_CLASS = {ord("d"): _DIGIT, ord("w"): _WORD, ord("s"): _SPACE,
              ord("D"): ALL_BYTES & ~_DIGIT, ord("W"): ALL_BYTES & ~_WORD,
              ord("S"): ALL_BYTES & ~_SPACE}


class _Parser:
    """Recursive descent over the pattern bytes; builds a small tuple AST.

    AST nodes: ('set', mask) | ('cat', [nodes]) | ('alt', [nodes]) |
               ('rep', node, lo, hi_or_None) | ('eps',)
    """

    def __init__(self, pattern: bytes):
        self.p = pattern
        self.i = 0
        self.positive = 0     # union of the byte sets written positively (not via [^...] or .)

    def peek(self) -> int | None:
        return self.p[self.i] if self.i < len(self.p) else None

    def take(self) -> int:
        c = self.p[self.i]
        self.i += 1
        return c

    def parse(self):
        node = self.alt()
        if self.i != len(self.p):
            raise ValueError(f"unexpected {chr(self.p[self.i])!r} at {self.i}")
        return node

    def alt(self):
        parts = [self.cat()]
        while self.peek() == ord("|"):
            self.take()
            parts.append(self.cat())
        return parts[0] if len(parts) == 1 else ("alt", parts)

    def cat(self):
        items = []
        while self.peek() is not None and self.peek() not in (ord("|"), ord(")")):
            items.append(self.repeat())
        if not items:
            return ("eps",)
        return items[0] if len(items) == 1 else ("cat", items)

    def repeat(self):
        node = self.atom()
        while True:
            c = self.peek()
            if c == ord("*"):
                self.take(); node = ("rep", node, 0, None)
            elif c == ord("+"):
                self.take(); node = ("rep", node, 1, None)
            elif c == ord("?"):
                self.take(); node = ("rep", node, 0, 1)
            elif c == ord("{"):
                self.take()
                lo = self.number()
                hi: int | None = lo
                if self.peek() == ord(","):
                    self.take()
                    hi = None if self.peek() == ord("}") else self.number()
                if self.take() != ord("}"):
                    raise ValueError("expected }")
                if hi is not None and hi < lo:
                    raise ValueError("bad repeat bounds")
                node = ("rep", node, lo, hi)
            else:
                return node

    def number(self) -> int:
        s = self.i
        while self.peek() is not None and 0x30 <= self.peek() <= 0x39:
            self.take()
        if s == self.i:
            raise ValueError("expected number")
        return int(self.p[s:self.i])

    def escape(self) -> int:
        """Byte set denoted by the escape whose backslash was just consumed."""
        c = self.take()
        if c in _ESC_CLASS:
            return _ESC_CLASS[c]
        if c in _ESC_SINGLE:
            return _set(_ESC_SINGLE[c])
        if c == ord("x"):
            v = int(self.p[self.i:self.i + 2], 16)
            self.i += 2
            return _set(v)
        return _set(c)

    def atom(self):
        c = self.take()
        if c == ord("("):
            if self.p[self.i:self.i + 2] == b"?:":
                self.i += 2
            node = self.alt()
            if self.peek() != ord(")"):
                raise ValueError("expected )")
            self.take()
            return node
        if c == ord("["):
            return ("set", self.char_class())
        if c == ord("."):
            return ("set", ALL_BYTES & ~_set(0x0A))
        if c == ord("\\"):
            m = self.escape()
            if bin(m).count("1") <= 128:
                self.positive |= m
            return ("set", m)
        if c in b"*+?{":
            raise ValueError(f"nothing to repeat at {self.i - 1}")
        self.positive |= _set(c)
        return ("set", _set(c))

    def char_class(self) -> int:
        neg = False
        if self.peek() == ord("^"):
            self.take(); neg = True
        mask = 0
        first = True
        while True:
            c = self.take()
            if c == ord("]") and not first:
                break
            first = False
            if c == ord("\\"):
                m = self.escape()
                single = m if m & (m - 1) == 0 else None
            else:
                m = _set(c)
                single = m
            if (single is not None and self.peek() == ord("-")
                    and self.i + 1 < len(self.p) and self.p[self.i + 1] != ord("]")):
                self.take()
                d = self.take()
                if d == ord("\\"):
                    hm = self.escape()
                    if hm & (hm - 1):
                        raise ValueError("bad range end")
                    hi = hm.bit_length() - 1
                else:
                    hi = d
                lo = single.bit_length() - 1
                if hi < lo:
                    raise ValueError("bad range")
                m = _range(lo, hi)
            mask |= m
        if not neg:
            self.positive |= mask
        return (ALL_BYTES & ~mask) if neg else mask


# --------------------------------------------------------------------------- NFA
class _NFA:
    def __init__(self):
        self.eps: list[list[int]] = []
        self.edges: list[list[tuple[int, int]]] = []   # (byte-set mask, dst)

    def new(self) -> int:
        self.eps.append([])
        self.edges.append([])
        return len(self.eps) - 1

    def build(self, node) -> tuple[int, int]:
        """Thompson fragment (entry, exit) for an AST node."""
        kind = node[0]
        if kind == "eps":
            s = self.new(); t = self.new(); self.eps[s].append(t); return s, t
        if kind == "set":
            s = self.new(); t = self.new(); self.edges[s].append((node[1], t)); return s, t
        if kind == "cat":
            s, t = self.build(node[1][0])
            for sub in node[1][1:]:
                s2, t2 = self.build(sub)
                self.eps[t].append(s2)
                t = t2
            return s, t
        if kind == "alt":
            s = self.new(); t = self.new()
            for sub in node[1]:
                s2, t2 = self.build(sub)
                self.eps[s].append(s2); self.eps[t2].append(t)
            return s, t
        if kind == "rep":
            _, sub, lo, hi = node
            s = self.new(); t = s
            for _ in range(lo):
                s2, t2 = self.build(sub)
                self.eps[t].append(s2); t = t2
            if hi is None:
                s2, t2 = self.build(sub)
                loop_in = self.new(); out = self.new()
                self.eps[t].append(loop_in)
                self.eps[loop_in].append(s2); self.eps[loop_in].append(out)
                self.eps[t2].append(loop_in)
                t = out
            else:
                out = self.new()
                for _ in range(hi - lo):
                    self.eps[t].append(out)
                    s2, t2 = self.build(sub)
                    self.eps[t].append(s2); t = t2
                self.eps[t].append(out)
                t = out
            return s, t
        raise AssertionError(kind)


def _byte_classes(masks: list[int]) -> tuple[np.ndarray, int]:
    """Partition 0..255 so bytes in one class occur in exactly the same edge sets."""
    sig: dict[tuple, int] = {}
    cls = np.zeros(256, dtype=np.int32)
    distinct = sorted(set(masks))
    for b in range(256):
        key = tuple(i for i, m in enumerate(distinct) if (m >> b) & 1)
        cls[b] = sig.setdefault(key, len(sig))
    return cls, len(sig)


def regex_alphabet(pattern: str | bytes) -> np.ndarray:
    """Bytes the pattern names positively (literals and non-negated classes), sorted."""
    if isinstance(pattern, str):
        pattern = pattern.encode("latin-1")
    ps = _Parser(pattern)
    ps.parse()
    return np.array([b for b in range(256) if (ps.positive >> b) & 1], dtype=np.uint8)


def compile_regex(pattern: str | bytes) -> CharDFA:
    """Minimal trim DFA over bytes for `pattern` (full-match semantics)."""
    if isinstance(pattern, str):
        pattern = pattern.encode("latin-1")
    ast = _Parser(pattern).parse()
    nfa = _NFA()
    n_start, n_final = nfa.build(ast)
    n = len(nfa.eps)

    cls, n_cls = _byte_classes([m for es in nfa.edges for m, _ in es])
    rep = [int(np.nonzero(cls == c)[0][0]) for c in range(n_cls)]

    # epsilon closures, memoised per NFA state
    closure_cache: dict[int, frozenset[int]] = {}

    def closure_of(seed_states) -> frozenset[int]:
        out: set[int] = set()
        for s0 in seed_states:
            c = closure_cache.get(s0)
            if c is None:
                seen = {s0}; stack = [s0]
                while stack:
                    u = stack.pop()
                    for v in nfa.eps[u]:
                        if v not in seen:
                            seen.add(v); stack.append(v)
                c = frozenset(seen)
                closure_cache[s0] = c
            out |= c
        return frozenset(out)

    # per NFA state: list of (class id -> dst) moves
    moves: list[list[tuple[int, int]]] = []
    for s in range(n):
        mv = []
        for m, d in nfa.edges[s]:
            for c in range(n_cls):
                if (m >> rep[c]) & 1:
                    mv.append((c, d))
        moves.append(mv)

    start_set = closure_of([n_start])
    ids = {start_set: 0}
    order = [start_set]
    ctrans: list[list[int]] = []
    qi = 0
    while qi < len(order):
        cur = order[qi]; qi += 1
        by_cls: dict[int, set[int]] = {}
        for s in cur:
            for c, d in moves[s]:
                by_cls.setdefault(c, set()).add(d)
        row = [DEAD] * n_cls
        for c, dsts in by_cls.items():
            tgt = closure_of(dsts)
            j = ids.get(tgt)
            if j is None:
                j = len(order); ids[tgt] = j; order.append(tgt)
            row[c] = j
        ctrans.append(row)
    nd = len(order)
    T = np.array(ctrans, dtype=np.int64).reshape(nd, n_cls)
    acc = np.array([n_final in s for s in order], dtype=bool)

    # trim: keep states from which an accepting state is reachable
    rev: list[list[int]] = [[] for _ in range(nd)]
    for s in range(nd):
        for d in set(T[s].tolist()):
            if d >= 0:
                rev[d].append(s)
    live = acc.copy()
    dq = deque(np.nonzero(acc)[0].tolist())
    while dq:
        u = dq.popleft()
        for v in rev[u]:
            if not live[v]:
                live[v] = True; dq.append(v)
    if not live[0]:
        raise ValueError("regex matches nothing")
    T = np.where((T >= 0) & live[np.clip(T, 0, None)], T, DEAD)

    # partition refinement (Moore) on live states; the implicit DEAD sink is its own block
    live_idx = np.nonzero(live)[0]
    block = np.full(nd, -1, dtype=np.int64)
    block[live_idx] = acc[live_idx].astype(np.int64)
    while True:
        tb = np.where(T[live_idx] >= 0, block[np.clip(T[live_idx], 0, None)], -1)
        sig = np.concatenate([block[live_idx, None], tb], axis=1)
        _, new = np.unique(sig, axis=0, return_inverse=True)
        new = new.reshape(-1)
        changed = len(np.unique(new)) != len(np.unique(block[live_idx]))
        block[live_idx] = new
        if not changed:
            break
    nb = int(block[live_idx].max()) + 1
    rep_state = np.full(nb, -1, dtype=np.int64)
    for s in live_idx[::-1]:
        rep_state[block[s]] = s
    MT = np.where(T[rep_state] >= 0, block[np.clip(T[rep_state], 0, None)], DEAD)
    macc = acc[rep_state]

    # breadth-first renumbering from the start block (drops nothing: all are reachable)
    new_id = np.full(nb, -1, dtype=np.int64)
    bfs = [int(block[0])]
    new_id[bfs[0]] = 0
    k = 0
    while k < len(bfs):
        u = bfs[k]; k += 1
        for d in MT[u].tolist():
            if d >= 0 and new_id[d] < 0:
                new_id[d] = len(bfs); bfs.append(d)
    assert len(bfs) == nb
    bfs_arr = np.array(bfs)
    MT = MT[bfs_arr]
    MT = np.where(MT >= 0, new_id[np.clip(MT, 0, None)], DEAD)
    trans = MT[:, cls].astype(np.int32)           # expand classes back to 256 bytes
    return CharDFA(trans=np.ascontiguousarray(trans),
                   accept=macc[bfs_arr].astype(np.uint8), start=0)


def random_dfa(n_states: int, p_dead: float, p_accept: float, rng: np.random.Generator) -> CharDFA:
    """Seeded random complete-table DFA over 256 bytes, used as drawn (not minimised/trimmed)."""
    dst = rng.integers(0, n_states, size=(n_states, 256), dtype=np.int32)
    dead = rng.random((n_states, 256)) < p_dead
    trans = np.where(dead, np.int32(DEAD), dst).astype(np.int32)
    accept = (rng.random(n_states) < p_accept).astype(np.uint8)
    return CharDFA(trans=trans, accept=accept, start=0)
