"""Test tooling for terminal labels (Section 2.5.1): a placeholder byte in a regex stands for a
terminal label; its transitions are taken out of the byte automaton and listed as terminal edges."""
from __future__ import annotations

import numpy as np

from workloads.regex_dfa import compile_regex


def dfa_with_terminals(pattern: bytes, placeholders: dict[int, int]):
    """(dfa without the placeholder transitions, edges [(state, label, target)]) for a pattern in
    which byte `b` stands for terminal label placeholders[b].  Edges are listed by state, then by
    label: that order is the precedence order."""
    d = compile_regex(pattern)
    edges = []
    for q in range(d.n_states):
        for b, label in sorted(placeholders.items(), key=lambda kv: kv[1]):
            if d.trans[q, b] >= 0:
                edges.append((q, label, int(d.trans[q, b])))
    for b in placeholders:
        d.trans[:, b] = -1
    return d, np.array(edges, dtype=np.int32).reshape(-1, 3)
