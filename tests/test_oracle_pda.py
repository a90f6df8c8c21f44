"""Pins of the push-down oracle (oracle/pda_oracle.c) against what the paper and the definitions fix:
the worked example of Figs. 6-7, Theorem 3 by brute force (P_{G o V}(x) = P_G(D(x))) with the
character automata themselves checked against hand-written recognisers, the algebra of
concatenated stack edits, the regular special case, detection of non-determinism, and the decode
step of Algorithm 3, greedy and sampled."""
import itertools
import os

import numpy as np
import pytest
from scipy import stats

from workloads import configs, pda as P, vocab as V
from workloads.logits import f32_to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")
F32, BF16 = 0, 1


def _token_run(oracle, pda, edges, seq, stack=(P.S0,)):
    """Runs a token sequence through the token edges as Algorithm 3 does; None if some token has no matching edge."""
    q, st = pda.start, list(stack)
    by = {}
    for e in edges.as_set():
        by.setdefault((e[0], e[1]), []).append(e)
    for t in seq:
        hits = [e for e in by.get((q, t), []) if len(e[2]) <= len(st) and tuple(st[len(st) - len(e[2]):]) == e[2]]
        assert len(hits) <= 1, "two token edges match one configuration"
        if not hits:
            return None
        _, _, pops, q, pushes = hits[0]
        del st[len(st) - len(pops):]
        st += list(pushes)
    return q, tuple(st)


def _compile(oracle, pda, toks):
    vocab = V.from_tokens(toks)
    return oracle.pda_compile(pda, vocab.data, vocab.offsets), vocab


def test_fig7_token_edges(oracle):
    want = set()
    for ln in open(os.path.join(GOLD, "fig7_anbn_token_edges.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        s, t, pops, d, pushes = ln.split()
        f = lambda x: () if x == "-" else tuple(int(v) for v in x.split(","))
        want.add((int(s), int(t), f(pops), int(d), f(pushes)))
    edges, _ = _compile(oracle, P.anbn(), [b"a", b"b", b"bb", b"aaab"])
    assert edges.as_set() == want
    # the caption's point: one token edge crosses a non-terminal boundary and pops / pushes several symbols
    assert (2, 2, (1, 1), 2, ()) in want and (0, 3, (), 2, (1, 1)) in want


def test_fig7_sequences(oracle):
    pda = P.anbn()
    edges, _ = _compile(oracle, pda, [b"a", b"b", b"bb", b"aaab"])
    acc = lambda cfg: cfg is not None and oracle.pda_accepting(pda, pda.accept, cfg[0], cfg[1])
    assert acc(_token_run(oracle, pda, edges, [3, 2]))                 # aaab bb
    assert acc(_token_run(oracle, pda, edges, [0, 0, 0, 1, 1, 1]))     # a a a b b b
    assert acc(_token_run(oracle, pda, edges, [0, 0, 2]))              # a a bb: the token crosses S's boundary
    half = _token_run(oracle, pda, edges, [3, 1])                      # aaab b: viable, not complete
    assert half is not None and not acc(half)
    assert _token_run(oracle, pda, edges, [3, 2, 1]) is None           # one b too many
    assert _token_run(oracle, pda, edges, [1]) is None


# ---- the character automata against recognisers written without automata

def _is_anbn(s: bytes) -> bool:
    n = len(s) // 2
    return n >= 1 and s == b"a" * n + b"b" * n


def _is_dyck(s: bytes) -> bool:
    st = []
    for ch in s:
        if ch in b"([":
            st.append(ch)
        elif not st or st.pop() != {41: 40, 93: 91}[ch]:
            return False
    return not st


def _is_int_list(s: bytes) -> bool:
    pos = 0

    def value():
        nonlocal pos
        if pos < len(s) and s[pos:pos + 1].isdigit():
            while pos < len(s) and s[pos:pos + 1].isdigit():
                pos += 1
            return True
        if s[pos:pos + 1] != b"[":
            return False
        pos += 1
        if s[pos:pos + 1] == b"]":
            pos += 1
            return True
        while True:
            if not value():
                return False
            if s[pos:pos + 1] == b",":
                pos += 1
                continue
            if s[pos:pos + 1] == b"]":
                pos += 1
                return True
            return False

    return value() and pos == len(s)


CASES = [
    (P.anbn, b"ab", 8, _is_anbn),
    (P.dyck2, b"()[]", 6, _is_dyck),
    (P.int_lists, b"1[],", 7, _is_int_list),
]


@pytest.mark.parametrize("make,alphabet,max_len,member", CASES)
def test_char_automata_match_recognisers(oracle, make, alphabet, max_len, member):
    """The inputs themselves: every string up to max_len is accepted by the character automaton iff the
    hand-written recogniser says so (acceptance after the closing epsilon edges)."""
    pda = make()
    assert oracle.pda_check_deterministic(pda) == 0
    n_acc = 0
    for n in range(max_len + 1):
        for tup in itertools.product(alphabet, repeat=n):
            s = bytes(tup)
            cfg = P.run_chars(pda, s)
            got = cfg is not None and oracle.pda_accepting(pda, pda.accept, cfg[0], cfg[1])
            assert got == member(s), s
            n_acc += got
    assert n_acc >= 3


def test_json_like_automaton_against_json_module(oracle):
    """The JSON-like input automaton accepts exactly what Python's json module parses, on generated documents
    and on one-character mutations of them (documents inside the automaton's subset: no white space, no
    escapes, no fractions, top level an array or an object)."""
    import json
    import random
    pda = P.json_like()
    assert oracle.pda_check_deterministic(pda) == 0
    rnd = random.Random(1)

    def gen(depth=0):
        r = rnd.random()
        if depth > 3 or r < 0.3:
            return rnd.choice([0, 7, -12, 105, True, False, None, "ab c", "x_1", ""])
        if r < 0.65:
            return [gen(depth + 1) for _ in range(rnd.randint(0, 3))]
        return {rnd.choice(["k", "key_2", "a b", ""]) + str(i): gen(depth + 1) for i in range(rnd.randint(0, 3))}

    n_ok = n_bad = 0
    for _ in range(3000):
        v = gen()
        if not isinstance(v, (list, dict)):
            v = [v]
        s = json.dumps(v, separators=(",", ":"))
        if rnd.random() < 0.5:
            k = rnd.randrange(len(s) + 1)
            s = s[:k] + rnd.choice('[]{},:"0a') + s[k + (rnd.random() < 0.5):]
        if not s or s[0] not in "[{":
            continue
        try:
            doc = json.loads(s)
            want = True
        except ValueError:
            want = False
        if want:                                         # a mutation inside a string may leave the automaton's string alphabet
            strings, todo = [], [doc]
            while todo:
                x = todo.pop()
                if isinstance(x, str):
                    strings.append(x)
                elif isinstance(x, list):
                    todo += x
                elif isinstance(x, dict):
                    strings += list(x.keys())
                    todo += list(x.values())
            if any(ch not in "abcdefghijklmnopqrstuvwxyz0123456789_ " for st in strings for ch in st):
                continue
        cfg = P.run_chars(pda, s.encode())
        got = cfg is not None and oracle.pda_accepting(pda, pda.accept, cfg[0], cfg[1])
        assert got == want, s
        n_ok += want
        n_bad += not want
    assert n_ok > 500 and n_bad > 500


VOCABS = {
    "anbn": [b"a", b"b", b"bb", b"aaab", b"ab", b"aab", b"abb", b"ba"],
    "dyck2": [b"(", b")", b"[", b"]", b"()", b"[]", b"((", b"))", b")]", b"](", b"([)]", b"[()]", b"])"],
    "int_lists": [b"1", b"7", b"[", b"]", b",", b"12", b"[[", b"]]", b"],[", b"1,2", b",[", b"[]", b"3]", b"[4,", b"]],"],
}


@pytest.mark.parametrize("name,make,max_seq", [("anbn", P.anbn, 5), ("dyck2", P.dyck2, 4), ("int_lists", P.int_lists, 4)])
def test_theorem3_bruteforce(oracle, name, make, max_seq):
    """P_{G o V}(x) = P_G(D(x)) for every token sequence x up to max_seq tokens: the run over token edges ends in
    the same state with the same stack as the character automaton on the concatenated text, dies exactly
    when it dies, and accepts exactly the texts of the language."""
    pda = make()
    toks = VOCABS[name]
    edges, _ = _compile(oracle, pda, toks)
    member = {"anbn": _is_anbn, "dyck2": _is_dyck, "int_lists": _is_int_list}[name]
    alive = accepted = 0
    for n in range(max_seq + 1):
        for seq in itertools.product(range(len(toks)), repeat=n):
            text = b"".join(toks[t] for t in seq)
            tok_cfg = _token_run(oracle, pda, edges, seq)
            chr_cfg = P.run_chars(pda, text)
            assert (tok_cfg is None) == (chr_cfg is None), (seq, text)
            if tok_cfg is None:
                continue
            alive += 1
            # the character run has taken the epsilon edges before each byte but none after the last, as the
            # token edges do: same state, same stack
            assert tok_cfg == chr_cfg, (seq, text, tok_cfg, chr_cfg)
            got = oracle.pda_accepting(pda, pda.accept, tok_cfg[0], tok_cfg[1])
            assert got == member(text), (seq, text)
            accepted += got
    assert alive > 20 and accepted > 3


def test_appendixA_call_grammar(oracle):
    """Appendix A.2: tokens may cross the terminals of the grammar (such as r(4); all four tokenizations of
    the two calls are accepted, pieces in the wrong order are not."""
    pda = P.call_grammar()
    lines = [ln.split() for ln in open(os.path.join(GOLD, "appendixA_tokenizations.txt")) if ln.strip() and not ln.startswith("#")]
    pieces = sorted({p for ln in lines for p in ln})
    toks = [p.encode() for p in pieces]
    edges, _ = _compile(oracle, pda, toks)
    for ln in lines:
        seq = [pieces.index(p) for p in ln]
        cfg = _token_run(oracle, pda, edges, seq)
        assert cfg is not None and oracle.pda_accepting(pda, pda.accept, cfg[0], cfg[1]), ln
        assert _token_run(oracle, pda, edges, seq[::-1]) is None                 # the pieces in the wrong order
    assert any(b"(" in t and len(t) > 1 for t in toks)


def test_stack_edit_algebra(oracle):
    """Concatenation of stack edits, by hand: x pops (A B) pushes (C); y pops (D C) pushes (E F); z pops (F)."""
    A, B, Cc, D, E, Fs, G = 1, 2, 3, 4, 5, 6, 7
    pda = P.make_pda(5, 0, [3], [(0, "x", (A, B), 1, (Cc,)), (1, "y", (D, Cc), 2, (E, Fs)), (2, "z", (Fs,), 3, ()),
                                 (1, "w", (G,), 4, ())])
    edges, _ = _compile(oracle, pda, [b"x", b"xy", b"xyz", b"yz", b"xw", b"y"])
    got = edges.as_set()
    assert (0, 0, (A, B), 1, (Cc,)) in got
    assert (0, 1, (D, A, B), 2, (E, Fs)) in got              # y reaches below what x pushed: D lies under A B
    assert (0, 2, (D, A, B), 3, (E,)) in got                 # z pops what y pushed last
    assert (1, 3, (D, Cc), 3, (E,)) in got
    assert (1, 5, (D, Cc), 2, (E, Fs)) in got
    assert not any(e[0] == 0 and e[1] == 4 for e in got)     # w needs G on top, x has just pushed C
    assert len(got) == 5


def test_regular_special_case(oracle):
    """An automaton that never touches its stack: the token edges are the entries of delta_T (tdfa_oracle.c)."""
    w = configs.get("c1")
    d = w.dfas[0]
    pda = P.dfa_as_pda(d.trans, d.accept, d.start)
    edges = oracle.pda_compile(pda, w.vocab.data, w.vocab.offsets)
    table = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets)
    want = {(int(q), int(t), (), int(table[q, t]), ()) for q, t in zip(*np.nonzero(table >= 0))}
    assert edges.as_set() == want


def test_nondeterminism_is_reported(oracle):
    """Section 3.1: a non-deterministic automaton is an error, not something to resolve."""
    bad = P.make_pda(3, 0, [2], [(0, P.EPS, (), 1, ()), (0, "a", (), 2, ())])            # epsilon or a: both possible
    assert oracle.pda_check_deterministic(bad) == 1
    bad2 = P.make_pda(3, 0, [2], [(0, "a", (1,), 1, ()), (0, "a", (2, 1), 2, ())])       # (1) is a suffix of (2 1)
    assert oracle.pda_check_deterministic(bad2) == 1
    ok = P.make_pda(3, 0, [2], [(0, "a", (1,), 1, ()), (0, "a", (2,), 2, ()), (0, "b", (), 2, ())])
    assert oracle.pda_check_deterministic(ok) == 0
    v = V.from_tokens([b"a"])
    with pytest.raises(RuntimeError) as e:
        oracle.pda_compile(bad, v.data, v.offsets)
    assert "-3" in str(e.value)
    loop = P.make_pda(2, 0, [1], [(0, P.EPS, (0,), 0, (0,))])                            # an endless run of epsilon edges
    assert oracle.pda_check_deterministic(loop) == 0
    with pytest.raises(RuntimeError) as e:
        oracle.pda_compile(loop, v.data, v.offsets)
    assert "-5" in str(e.value)


# ---- decode step (Algorithm 3, loop body)

def _step(oracle, pda, edges, n_tokens, logits, dtype, states, stacks, depths, **kw):
    return oracle.pda_step(pda.n_states, n_tokens, edges, logits, dtype, states, stacks, depths, **kw)


def _sorted_edges(oracle, edges):
    order = np.argsort(edges.src, kind="stable")
    return oracle.TokenEdges(*[getattr(edges, k)[order] for k in ("src", "token", "dst", "n_pops", "pops", "n_push", "pushes")])


def test_step_closed_forms(oracle):
    pda = P.anbn()
    toks = [b"a", b"b", b"bb", b"aaab"]
    edges, _ = _compile(oracle, pda, toks)
    edges = _sorted_edges(oracle, edges)
    cap = 8
    R = 1
    cfgs = [(0, [0]), (1, [0]), (1, [0, R]), (2, [0, R]), (2, [0, R, R]), (2, [0]), (4, [0]), (-1, [0]), (7, [0]), (1, [0] + [R] * 7)]
    B = len(cfgs)
    states = np.array([c[0] for c in cfgs], dtype=np.int32)

    def fresh():
        st = np.full((B, cap), -7, dtype=np.int32)
        dp = np.zeros(B, dtype=np.int32)
        for i, (_, s) in enumerate(cfgs):
            st[i, :len(s)] = s
            dp[i] = len(s)
        return st, dp

    # allowed sets by hand: state 0: a, aaab; state 1 with (S): a, b, aaab; with (S R): + bb; state 2 with one R: b;
    # with two: b, bb; with none, or in the accepting state: nothing
    up = np.tile(np.arange(4, dtype=np.float32), (B, 1))
    st, dp = fresh()
    tok, new, masked = _step(oracle, pda, edges, 4, up, F32, states, st, dp, want_masked=True)
    # largest allowed id; the last row's stack is full, the chosen token would push three more: the sequence ends
    assert tok.tolist() == [3, 3, 3, 1, 2, -1, -1, -1, -1, -1]
    assert new.tolist() == [2, 2, 2, 2, 2, 2, 4, -1, -1, -1]
    assert dp.tolist() == [3, 4, 5, 1, 1, 1, 1, 1, 1, 8]
    assert st[0, :3].tolist() == [0, R, R] and st[2, :5].tolist() == [0, R, R, R, R]
    assert np.isneginf(masked[5]).all() and np.isneginf(masked[7]).all()
    assert np.array_equal(masked[1], np.array([0, 1, -np.inf, 3], dtype=np.float32))
    flat = np.zeros((B, 4), dtype=np.float32)
    st, dp = fresh()
    tok, new = _step(oracle, pda, edges, 4, flat, F32, states, st, dp)
    assert tok.tolist() == [0, 0, 0, 1, 1, -1, -1, -1, -1, -1]           # lowest id among equals
    assert new[9] == -1 and dp[9] == 8                                   # a would push a ninth symbol: no room, the sequence ends
    nan = np.full((B, 4), np.nan, dtype=np.float32)
    st, dp = fresh()
    tok, _ = _step(oracle, pda, edges, 4, nan, F32, states, st, dp)
    assert tok.tolist()[:5] == [0, 0, 0, 1, 1]
    bits = f32_to_bf16_bits(up)
    st, dp = fresh()
    tok2, new2, m2 = _step(oracle, pda, edges, 4, bits, BF16, states, st, dp, want_masked=True)
    assert tok2.tolist() == [3, 3, 3, 1, 2, -1, -1, -1, -1, -1] and m2[1, 2] == 0xFF80 and m2[1, 3] == bits[1, 3]


@pytest.mark.parametrize("name,make", [("dyck2", P.dyck2), ("int_lists", P.int_lists)])
def test_decode_stays_in_the_language(oracle, name, make):
    """Chained steps with random logits: whatever has been generated is what the character automaton accepts as a
    prefix (same state, same stack), and a sequence that has no token left is in an accepting configuration."""
    pda = make()
    toks = VOCABS[name]
    edges, _ = _compile(oracle, pda, toks)
    edges = _sorted_edges(oracle, edges)
    rng = np.random.default_rng(5)
    B, cap, steps = 16, 6, 24
    states = np.full(B, pda.start, dtype=np.int32)
    stacks = np.full((B, cap), -7, dtype=np.int32)
    stacks[:, 0] = P.S0
    depths = np.ones(B, dtype=np.int32)
    texts = [b""] * B
    live = np.ones(B, dtype=bool)
    for s in range(steps):
        lg = rng.normal(0, 2, size=(B, len(toks))).astype(np.float32)
        tok, states = _step(oracle, pda, edges, len(toks), lg, F32, states, stacks, depths)
        for b in range(B):
            if not live[b]:
                assert tok[b] == -1
                continue
            if tok[b] < 0:
                live[b] = False
                if states[b] >= 0:       # nothing allowed: only the end of a complete text (or a full stack) may cause that
                    assert oracle.pda_accepting(pda, pda.accept, int(states[b]), stacks[b, :depths[b]]) or depths[b] >= cap - 1
                continue
            texts[b] += toks[tok[b]]
            cfg = P.run_chars(pda, texts[b])
            assert cfg is not None and cfg == (int(states[b]), tuple(stacks[b, :depths[b]].tolist())), (texts[b], cfg)
    assert sum(len(t) > 4 for t in texts) > B // 2


def _anbn_config(state, stack, B, cap=8):
    st = np.full((B, cap), -7, dtype=np.int32)
    st[:, :len(stack)] = stack
    return np.full(B, state, dtype=np.int32), st, np.full(B, len(stack), dtype=np.int32)


@pytest.mark.parametrize("dtype,temperature", [(F32, 1.0), (F32, 0.5), (BF16, 2.0)])
def test_sampled_step_draws_from_the_softmax_over_the_allowed_set(oracle, dtype, temperature):
    """Figs. 6-7: in state 1 with one R on the stack the allowed tokens are a, b, bb, aaab; in state 2 with two R
    they are b and bb (the sets derived by hand in test_step_closed_forms).  Chi-square of 20,000 draws against
    softmax(l / T) over exactly those sets, and the drawn token's edge is the one that is traversed."""
    pda = P.anbn()
    toks = [b"a", b"b", b"bb", b"aaab"]
    edges, _ = _compile(oracle, pda, toks)
    edges = _sorted_edges(oracle, edges)
    R = 1
    l = np.array([0.3, -0.4, 1.1, 0.2], dtype=np.float32)
    bits = l if dtype == F32 else f32_to_bf16_bits(l)
    lv = l if dtype == F32 else (bits.astype(np.uint32) << 16).view(np.float32)
    B, n_off = 500, 40
    # (state, depth) after each token, by hand from the automaton: in state 1 `a` pushes an R; `b` leads to state 2,
    # where the pop of an R belongs to the b that follows it; so bb ends one R lower, aaab three R higher
    for state, stack, allowed, after in ((1, [0, R], [0, 1, 2, 3], {0: (1, 3), 1: (2, 2), 2: (2, 1), 3: (2, 5)}),
                                         (2, [0, R, R], [1, 2], {1: (2, 2), 2: (2, 1)})):
        counts = np.zeros(4, dtype=np.int64)
        for off in range(n_off):
            states, st, dp = _anbn_config(state, stack, B)
            tok, new = oracle.pda_sample_step(pda.n_states, 4, edges, np.tile(bits, (B, 1)), dtype, states, st, dp, temperature, 7, off)
            counts += np.bincount(tok, minlength=4)
            for t, want in after.items():
                assert (new[tok == t] == want[0]).all() and (dp[tok == t] == want[1]).all(), (state, t)
        assert counts.sum() == B * n_off and counts[[t for t in range(4) if t not in allowed]].sum() == 0
        p = np.exp(lv[allowed].astype(np.float64) / temperature)
        p /= p.sum()
        assert stats.chisquare(counts[allowed], p * counts.sum()).pvalue > 1e-3, (state, counts, p * counts.sum())
        if temperature != 1.0:                            # T in place of 1/T, or no temperature at all, is rejected
            for wrong in (1.0, 1.0 / temperature):
                pw = np.exp(lv[allowed].astype(np.float64) / wrong)
                pw /= pw.sum()
                assert stats.chisquare(counts[allowed], pw * counts.sum()).pvalue < 1e-6


def test_sampled_step_limits(oracle):
    """A very low temperature, and top_k = 1, give the greedy step of Algorithm 3 (tokens, states, stacks); the
    same seed and offset give the same draw, another offset another; the penalised row shows the constraint."""
    pda = P.dyck2()
    toks = VOCABS["dyck2"]
    edges, _ = _compile(oracle, pda, toks)
    edges = _sorted_edges(oracle, edges)
    rng = np.random.default_rng(3)
    B, cap = 64, 6
    lg = rng.normal(0, 2, size=(B, len(toks))).astype(np.float32)

    def fresh():
        st = np.full((B, cap), -7, dtype=np.int32)
        st[:, 0] = P.S0
        return np.full(B, pda.start, dtype=np.int32), st, np.ones(B, dtype=np.int32)

    s0, st0, dp0 = fresh()
    g_tok, g_new, g_masked = oracle.pda_step(pda.n_states, len(toks), edges, lg, F32, s0, st0, dp0, want_masked=True)
    for kw in (dict(temperature=1e-4), dict(temperature=1.0, top_k=1)):
        s1, st1, dp1 = fresh()
        tok, new, masked = oracle.pda_sample_step(pda.n_states, len(toks), edges, lg, F32, s1, st1, dp1, seed=5, offset=0,
                                                  want_masked=True, **kw)
        assert np.array_equal(tok, g_tok) and np.array_equal(new, g_new) and np.array_equal(dp1, dp0)
        assert np.array_equal(st1, st0) and np.array_equal(masked.view(np.uint32), g_masked.view(np.uint32))
    draws = []
    for off in (0, 0, 1):
        s1, st1, dp1 = fresh()
        draws.append(oracle.pda_sample_step(pda.n_states, len(toks), edges, lg, F32, s1, st1, dp1, 1.0, 5, off)[0])
    assert np.array_equal(draws[0], draws[1]) and not np.array_equal(draws[0], draws[2])
    assert (draws[0] != g_tok).any()                      # at temperature 1 the draw is not the argmax everywhere
