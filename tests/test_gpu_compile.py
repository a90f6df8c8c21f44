"""GPU parity of the compile stage against the oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

from workloads import configs, vocab as V
from workloads.regex_dfa import compile_regex, random_dfa
import gpu_util as G
import invariants as inv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import paper_2407_08103_amd as T
    assert torch.cuda.is_available()
    return T


def _compile(T, dfa, vocab):
    v = T.Vocab(vocab.data, vocab.offsets)
    d = T.CharDFA(dfa.trans, dfa.accept, dfa.start)
    table = T.compile_token_dfa(v, d)
    torch.cuda.synchronize()
    return table, v, d


def _full_check(T, oracle, dfa, vocab, compose_rows=None, threads=8):
    table, v, d = _compile(T, dfa, vocab)
    walk = oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, n_threads=threads)
    G.check_rows(table, walk, np.arange(dfa.n_states))
    if compose_rows is None:
        comp = oracle.compile_compose(dfa.trans, vocab.data, vocab.offsets, n_threads=threads)
        assert np.array_equal(comp, walk)
    else:
        lo, hi = compose_rows
        comp = oracle.compile_compose(dfa.trans, vocab.data, vocab.offsets, q_lo=lo, q_hi=hi, n_threads=threads)
        G.check_rows(table, comp, np.arange(lo, hi))
    return table, walk


def test_fig4_example(T, oracle):
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table, _ = _full_check(T, oracle, d, vocab)
    want = np.array([[1, -1, 3, -1, 4], [-1, 3, -1, -1, -1], [-1] * 5, [1, -1, 3, -1, 4], [-1] * 5], dtype=np.int32)
    assert np.array_equal(table.delta.cpu().numpy(), want)


@pytest.mark.parametrize("seed", range(6))
def test_small_seeded(T, oracle, seed):
    """Several token tiles with a ragged tail, several state groups."""
    w = configs.small(seed, n_tokens=300 + 97 * seed)
    _full_check(T, oracle, w.dfas[0], w.vocab)


@pytest.mark.parametrize("n_states,n_tokens", [(1, 1), (63, 255), (64, 256), (65, 257), (129, 513), (300, 1000)])
def test_random_dfa_shapes(T, oracle, n_states, n_tokens):
    """Tile-boundary shapes on a dense random automaton (long live walks)."""
    rng = np.random.default_rng(n_states * 1000 + n_tokens)
    dfa = random_dfa(n_states, 0.3, 0.2, rng)
    ls, ps = V.zipf_lengths(1, 9, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    _full_check(T, oracle, dfa, vocab)


def test_empty_duplicate_and_long_tokens(T, oracle):
    d = compile_regex(r"(ab)*c|x{0,300}y")
    toks = [b"ab", b"", b"ab", b"c", b"", b"x" * 299 + b"y", b"x" * 301, b"abc", b"x" * 150]
    table, walk = _full_check(T, oracle, d, V.from_tokens(toks))
    assert (walk[:, 1] == -1).all() and np.array_equal(walk[:, 0], walk[:, 2])
    assert walk[0, 5] >= 0 and (walk[:, 6] == -1).all()


def test_wide_states_int32_path(T, oracle):
    """More than 32767 states: the table is kept in 32-bit form on the device."""
    rng = np.random.default_rng(5)
    dfa = random_dfa(33000, 0.6, 0.1, rng)
    ls, ps = V.zipf_lengths(1, 6, 1.0)
    vocab = V.make_vocab(rng, 700, np.zeros(0, np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    table, _, _ = _compile(T, dfa, vocab)
    rows = np.concatenate([np.arange(0, 130), np.arange(32700, 33000)])
    want = np.concatenate([oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, q_lo=0, q_hi=130),
                           oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, q_lo=32700, q_hi=33000)])
    G.check_rows(table, want, rows)
    assert int(table.delta.max()) > 32767


@pytest.mark.parametrize("n_states", [32703, 32704, 32767, 32768])
def test_state_width_boundary(T, oracle, n_states):
    """Around the largest automaton whose states still fit the 16-bit device table."""
    rng = np.random.default_rng(n_states)
    dfa = random_dfa(n_states, 0.5, 0.1, rng)
    dfa.trans[n_states - 1, :8] = n_states - 1        # the highest state id is a live target
    dfa.trans[0, :4] = n_states - 1
    ls, ps = V.zipf_lengths(1, 5, 1.0)
    vocab = V.make_vocab(rng, 300, np.arange(8, dtype=np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    table, _, _ = _compile(T, dfa, vocab)
    rows = np.concatenate([np.arange(0, 70), np.arange(n_states - 200, n_states)])
    want = np.concatenate([oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, q_lo=0, q_hi=70),
                           oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, q_lo=n_states - 200, q_hi=n_states)])
    G.check_rows(table, want, rows)
    assert int(table.delta.max()) == n_states - 1


def test_c1_full(T, oracle):
    w = configs.get("c1")
    _full_check(T, oracle, w.dfas[0], w.vocab)


def test_c2_full(T, oracle):
    w = configs.get("c2")
    table, walk = _full_check(T, oracle, w.dfas[0], w.vocab, compose_rows=(0, 64))
    d = w.dfas[0]
    assert inv.check_singletons(walk, d.trans, w.vocab) == 256
    inv.check_liveness(walk, d.accept, d.start)


def test_c3_full_size(T, oracle):
    """Full 128,256-token table: every row against the closed form in chunks, sampled rows against
    the composition oracle."""
    w = configs.get("c3")
    d = w.dfas[0]
    table, v, dd = _compile(T, d, w.vocab)
    assert table.delta.shape == (d.n_states, 128256)
    step = 512
    for lo in range(0, d.n_states, step):
        hi = min(d.n_states, lo + step)
        want = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, q_lo=lo, q_hi=hi, n_threads=16)
        G.check_rows(table, want, np.arange(lo, hi))
    rng = np.random.default_rng(3)
    for q in sorted(rng.choice(d.n_states, size=12, replace=False).tolist()) + [0, d.n_states - 1]:
        want = oracle.compile_compose(d.trans, w.vocab.data, w.vocab.offsets, q_lo=q, q_hi=q + 1)
        G.check_rows(table, want, [q])


def test_c4_full_size(T, oracle):
    """256,000 tokens x 20,000 states (20 GB): the whole table against the closed form, in blocks of
    rows; sampled rows against the composition oracle; the properties that hold at any size
    (singletons, live fraction)."""
    w = configs.get("c4")
    d = w.dfas[0]
    table, v, dd = _compile(T, d, w.vocab)
    assert table.delta.shape == (20000, 256000)
    step = 1000
    live = 0
    for lo in range(0, d.n_states, step):
        hi = min(d.n_states, lo + step)
        want = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, q_lo=lo, q_hi=hi, n_threads=16)
        G.check_rows(table, want, np.arange(lo, hi))
        live += int((want >= 0).sum())
        del want
    rng = np.random.default_rng(4)
    for q in [0, 127, 128, 19999] + sorted(rng.choice(20000, size=4, replace=False).tolist()):
        comp = oracle.compile_compose(d.trans, w.vocab.data, w.vocab.offsets, q_lo=int(q), q_hi=int(q) + 1)
        G.check_rows(table, comp, [int(q)])
    lens = np.diff(w.vocab.offsets.astype(np.int64))
    single = np.nonzero(lens == 1)[0]
    bs = w.vocab.data[w.vocab.offsets[single].astype(np.int64)]
    got = table.delta[:, torch.as_tensor(single, device="cuda")].cpu().numpy()
    assert np.array_equal(got, d.trans[:, bs])
    expect = float(np.mean(0.3 ** lens))
    assert abs(live / (20000 * 256000) - expect) < 0.002


def test_compile_twice_same_bytes(T, oracle):
    """Determinism: two compiles of the same constraint into different buffers give the same bytes
    (tables and allowed bits), also when the second runs while the device is busy with other work."""
    w = configs.get("c2")
    d = w.dfas[0]
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    h = T.CharDFA(d.trans, d.accept, d.start)
    a = T.compile_token_dfa(v, h)
    junk = torch.randn(4096, 4096, device="cuda")
    junk = junk @ junk
    b = T.compile_token_dfa(v, h)
    torch.cuda.synchronize()
    assert torch.equal(a.delta, b.delta) and torch.equal(a.allow, b.allow)
    h2 = T.CharDFA(d.trans, d.accept, d.start)                      # a second upload of the same automaton
    c = T.compile_token_dfa(v, h2)
    torch.cuda.synchronize()
    assert torch.equal(a.delta, c.delta) and torch.equal(a.allow, c.allow)


def test_concat_c5_subset(T, oracle):
    """Three of the multi-constraint tables stacked with row offsets."""
    w = configs.get("c5")
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    tabs, want = [], []
    for i in (0, 7, 33):
        d = w.dfas[i]
        tabs.append(T.compile_token_dfa(v, T.CharDFA(d.trans, d.accept, d.start)))
        want.append(oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=16))
    big, offs = T.table_concat(tabs)
    torch.cuda.synchronize()
    ref, ref_offs = oracle.concat_tables(want)
    assert np.array_equal(offs, ref_offs)
    G.check_rows(big, ref, np.arange(ref.shape[0]))
    # the same rows from one batched call, and from one call per constraint into its slice
    handles = [T.CharDFA(w.dfas[i].trans, w.dfas[i].accept, w.dfas[i].start) for i in (0, 7, 33)]
    stacked, offs2 = T.compile_stacked(v, handles)
    torch.cuda.synchronize()
    assert np.array_equal(offs2, ref_offs)
    G.check_rows(stacked, ref, np.arange(ref.shape[0]))
    delta = torch.full_like(stacked.delta, -7)
    allow = torch.zeros_like(stacked.allow)
    for c, h in enumerate(handles):
        lo, hi = int(ref_offs[c]), int(ref_offs[c + 1])
        T.compile_token_dfa(v, h, out=(delta[lo:hi], allow[lo:hi]), row_base=lo)
    torch.cuda.synchronize()
    G.check_rows(T.table_wrap(delta, allow), ref, np.arange(ref.shape[0]))


def test_union_equals_stacked(T, oracle):
    """The disjoint union of the automata, compiled as one automaton, is the stacked table."""
    w = configs.get("c5")
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    pick = (0, 7, 33, 7, 12)
    handles = [T.CharDFA(w.dfas[i].trans, w.dfas[i].accept, w.dfas[i].start) for i in pick]
    union, offs = T.dfa_union(handles)
    table = T.compile_token_dfa(v, union)
    torch.cuda.synchronize()
    want = [oracle.compile_walk(w.dfas[i].trans, w.vocab.data, w.vocab.offsets, n_threads=16) for i in pick]
    ref, ref_offs = oracle.concat_tables(want)
    assert np.array_equal(offs, ref_offs) and union.n_states == ref.shape[0]
    G.check_rows(table, ref, np.arange(ref.shape[0]))
    # and with small random automata, a vocabulary whose row length is odd
    rng = np.random.default_rng(21)
    ls, ps = V.zipf_lengths(1, 5, 1.0)
    vocab = V.make_vocab(rng, 301, np.arange(16, dtype=np.uint8), ls, ps, np.arange(64, dtype=np.uint8), 1.0, None)
    dfas = [random_dfa(n, 0.5, 0.2, rng) for n in (3, 70, 129, 1)]
    union, offs = T.dfa_union([T.CharDFA(d.trans, d.accept, d.start) for d in dfas])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), union)
    torch.cuda.synchronize()
    ref, ref_offs = oracle.concat_tables([oracle.compile_walk(d.trans, vocab.data, vocab.offsets) for d in dfas])
    assert np.array_equal(offs, ref_offs)
    G.check_rows(table, ref, np.arange(ref.shape[0]))


def test_union_from_host_automata(T, oracle):
    """tdfa_dfa_union_host: the union made without uploading each automaton first compiles to the same stacked
    table; missing accept arrays and a bad entry (named by its place in the union) are handled."""
    rng = np.random.default_rng(22)
    ls, ps = V.zipf_lengths(1, 5, 1.0)
    vocab = V.make_vocab(rng, 301, np.arange(16, dtype=np.uint8), ls, ps, np.arange(64, dtype=np.uint8), 1.0, None)
    dfas = [random_dfa(n, 0.5, 0.2, rng) for n in (3, 70, 2500, 1, 129)]
    union, offs = T.dfa_union_host([(d.trans, d.accept if i % 2 == 0 else None, d.start) for i, d in enumerate(dfas)])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), union)
    torch.cuda.synchronize()
    ref, ref_offs = oracle.concat_tables([oracle.compile_walk(d.trans, vocab.data, vocab.offsets) for d in dfas])
    assert np.array_equal(offs, ref_offs) and union.n_states == ref.shape[0] and union.start == dfas[0].start
    G.check_rows(table, ref, np.arange(ref.shape[0]))
    bad = dfas[1].trans.copy()
    bad[5, 9] = 70                                                     # one past its own automaton's last state
    with pytest.raises(T.TdfaError) as e:
        T.dfa_union_host([(dfas[0].trans, None, 0), (bad, None, 0)])
    assert e.value.code == -1 and "trans[8][9]" in str(e.value)


def test_stacked_mixed_widths(T, oracle):
    """A batch that mixes 16-bit and 32-bit device tables and more automata than one launch holds."""
    rng = np.random.default_rng(11)
    ls, ps = V.zipf_lengths(1, 5, 1.0)
    vocab = V.make_vocab(rng, 200, np.arange(16, dtype=np.uint8), ls, ps, np.arange(64, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    sizes = [3, 70, 33000, 5, 129] + [2 + i for i in range(50)]
    dfas = [random_dfa(n, 0.5, 0.2, rng) for n in sizes]
    stacked, offs = T.compile_stacked(v, [T.CharDFA(d.trans, d.accept, d.start) for d in dfas])
    torch.cuda.synchronize()
    for c, d in enumerate(dfas):
        if d.n_states > 1000:
            rows = np.concatenate([np.arange(0, 64), np.arange(d.n_states - 64, d.n_states)])
        else:
            rows = np.arange(d.n_states)
        want = np.concatenate([oracle.compile_walk(d.trans, vocab.data, vocab.offsets, q_lo=int(q), q_hi=int(q) + 1)
                               for q in rows])
        want = np.where(want >= 0, want + offs[c], -1).astype(np.int32)
        G.check_rows(stacked, want, rows + offs[c])


def test_bad_arguments(T):
    with pytest.raises(T.TdfaError) as e:
        T.CharDFA(np.full((2, 256), 7, dtype=np.int32), None, 0)
    assert e.value.code == -1 and "outside" in str(e.value)
    with pytest.raises(T.TdfaError):
        T.CharDFA(np.full((2, 256), -1, dtype=np.int32), None, 2)
    with pytest.raises(T.TdfaError):
        T.Vocab(np.zeros(4, np.uint8), np.array([0, 3, 2], dtype=np.uint64))


# ---- automata with counter-like classes: the jump tables and start bytes of the compile kernel

def _counter_vocab(rng, alphabet: bytes, n_random: int, extra: list[bytes]):
    """Distinct tokens over `alphabet` with lengths 1..40 (beyond the 32 bytes a jump covers),
    plus hand-made ones; ids shuffled."""
    toks = set(extra)
    alpha = np.frombuffer(alphabet, dtype=np.uint8)
    while len(toks) < n_random + len(extra):
        n = int(rng.integers(1, 41))
        toks.add(bytes(alpha[rng.integers(0, len(alpha), size=n)]))
    toks = sorted(toks)
    rng.shuffle(toks)
    return V.from_tokens(toks)


@pytest.mark.parametrize("pattern,alphabet,n_random", [
    (r'"[^"\\]{0,40}"', b'ab"\\ z', 1000),                      # one class, chain ends in a literal state
    (r'"[^"\\]{0,40}"', b'ab"\\ z', 1001),                      # a row length that is not a multiple of 4
    (r'[a-c_][a-c0-2_]{0,45}=[0-2]{1,40};', b'abc_012=;x', 1500),   # two classes with large complements
    (r'[ab]{70}[bc]{70}d', b'abcd', 900),                       # a chain that leaves its class: partly valid
    (r'([ab]{26}[cd]{26}[ef]{26}[gh]{26}[ij]{26}[kl]{26}[mn]{26}[op]{26}[qr]{26}[st]{26})?u', b'abcdefghijklmnopqrstu', 1200),  # more classes than are kept
    (r'(x[a-d]*y|z[0-9]{0,30})+', b'xyzabcd0123456789', 800),    # an unbounded loop state as a class
])
def test_counter_classes(T, oracle, pattern, alphabet, n_random):
    dfa = compile_regex(pattern)
    rng = np.random.default_rng(len(pattern) * 7919 + n_random)
    a0 = alphabet[:1]
    extra = [b"", a0 * 31, a0 * 32, a0 * 33, a0 * 64, a0 * 100, alphabet[-1:] + a0 * 35, a0 * 20 + alphabet[-1:] + a0 * 20,
             alphabet[1:2] * 32 + alphabet[:1], alphabet[1:2] * 31 + alphabet[-1:]]
    vocab = _counter_vocab(rng, alphabet, n_random, extra)
    assert len(vocab.offsets) - 1 == n_random + len(extra)
    _full_check(T, oracle, dfa, vocab, compose_rows=(0, min(dfa.n_states, 40)))


def test_counter_classes_stacked_with_plain(T, oracle):
    """One launch that holds automata with and without jump classes, and a repeated handle."""
    rng = np.random.default_rng(77)
    alphabet = b'ab"\\ z01'
    vocab = _counter_vocab(rng, alphabet, 700, [b"", b"a" * 40, b'"' + b"b" * 33 + b'"'])
    v = T.Vocab(vocab.data, vocab.offsets)
    dfas = [compile_regex(r'"[^"\\]{0,40}"'), random_dfa(90, 0.5, 0.2, rng), compile_regex(r'[ab]{70}[01]{30}z'),
            random_dfa(3, 0.2, 0.5, rng)]
    handles = [T.CharDFA(d.trans, d.accept, d.start) for d in dfas]
    order = [0, 1, 2, 0, 3]
    stacked, offs = T.compile_stacked(v, [handles[i] for i in order])
    torch.cuda.synchronize()
    for c, i in enumerate(order):
        d = dfas[i]
        want = oracle.compile_walk(d.trans, vocab.data, vocab.offsets, n_threads=8)
        want = np.where(want >= 0, want + offs[c], -1).astype(np.int32)
        G.check_rows(stacked, want, np.arange(d.n_states) + offs[c])


def test_without_start_byte_workspace(T, oracle):
    """An automaton whose start-byte workspace would exceed its limit is compiled without it
    (forced here by lowering the limit): same table."""
    dfa = compile_regex(r'"[^"\\]{0,40}"(,[0-9]{1,30})*')
    rng = np.random.default_rng(5)
    vocab = _counter_vocab(rng, b'ab"\\,019', 600, [b"", b"a" * 40])
    v = T.Vocab(vocab.data, vocab.offsets)
    walk = oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, n_threads=8)
    for limit in (1000, None):
        d = T.CharDFA(dfa.trans, dfa.accept, dfa.start)
        if limit is not None:
            d.workspace_limit(limit)
        table = T.compile_token_dfa(v, d)
        torch.cuda.synchronize()
        G.check_rows(table, walk, np.arange(dfa.n_states))


# ---- the two-byte-prefix pair lists (TDFA_PATH_PAIRS), forced on automata of every small shape

def _pairs_check(T, oracle, dfa, vocab, threads=8):
    v = T.Vocab(vocab.data, vocab.offsets)
    walk = oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, n_threads=threads)
    for path in (T.PATH_PAIRS, T.PATH_WALK):
        d = T.CharDFA(dfa.trans, dfa.accept, dfa.start)
        d.compile_path(path)
        table = T.compile_token_dfa(v, d)
        torch.cuda.synchronize()
        G.check_rows(table, walk, np.arange(dfa.n_states))
    return walk


@pytest.mark.parametrize("n_states,n_tokens,p_live", [(1, 1, 0.5), (5, 3, 0.9), (255, 255, 0.3), (256, 256, 0.3), (257, 257, 0.3),
                                                      (700, 1027, 0.3), (513, 2048, 0.6), (1500, 777, 0.1), (300, 1000, 1.0)])
def test_pairs_random_shapes(T, oracle, n_states, n_tokens, p_live):
    """Dense and sparse random automata, state counts around the 256-state tile, vocabulary sizes
    around the 64- and 256-token blocks, row lengths that are and are not multiples of 4."""
    rng = np.random.default_rng(n_states * 7 + n_tokens)
    dfa = random_dfa(n_states, 1.0 - p_live, 0.2, rng)
    ls, ps = V.zipf_lengths(1, 9, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256 if n_tokens > 300 else 8, dtype=np.uint8), 1.0, None)
    _pairs_check(T, oracle, dfa, vocab)


def test_pairs_token_lengths(T, oracle):
    """Empty, one-byte, two-byte, duplicate and long tokens (beyond the 32 bytes kept per token)."""
    rng = np.random.default_rng(12)
    dfa = random_dfa(400, 0.02, 0.3, rng)                          # nearly complete: long walks stay alive
    dfa.trans[:, 4:] = -1                                          # over the bytes 0..3 only
    toks = [b"", b"\x00", b"\x01\x02", b"\x01\x02", b"\x03" * 31, b"\x03" * 32, b"\x03" * 33, b"\x02" * 64, b"\x01" * 100,
            b"\x00\x01\x02", b"", b"\x09", b"\x01\x09", b"\x01\x02\x09", b"\x01" * 40 + b"\x09"]
    alpha = np.arange(4, dtype=np.uint8)
    for n in range(1, 60):
        toks.append(bytes(alpha[rng.integers(0, 4, size=n)]))
    walk = _pairs_check(T, oracle, dfa, V.from_tokens(toks))
    assert (walk[:, 0] == -1).all() and (walk[:, 8] >= 0).any() and (walk[:, 11] == -1).all()


# ---- the walk with the automaton's table staged in LDS (TDFA_PATH_STAGED)

@pytest.mark.parametrize("n_states,n_tokens,p_live", [(1, 1, 0.5), (5, 3, 0.9), (63, 700, 0.5), (64, 1027, 0.4), (127, 4100, 0.3),
                                                      (191, 2048, 0.6), (150, 40000, 0.2)])
def test_staged_random_shapes(T, oracle, n_states, n_tokens, p_live):
    """Automata small enough for their whole table to sit in LDS beside the tile, up to the largest
    that does (191 states), against the oracle and against the walk that reads the table from memory."""
    rng = np.random.default_rng(n_states * 11 + n_tokens)
    dfa = random_dfa(n_states, 1.0 - p_live, 0.2, rng)
    ls, ps = V.zipf_lengths(1, 9, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256 if n_tokens > 300 else 8, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    walk = oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, n_threads=8)
    d = T.CharDFA(dfa.trans, dfa.accept, dfa.start)
    d.compile_path(T.PATH_STAGED)
    assert d.info()[2] == T.PATH_STAGED
    table = T.compile_token_dfa(v, d)
    torch.cuda.synchronize()
    G.check_rows(table, walk, np.arange(dfa.n_states))


def test_staged_workloads_and_limit(T, oracle):
    """c1 (a counter-like class: jump tables beside the staged table), a stacked table that mixes staged and
    unstaged automata, and an automaton one state too large, which takes the walk."""
    w = configs.get("c1")
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    d = T.CharDFA(w.dfas[0].trans, w.dfas[0].accept, w.dfas[0].start)
    d.compile_path(T.PATH_STAGED)
    table = T.compile_token_dfa(v, d)
    torch.cuda.synchronize()
    G.check_rows(table, oracle.compile_walk(w.dfas[0].trans, w.vocab.data, w.vocab.offsets), np.arange(w.dfas[0].n_states))
    rng = np.random.default_rng(5)
    ls, ps = V.zipf_lengths(1, 6, 1.0)
    vocab = V.make_vocab(rng, 900, np.arange(16, dtype=np.uint8), ls, ps, np.arange(32, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    dfas = [random_dfa(n, 0.5, 0.2, rng) for n in (100, 40, 300, 7)]
    handles = [T.CharDFA(x.trans, x.accept, x.start) for x in dfas]
    for h in handles[:3]:
        h.compile_path(T.PATH_STAGED)
    assert [h.info()[2] for h in handles] == [T.PATH_STAGED, T.PATH_STAGED, T.PATH_WALK, T.PATH_WALK]
    stacked, offs = T.compile_stacked(v, handles)
    torch.cuda.synchronize()
    ref, ref_offs = oracle.concat_tables([oracle.compile_walk(x.trans, vocab.data, vocab.offsets) for x in dfas])
    assert np.array_equal(offs, ref_offs)
    G.check_rows(stacked, ref, np.arange(ref.shape[0]))
    big = random_dfa(192, 0.5, 0.2, rng)
    h = T.CharDFA(big.trans, big.accept, big.start)
    h.compile_path(T.PATH_STAGED)
    assert h.info()[2] == T.PATH_WALK


def test_workspace_blocks_are_reused(T, oracle):
    """Automata that take the sweep one after the other: the large workspace arrays of a destroyed automaton
    go to the next one (of another size, too), the tables stay right, and tdfa_trim gives them back."""
    rng = np.random.default_rng(77)
    ls, ps = V.zipf_lengths(1, 7, 1.0)
    vocab = V.make_vocab(rng, 3000, np.zeros(0, np.uint8), ls, ps, np.arange(64, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    for n_states in (600, 600, 350, 900, 600):
        dfa = random_dfa(n_states, 0.6, 0.2, rng)
        d = T.CharDFA(dfa.trans, dfa.accept, dfa.start)
        d.compile_path(T.PATH_PAIRS)
        for _ in range(2):                                              # the first call sizes, the second finds all in place
            table = T.compile_token_dfa(v, d)
            torch.cuda.synchronize()
            G.check_rows(table, oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets, n_threads=8), np.arange(n_states))
        del d, table
    T.trim()
    T.trim()


def test_pairs_in_a_stacked_table(T, oracle):
    """Automata compiled through the pair lists inside a stacked table, next to automata compiled by
    the walk, and one written straight into its slice with a row offset."""
    rng = np.random.default_rng(31)
    ls, ps = V.zipf_lengths(1, 6, 1.0)
    vocab = V.make_vocab(rng, 900, np.arange(16, dtype=np.uint8), ls, ps, np.arange(32, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    dfas = [random_dfa(n, 0.5, 0.2, rng) for n in (300, 40, 513, 7)]
    handles = [T.CharDFA(d.trans, d.accept, d.start) for d in dfas]
    handles[0].compile_path(T.PATH_PAIRS)
    handles[2].compile_path(T.PATH_PAIRS)
    stacked, offs = T.compile_stacked(v, handles)
    torch.cuda.synchronize()
    ref, ref_offs = oracle.concat_tables([oracle.compile_walk(d.trans, vocab.data, vocab.offsets) for d in dfas])
    assert np.array_equal(offs, ref_offs)
    G.check_rows(stacked, ref, np.arange(ref.shape[0]))
    delta = torch.full_like(stacked.delta, -7)
    allow = torch.zeros_like(stacked.allow)
    for c, h in enumerate(handles):
        lo, hi = int(ref_offs[c]), int(ref_offs[c + 1])
        T.compile_token_dfa(v, h, out=(delta[lo:hi], allow[lo:hi]), row_base=lo)
    torch.cuda.synchronize()
    G.check_rows(T.table_wrap(delta, allow), ref, np.arange(ref.shape[0]))


def test_pairs_on_regex_automata(T, oracle):
    """The same path on structured automata (c2's JSON-like constraint; counter classes make the
    library fall back to the walk, which must give the same table)."""
    w = configs.get("c2")
    _pairs_check(T, oracle, w.dfas[0], w.vocab)
    d = compile_regex(r"(foo)+d")
    _pairs_check(T, oracle, d, V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"]))


def test_automata_created_compiled_and_destroyed_back_to_back(T, oracle):
    """A destroyed automaton's device memory is handed to the next one, but only once the compile call that used it
    has run: twelve automata of one size and different content, each created, compiled into a table of its own
    and destroyed without waiting for the GPU, on two streams in turn; every table must be its own automaton's."""
    rng = np.random.default_rng(123)
    n_states, n_tokens = 700, 6000
    ls, ps = V.zipf_lengths(1, 6, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    v = T.Vocab(vocab.data, vocab.offsets)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dfas, tables = [], []
    for i in range(12):
        d = random_dfa(n_states, 0.9, 0.2, rng)
        dfas.append(d)
        with torch.cuda.stream(streams[i % 2]):
            h = T.CharDFA(d.trans, d.accept, d.start)
            tables.append(T.compile_token_dfa(v, h))
            del h                                        # destroyed while its compile may still be queued or running
    torch.cuda.synchronize()
    for d, t in zip(dfas, tables):
        G.check_rows(t, oracle.compile_walk(d.trans, vocab.data, vocab.offsets), np.arange(n_states))
    T.trim()
