"""GPU parity of the token-level optimisation against the oracle, bit for bit (new table, allowed
bits, state map, final states), and decode steps on the optimised table."""
import numpy as np
import pytest
import torch

from workloads import configs, logits as LG, vocab as V
from workloads.regex_dfa import compile_regex
import gpu_util as G

pytestmark = pytest.mark.gpu
DEAD = -1
BF16 = 1


@pytest.fixture(scope="module")
def T():
    import paper_2407_08103_amd as T
    assert torch.cuda.is_available()
    return T


def _upload_table(T, table_np):
    delta = torch.from_numpy(np.ascontiguousarray(table_np)).cuda()
    rw = T.allow_row_words(table_np.shape[1])
    allow = torch.from_numpy(G.bits_from_table(table_np, rw).view(np.int32)).cuda()
    return T.table_wrap(delta, allow)


def _as_torch(T, table):
    """A library-owned table copied into torch buffers (one-table concat = plain copy)."""
    out, _ = T.table_concat([table])
    torch.cuda.synchronize()
    return out


def _check(T, oracle, table, table_np, accept, starts):
    new, acc, mp = T.table_minimize(table, accept, starts)
    want, want_acc, want_mp = oracle.minimize(table_np, accept, starts)
    assert np.array_equal(mp, want_mp)
    assert new.n_rows == want.shape[0] and np.array_equal(acc, want_acc)
    if new.n_rows:
        G.check_rows(_as_torch(T, new), want, np.arange(want.shape[0]))
    return new, want, mp


def test_fig4_example(T, oracle):
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), T.CharDFA(d.trans, d.accept, d.start))
    table_np = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    new, want, mp = _check(T, oracle, table, table_np, d.accept, [d.start])
    assert mp.tolist() == [0, 1, DEAD, 0, 2] and want.tolist() == [[1, -1, 0, -1, 2], [-1, 0, -1, -1, -1], [-1] * 5]


@pytest.mark.parametrize("seed", range(6))
def test_random_tables(T, oracle, seed):
    rng = np.random.default_rng(100 + seed)
    n, v = int(rng.integers(2, 200)), int(rng.integers(1, 700))
    table_np = rng.integers(0, n, size=(n, v), dtype=np.int32)
    table_np[rng.random((n, v)) < (0.5 + 0.08 * seed)] = DEAD
    # classes to merge: blocks of states that share their row and their flag
    for q in range(n // 2, n):
        table_np[q] = table_np[q % max(1, n // 4)]
    accept = (rng.random(n) < 0.3).astype(np.uint8)
    for q in range(n // 2, n):
        accept[q] = accept[q % max(1, n // 4)]
    starts = rng.integers(0, n, size=int(rng.integers(1, 4))).astype(np.int32)
    _check(T, oracle, _upload_table(T, table_np), table_np, accept, starts)


def _most_targets(table_np):
    return max(len(np.unique(r[r >= 0])) for r in table_np)


def test_long_chains_merge(T, oracle):
    """Two copies of a counter of 300 states: the copies merge state by state, one refinement round
    per state of the chain (the rounds run on the rows' lists of distinct targets)."""
    L, v = 300, 50
    n = 2 * L + 1
    table_np = np.full((n, v), DEAD, dtype=np.int32)
    table_np[0, 0], table_np[0, 1] = 1, L + 1
    for half in (0, L):
        for i in range(1, L + 1):
            q = half + i
            nxt = q + 1 if i < L else q
            table_np[q, i % v] = nxt
            table_np[q, (3 * i + 7) % v] = nxt if i % 5 else q
    accept = np.zeros(n, np.uint8)
    accept[L], accept[2 * L] = 1, 1
    assert _most_targets(table_np) <= 3072
    new, want, mp = _check(T, oracle, _upload_table(T, table_np), table_np, accept, [0])
    assert new.n_rows == L + 1 and np.array_equal(mp[1:L + 1], mp[L + 1:])


def test_rows_with_many_distinct_targets(T, oracle):
    """A table whose rows have more distinct targets than the list-building pass keeps per row:
    the call streams the dense rows instead, with the same result."""
    rng = np.random.default_rng(77)
    n, v = 5000, 12000
    table_np = rng.integers(0, n, size=(n, v), dtype=np.int32)
    table_np[rng.random((n, v)) < 0.3] = DEAD
    for q in range(n - 40, n):                       # a few classes to merge
        table_np[q] = table_np[q - 40]
    accept = (rng.random(n) < 0.3).astype(np.uint8)
    accept[n - 40:] = accept[n - 80:n - 40]
    assert _most_targets(table_np) > 3072
    _check(T, oracle, _upload_table(T, table_np), table_np, accept, [0, 17])


def test_lists_longer_than_first_guessed(T, oracle):
    """Rows with about 700 distinct targets each: more list entries in all than the first pass makes room for, so
    the lists are built a second time at their true size."""
    rng = np.random.default_rng(31)
    n, v = 2500, 1200
    table_np = rng.integers(0, n, size=(n, v), dtype=np.int32)
    table_np[rng.random((n, v)) < 0.3] = DEAD
    for q in range(n - 30, n):
        table_np[q] = table_np[q - 30]
    accept = (rng.random(n) < 0.3).astype(np.uint8)
    accept[n - 30:] = accept[n - 60:n - 30]
    per_row = [len(np.unique(r[r >= 0])) for r in table_np]
    assert max(per_row) <= 3072 and sum(per_row) > max(1 << 20, n * 512)
    _check(T, oracle, _upload_table(T, table_np), table_np, accept, [0])


def test_nothing_left(T, oracle):
    table_np = np.array([[1, -1], [0, 1]], dtype=np.int32)
    new, want, mp = _check(T, oracle, _upload_table(T, table_np), table_np, np.zeros(2, np.uint8), [0])
    assert new.n_rows == 0 and mp.tolist() == [DEAD, DEAD]


def test_c2_and_decode(T, oracle):
    w = configs.get("c2")
    d = w.dfas[0]
    table_np = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=8)
    table = T.compile_token_dfa(T.Vocab(w.vocab.data, w.vocab.offsets), T.CharDFA(d.trans, d.accept, d.start))
    new, want, mp = _check(T, oracle, table, table_np, d.accept, [d.start])
    assert 0 < new.n_rows <= d.n_states
    # the same greedy decode on both tables: same tokens, states related by the map
    B, steps, Vn = 32, 40, table_np.shape[1]
    st_a = torch.full((B,), d.start, dtype=torch.int32, device="cuda")
    st_b = torch.full((B,), int(mp[d.start]), dtype=torch.int32, device="cuda")
    tok_a = torch.empty(B, dtype=torch.int32, device="cuda")
    tok_b = torch.empty(B, dtype=torch.int32, device="cuda")
    mp_dev = torch.from_numpy(mp).cuda()
    for s in range(steps):
        lg = torch.from_numpy(LG.gen_logits(configs.logits_seed(2), s, B, Vn, 2.0, "bf16").view(np.int16)).cuda().view(torch.bfloat16)
        T.mask_step(table, lg, st_a, tok_a, st_a)
        T.mask_step(new, lg, st_b, tok_b, st_b)
        torch.cuda.synchronize()
        assert torch.equal(tok_a, tok_b)
        assert torch.equal(mp_dev[st_a.long()], st_b)


def test_stacked_with_several_starts(T, oracle):
    w = configs.get("c5")
    pick = (3, 9, 3)
    vocab = V.from_tokens([bytes(w.vocab.token(t)) for t in range(0, w.vocab.n_tokens, 97)])
    tabs = [oracle.compile_walk(w.dfas[i].trans, vocab.data, vocab.offsets) for i in pick]
    ref, offs = oracle.concat_tables(tabs)
    accept = np.concatenate([w.dfas[i].accept for i in pick]).astype(np.uint8)
    starts = [int(offs[c]) + w.dfas[i].start for c, i in enumerate(pick)]
    _check(T, oracle, _upload_table(T, ref), ref, accept, starts)


def test_bad_arguments(T):
    table = _upload_table(T, np.zeros((2, 3), dtype=np.int32))
    with pytest.raises(T.TdfaError):
        T.table_minimize(table, np.zeros(2, np.uint8), [5])
    with pytest.raises(ValueError):
        T.table_minimize(table, np.zeros(3, np.uint8), [0])
