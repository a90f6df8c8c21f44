"""GPU parity of terminal labels (Section 2.5.1) against the oracle, bit for bit: the table and its
allowed bits after tdfa_table_apply_terminals, and decode steps on the result."""
import numpy as np
import pytest
import torch

from workloads import configs, logits as LG, vocab as V
from workloads.regex_dfa import random_dfa
from terminals_util import dfa_with_terminals
import gpu_util as G

pytestmark = pytest.mark.gpu
DEAD = -1
BF16 = 1


@pytest.fixture(scope="module")
def T():
    import paper_2407_08103_amd as T
    assert torch.cuda.is_available()
    return T


def _mask_rows(T, masks_np):
    """Bit rows (the layout of the allowed bits) from one byte per token."""
    n_labels, n_tokens = masks_np.shape
    rw = T.allow_row_words(n_tokens)
    live = np.zeros((n_labels, rw * 32), dtype=np.uint8)
    live[:, :n_tokens] = masks_np != 0
    words = np.packbits(live, axis=1, bitorder="little").view(np.uint32).reshape(n_labels, rw)
    return torch.from_numpy(words.view(np.int32)).cuda()


def _check(T, oracle, dfa, vocab, edges, masks_np):
    v = T.Vocab(vocab.data, vocab.offsets)
    table = T.compile_token_dfa(v, T.CharDFA(dfa.trans, dfa.accept, dfa.start))
    T.table_apply_terminals(table, edges, _mask_rows(T, masks_np))
    torch.cuda.synchronize()
    want = oracle.apply_terminals(oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets), edges, masks_np)
    G.check_rows(table, want, np.arange(dfa.n_states))
    return table, want


def test_bulleted_list(T, oracle):
    d, edges = dfa_with_terminals(b"S:(\n\\* \xff+){1,2}", {0xFF: 0})
    toks = [b"S:", b"S", b":", b"\n", b"* ", b"\n* ", b"a", b"bc", b"d\ne", b"*", b" "]
    mask = np.array([[0 if b"\n" in t else 1 for t in toks]], dtype=np.uint8)
    _check(T, oracle, d, V.from_tokens(toks), edges, mask)


@pytest.mark.parametrize("n_states,n_tokens,n_labels,n_edges", [(5, 33, 1, 3), (70, 257, 3, 40), (300, 1000, 8, 500),
                                                                (40, 4097, 2, 25)])
def test_random(T, oracle, n_states, n_tokens, n_labels, n_edges):
    """Random automata, masks and edge lists: several edges per state with overlapping masks, row
    lengths that are not multiples of 32 or 256, states without edges."""
    rng = np.random.default_rng(n_states + n_tokens)
    dfa = random_dfa(n_states, 0.85, 0.2, rng)
    ls, ps = V.zipf_lengths(1, 4, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    edges = np.stack([rng.integers(0, n_states, n_edges), rng.integers(0, n_labels, n_edges),
                      rng.integers(0, n_states, n_edges)], axis=1).astype(np.int32)
    masks = (rng.random((n_labels, n_tokens)) < 0.3).astype(np.uint8)
    table, want = _check(T, oracle, dfa, vocab, edges, masks)
    assert (want >= 0).sum() > (oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets) >= 0).sum()
    # decode steps on the table with terminal edges
    B = 64
    states = rng.integers(0, n_states, B).astype(np.int32)
    lg_np = LG.gen_logits(configs.logits_seed(1), 3, B, n_tokens + (-n_tokens) % 8, 2.0, "bf16")
    lg = torch.from_numpy(lg_np.view(np.int16)).cuda().view(torch.bfloat16)
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    new = torch.empty(B, dtype=torch.int32, device="cuda")
    out = torch.empty_like(lg)
    T.mask_step(table, lg, torch.from_numpy(states).cuda(), tok, new, out)
    torch.cuda.synchronize()
    res = oracle.mask_step(want, lg_np, BF16, states, want_masked=True)
    assert np.array_equal(tok.cpu().numpy(), res[0]) and np.array_equal(new.cpu().numpy(), res[1])
    assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16)[:, :n_tokens], res[2][:, :n_tokens])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("batch", [5, 300])
def test_states_that_allow_nothing_before_and_after(T, oracle, dtype, batch):
    """A compiled table knows how many tokens each state allows, and a step is done early with a sequence whose
    state allows none.  Terminal edges out of such a state must undo that: the same step, before and after
    tdfa_table_apply_terminals, without the penalised rows (small batch: rows split over workgroups)."""
    rng = np.random.default_rng(batch)
    n_states, n_tokens = 40, 9000
    dfa = random_dfa(n_states, 0.85, 0.2, rng)
    dfa.trans[::3] = DEAD                                   # every third state allows no byte, so no token
    ls, ps = V.zipf_lengths(1, 4, 1.0)
    vocab = V.make_vocab(rng, n_tokens, np.zeros(0, np.uint8), ls, ps, np.arange(256, dtype=np.uint8), 1.0, None)
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), T.CharDFA(dfa.trans, dfa.accept, dfa.start))
    want = oracle.compile_walk(dfa.trans, vocab.data, vocab.offsets)
    assert (want[::3] == DEAD).all() and (want >= 0).any()
    states = rng.integers(0, n_states, batch).astype(np.int32)
    states[:3] = [0, 3, -1]
    lg_np = LG.gen_logits(configs.logits_seed(1), 5, batch, n_tokens, 2.0, dtype)
    lg = (torch.from_numpy(lg_np.view(np.int16)).cuda().view(torch.bfloat16) if dtype == "bf16" else torch.from_numpy(lg_np).cuda())
    code = BF16 if dtype == "bf16" else 0

    def step_and_check(ref):
        tok = torch.full((batch,), -9, dtype=torch.int32, device="cuda")
        new = torch.full((batch,), -9, dtype=torch.int32, device="cuda")
        T.mask_step(table, lg, torch.from_numpy(states).cuda(), tok, new)
        torch.cuda.synchronize()
        res = oracle.mask_step(ref, lg_np, code, states)
        assert np.array_equal(tok.cpu().numpy(), res[0]) and np.array_equal(new.cpu().numpy(), res[1])
        return res[0]

    first = step_and_check(want)
    assert (first[states % 3 == 0] == -1).all() and (first >= 0).any()
    edges = np.array([[q, 0, (q + 1) % n_states] for q in range(0, n_states, 6)], dtype=np.int32)
    masks = (rng.random((1, n_tokens)) < 0.01).astype(np.uint8)
    T.table_apply_terminals(table, edges, _mask_rows(T, masks))
    after = step_and_check(oracle.apply_terminals(want, edges, masks))
    assert (after[states % 6 == 0] >= 0).all() and (after[states % 6 == 3] == -1).all()


def test_bad_arguments(T, oracle):
    d, edges = dfa_with_terminals(b"a\xff+b", {0xFF: 0})
    vocab = V.from_tokens([b"a", b"b", b"x"])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), T.CharDFA(d.trans, d.accept, d.start))
    masks = _mask_rows(T, np.ones((1, 3), dtype=np.uint8))
    for bad in ([(99, 0, 0)], [(0, 1, 0)], [(0, 0, -1)]):
        with pytest.raises(T.TdfaError):
            T.table_apply_terminals(table, bad, masks)
    T.table_apply_terminals(table, np.zeros((0, 3), np.int32), masks)          # no edges: nothing to do
