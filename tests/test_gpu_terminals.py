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


def test_bad_arguments(T, oracle):
    d, edges = dfa_with_terminals(b"a\xff+b", {0xFF: 0})
    vocab = V.from_tokens([b"a", b"b", b"x"])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), T.CharDFA(d.trans, d.accept, d.start))
    masks = _mask_rows(T, np.ones((1, 3), dtype=np.uint8))
    for bad in ([(99, 0, 0)], [(0, 1, 0)], [(0, 0, -1)]):
        with pytest.raises(T.TdfaError):
            T.table_apply_terminals(table, bad, masks)
    T.table_apply_terminals(table, np.zeros((0, 3), np.int32), masks)          # no edges: nothing to do
