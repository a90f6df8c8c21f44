"""GPU parity of the edge-list (packed) form of a table against the oracle's, array by array, and
of the decode calls on a packed table against the oracle's results on the dense one."""
import numpy as np
import pytest
import torch

from workloads import configs, logits as LG, vocab as V
from workloads.regex_dfa import compile_regex
import gpu_util as G

pytestmark = pytest.mark.gpu
DEAD = -1
F32, BF16 = 0, 1


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


def _check_pack(T, oracle, table, table_np):
    packed = T.table_pack(table)
    assert packed.delta_ptr is None or packed.delta_ptr == 0
    assert (packed.n_rows, packed.n_tokens, packed.row_words) == (table.n_rows, table.n_tokens, table.row_words)
    targets, row_begin, dirs, allow = (x.cpu().numpy() for x in T.table_pack_arrays(packed))
    want_begin, want_targets = oracle.compact(table_np)
    assert np.array_equal(row_begin, want_begin)
    assert np.array_equal(targets, want_targets)
    # the library's per-row directory (edges of the row below each block of 128 tokens), counted naively
    n_tokens = table_np.shape[1]
    n_blocks = (n_tokens + 127) // 128
    live = np.zeros((table_np.shape[0], n_blocks * 128), dtype=np.int64)
    live[:, :n_tokens] = table_np >= 0
    per_block = live.reshape(table_np.shape[0], n_blocks, 128).sum(2)
    want_dir = (np.cumsum(per_block, axis=1) - per_block).astype(np.uint32)
    assert dirs.shape[1] == table.row_words // 4 >= n_blocks
    assert np.array_equal(dirs.view(np.uint32)[:, :n_blocks], want_dir)
    # blocks beyond the vocabulary (row padding) start after all of the row's edges
    assert (dirs.view(np.uint32)[:, n_blocks:] == np.diff(want_begin)[:, None]).all()
    assert np.array_equal(allow.view(np.uint32), G.bits_from_table(table_np, table.row_words))
    return packed


def test_fig4_example(T, oracle):
    d = compile_regex(r"(foo)+d")
    vocab = V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])
    table = T.compile_token_dfa(T.Vocab(vocab.data, vocab.offsets), T.CharDFA(d.trans, d.accept, d.start))
    torch.cuda.synchronize()
    table_np = oracle.compile_walk(d.trans, vocab.data, vocab.offsets)
    packed = _check_pack(T, oracle, table, table_np)
    targets, row_begin, _, _ = T.table_pack_arrays(packed)
    assert row_begin.tolist() == [0, 3, 4, 4, 7, 7] and targets.tolist() == [1, 3, 4, 3, 1, 3, 4]


@pytest.mark.parametrize("n_rows,n_tokens,p_live", [(1, 1, 1.0), (7, 127, 0.5), (9, 128, 0.02), (6, 129, 0.9),
                                                    (300, 1000, 0.3), (4, 5000, 0.0), (3, 640, 1.0),
                                                    (40, 40000, 0.01), (5, 128256, 0.85)])
def test_random_tables(T, oracle, n_rows, n_tokens, p_live):
    rng = np.random.default_rng(n_rows * 1000 + n_tokens)
    tab = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
    tab[rng.random((n_rows, n_tokens)) >= p_live] = DEAD
    if n_rows > 2:
        tab[1] = DEAD                                        # a state without edges between others
    table = _upload_table(T, tab)
    packed = _check_pack(T, oracle, table, tab)
    # every decode call gives on the packed table what the oracle gives on the dense one
    B = 37
    states = rng.integers(-1, n_rows + 1, size=B).astype(np.int32)
    stride = (n_tokens + 7) // 8 * 8
    x = np.zeros((B, stride), dtype=np.float32)
    x[:, :n_tokens] = rng.normal(0, 2, size=(B, n_tokens))
    for dtype in (F32, BF16):
        lg_np = x if dtype == F32 else LG.f32_to_bf16_bits(x)
        lg = torch.from_numpy(lg_np).cuda() if dtype == F32 else torch.from_numpy(lg_np.view(np.int16)).cuda().view(torch.bfloat16)
        st = torch.from_numpy(states).cuda()
        tok = torch.full((B,), -9, dtype=torch.int32, device="cuda")
        new = torch.full((B,), -9, dtype=torch.int32, device="cuda")
        T.mask_step(packed, lg, st, tok, new)
        torch.cuda.synchronize()
        want_tok, want_new, want_masked = oracle.mask_step(tab, lg_np, dtype, states, row_stride=stride, want_masked=True)
        assert np.array_equal(tok.cpu().numpy(), want_tok) and np.array_equal(new.cpu().numpy(), want_new)
        out = torch.full_like(lg, 7.0)
        tok.fill_(-9)
        T.mask_step(packed, lg, st, tok, new, out)               # the same with the masked row written
        torch.cuda.synchronize()
        assert np.array_equal(tok.cpu().numpy(), want_tok) and np.array_equal(new.cpu().numpy(), want_new)
        got = out.cpu().numpy().view(np.uint32) if dtype == F32 else out.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got[:, :n_tokens], want_masked.view(got.dtype)[:, :n_tokens])
        assert (out[:, n_tokens:].float() == 7.0).all()
        T.sample_step(packed, lg, st, 0.9, 5, 3, tok, new)
        torch.cuda.synchronize()
        want_tok, want_new = oracle.sample_step(tab, lg_np, dtype, states, 0.9, 5, 3, row_stride=stride, n_threads=16)
        assert np.array_equal(tok.cpu().numpy(), want_tok) and np.array_equal(new.cpu().numpy(), want_new)
    k = 6
    runs = rng.integers(-1, n_tokens + 1, size=(B, k)).astype(np.int32)
    live_rows = np.nonzero((tab >= 0).any(1))[0]
    if len(live_rows):                                       # some runs that do follow edges
        for b in range(0, B, 2):
            s = int(live_rows[b % len(live_rows)])
            states[b] = s
            for i in range(k):
                nz = np.nonzero(tab[s] >= 0)[0] if s >= 0 else []
                if len(nz) == 0:
                    break
                runs[b, i] = nz[(b + i) % len(nz)]
                s = int(tab[s, runs[b, i]])
    hist = torch.empty((B, k + 1), dtype=torch.int32, device="cuda")
    nv = torch.empty((B,), dtype=torch.int32, device="cuda")
    T.advance_tokens(packed, torch.from_numpy(states).cuda(), torch.from_numpy(runs).cuda(), hist, nv)
    torch.cuda.synchronize()
    want_hist, want_nv = oracle.advance_tokens(tab, states, runs)
    assert np.array_equal(hist.cpu().numpy(), want_hist) and np.array_equal(nv.cpu().numpy(), want_nv)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_special_values_on_packed(T, oracle, dtype):
    """NaN, infinities, ties and signed zeros through the scan that packed tables use: a sparse
    state (gathered groups) and a wildcard-like one (streamed) side by side."""
    n_tokens = 4096 + 64
    rng = np.random.default_rng(9)
    tab = rng.integers(0, 4, size=(4, n_tokens), dtype=np.int32)
    tab[0, rng.random(n_tokens) > 0.01] = DEAD
    tab[1, rng.random(n_tokens) > 0.6] = DEAD
    tab[2] = DEAD
    tab[3, rng.random(n_tokens) > 0.12] = DEAD                 # close to the switch between the two scans
    packed = T.table_pack(_upload_table(T, tab))
    states = np.array([0, 1, 2, 3, 0, 1, 3], dtype=np.int32)
    B = len(states)
    cases = [np.full((B, n_tokens), 1.25, np.float32),
             np.tile(np.arange(n_tokens, dtype=np.float32) / 64.0 - 20, (B, 1)),
             np.tile(-np.arange(n_tokens, dtype=np.float32) / 64.0, (B, 1))]
    x = rng.normal(0, 2, size=(B, n_tokens)).astype(np.float32)
    x[:, rng.integers(0, n_tokens, 200)] = np.nan
    x[:, rng.integers(0, n_tokens, 50)] = np.inf
    x[:, rng.integers(0, n_tokens, 50)] = -np.inf
    cases.append(x)
    y = np.full((B, n_tokens), -np.inf, np.float32)
    y[:, rng.integers(0, n_tokens, 500)] = np.nan
    cases.append(y)
    cases.append(np.round(rng.normal(0, 2, size=(B, n_tokens))).astype(np.float32))
    cases.append(np.where(rng.random((B, n_tokens)) < 0.5, -0.0, 0.0).astype(np.float32))
    for x in cases:
        lg_np = x if dtype == F32 else LG.f32_to_bf16_bits(x)
        lg = torch.from_numpy(lg_np).cuda() if dtype == F32 else torch.from_numpy(lg_np.view(np.int16)).cuda().view(torch.bfloat16)
        tok = torch.full((B,), -9, dtype=torch.int32, device="cuda")
        new = torch.full((B,), -9, dtype=torch.int32, device="cuda")
        T.mask_step(packed, lg, torch.from_numpy(states).cuda(), tok, new)
        torch.cuda.synchronize()
        want_tok, want_new = oracle.mask_step(tab, lg_np, dtype, states)
        assert np.array_equal(tok.cpu().numpy(), want_tok) and np.array_equal(new.cpu().numpy(), want_new)


def test_errors(T, oracle):
    tab = np.array([[0, DEAD, 1], [DEAD, DEAD, 0]], dtype=np.int32)
    table = _upload_table(T, tab)
    packed = T.table_pack(table)
    with pytest.raises(T.TdfaError):
        T.table_pack(packed)
    with pytest.raises(T.TdfaError):
        T.table_concat([packed])
    with pytest.raises(T.TdfaError):
        T.table_minimize(packed, [1, 0], [0])
    with pytest.raises(T.TdfaError):
        T.table_pack_arrays(table)


def test_c3_full_size(T, oracle):
    """The API-call union at full size: 584 M dense entries become a few million edges; the arrays
    against the oracle's, then 64 chained decode steps on the packed table against the dense one."""
    w = configs.get("c3")
    d = w.dfas[0]
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    table = T.compile_token_dfa(v, T.CharDFA(d.trans, d.accept, d.start))
    torch.cuda.synchronize()
    tab = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=16)
    packed = _check_pack(T, oracle, table, tab)
    m = w.mask
    B, Vn, S = m.batch, w.vocab.n_tokens, 64
    hs = [torch.empty((S + 1, B), dtype=torch.int32, device="cuda") for _ in range(2)]
    ht = [torch.empty((S, B), dtype=torch.int32, device="cuda") for _ in range(2)]
    logits = torch.empty((B, Vn), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for h in hs:
        h[0] = d.start
    for s in range(S):
        LG.gen_logits_device(logits.data_ptr(), configs.logits_seed(3), s, B, Vn, Vn, m.sigma, m.dtype, stream)
        for i, tb in enumerate((table, packed)):
            T.mask_step(tb, logits, hs[i][s], ht[i][s], hs[i][s + 1])
    torch.cuda.synchronize()
    assert torch.equal(hs[0], hs[1]) and torch.equal(ht[0], ht[1])
    assert len(torch.unique(hs[0])) > 50
