"""GPU parity of the sampling step against the oracle: the noise bit for bit, then tokens, states
and masked rows of single steps and of chained decodes."""
import numpy as np
import pytest
import torch

from workloads import configs, logits as LG
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
    delta = torch.from_numpy(table_np).cuda()
    rw = T.allow_row_words(table_np.shape[1])
    allow = torch.from_numpy(G.bits_from_table(table_np, rw).view(np.int32)).cuda()
    return T.table_wrap(delta, allow)


def _to_dev(lg_np, dtype):
    if dtype == F32:
        return torch.from_numpy(lg_np).cuda()
    return torch.from_numpy(lg_np.view(np.int16)).cuda().view(torch.bfloat16)


def _bits(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _rand_table(n_rows, n_tokens, p_live, seed):
    rng = np.random.default_rng(seed)
    t = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
    t[rng.random((n_rows, n_tokens)) > p_live] = DEAD
    return t


def _step_and_check(T, oracle, table, table_np, lg_np, dtype, states_np, temperature, seed, offset, masked=True):
    B = len(states_np)
    lg = _to_dev(lg_np, dtype)
    st = torch.from_numpy(states_np).cuda()
    tok = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    new = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    out = torch.empty_like(lg) if masked else None
    T.sample_step(table, lg, st, temperature, seed, offset, tok, new, out)
    torch.cuda.synchronize()
    res = oracle.sample_step(table_np, lg_np, dtype, states_np, temperature, seed, offset, want_masked=masked,
                             n_threads=16)
    assert np.array_equal(tok.cpu().numpy(), res[0]), (tok.cpu().numpy()[:8], res[0][:8])
    assert np.array_equal(new.cpu().numpy(), res[1])
    if masked:
        V = table_np.shape[1]
        assert np.array_equal(_bits(out)[:, :V], res[2].view(_bits(out).dtype)[:, :V])
    return res


@pytest.mark.parametrize("batch,n_tokens,seed,offset", [(3, 1001, 1, 0), (2, 128256, 2 ** 63 + 5, 2 ** 40 + 9),
                                                         (70, 4099, 0, 2 ** 32 - 1)])
def test_noise_bit_for_bit(T, oracle, batch, n_tokens, seed, offset):
    """Every noise value, compared as bit patterns: the generator words, the uniform grid and both
    logarithms of each of them."""
    got = torch.empty((batch, n_tokens), dtype=torch.float32, device="cuda")
    T.sample_noise(got, seed, offset)
    torch.cuda.synchronize()
    want = oracle.sample_noise(batch, n_tokens, seed, offset)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("p_live", [0.02, 0.9])
@pytest.mark.parametrize("n_tokens,batch", [(8, 1), (37 * 8 + 3, 3), (1000 * 8 + 8, 5), (40000, 2), (50021, 300)])
def test_random_tables(T, oracle, dtype, p_live, n_tokens, batch):
    """Sparse and dense allowed sets; sizes cover one group, ragged rows, many parts per row and one
    workgroup per row; states include sinks, DEAD and ids that are no row."""
    tab = _rand_table(11, n_tokens, p_live, n_tokens + batch)
    tab[3] = DEAD
    tab[4] = DEAD
    tab[4, n_tokens - 1] = 6
    table = _upload_table(T, tab)
    rng = np.random.default_rng(batch)
    stride = (n_tokens + 7) // 8 * 8
    for trial, temperature in enumerate((1.0, 0.35, 3.0)):
        states = rng.integers(-1, 12, size=batch).astype(np.int32)
        states[: min(batch, 2)] = [3, 4][: min(batch, 2)]
        x = np.zeros((batch, stride), dtype=np.float32)
        x[:, :n_tokens] = rng.normal(0, 2, size=(batch, n_tokens))
        lg = x if dtype == F32 else LG.f32_to_bf16_bits(x)
        got = _sample_strided(T, oracle, table, tab, lg, dtype, states, temperature, 1234 + trial, 77 * trial,
                              masked=trial != 1)
    assert (got[0] >= 0).any() or batch <= 2


def _sample_strided(T, oracle, table, table_np, lg_np, dtype, states_np, temperature, seed, offset, masked, top_k=0):
    """Rows padded to a multiple of 8 elements (the alignment rule); the padding is not touched."""
    B, stride = lg_np.shape
    V = table_np.shape[1]
    lg = _to_dev(lg_np, dtype)
    st = torch.from_numpy(states_np).cuda()
    tok = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    new = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    out = torch.full_like(lg, 7.0) if masked else None
    T.sample_step(table, lg, st, temperature, seed, offset, tok, new, out, top_k=top_k)
    torch.cuda.synchronize()
    res = oracle.sample_step(table_np, lg_np, dtype, states_np, temperature, seed, offset, row_stride=stride,
                             want_masked=masked, n_threads=16, top_k=top_k)
    assert np.array_equal(tok.cpu().numpy(), res[0]), (tok.cpu().numpy()[:8], res[0][:8])
    assert np.array_equal(new.cpu().numpy(), res[1])
    if masked:
        assert np.array_equal(_bits(out)[:, :V], res[2].view(_bits(out).dtype)[:, :V])
        assert (out[:, V:].float() == 7.0).all()
    return res


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("p_live", [0.02, 0.9])
@pytest.mark.parametrize("n_tokens,batch", [(8, 1), (37 * 8 + 3, 3), (40000, 2), (50021, 200)])
def test_top_k(T, oracle, dtype, p_live, n_tokens, batch):
    """The cut at the k-th largest allowed logit: k from 1 to more than the vocabulary, logits with
    many ties (rounded), NaN and infinities, one and many workgroups per row."""
    tab = _rand_table(11, n_tokens, p_live, 7 * n_tokens + batch)
    tab[3] = DEAD
    tab[4] = DEAD
    tab[4, n_tokens - 1] = 6
    table = _upload_table(T, tab)
    rng = np.random.default_rng(batch + 1)
    stride = (n_tokens + 7) // 8 * 8
    for trial, k in enumerate((1, 2, 7, 50, 4000, 10 ** 6)):
        states = rng.integers(-1, 12, size=batch).astype(np.int32)
        states[: min(batch, 2)] = [3, 4][: min(batch, 2)]
        x = np.zeros((batch, stride), dtype=np.float32)
        x[:, :n_tokens] = rng.normal(0, 2, size=(batch, n_tokens))
        if trial % 3 == 1:
            x = np.round(x * 2) / 2                                  # heavy ties, also across the cut
        if trial % 3 == 2:
            x[:, rng.integers(0, n_tokens, max(1, n_tokens // 50))] = np.nan
            x[:, rng.integers(0, n_tokens, max(1, n_tokens // 200))] = -np.inf
            x[:, rng.integers(0, n_tokens, 2)] = np.inf
            x[:, rng.integers(0, n_tokens, max(1, n_tokens // 100))] = -0.0
        lg = x if dtype == F32 else LG.f32_to_bf16_bits(x)
        _sample_strided(T, oracle, table, tab, lg, dtype, states, (1.0, 0.4, 2.5)[trial % 3], 99 + trial, trial,
                        masked=trial == 0, top_k=k)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_special_values(T, oracle, dtype):
    n_tokens = 4096 + 64
    tab = _rand_table(5, n_tokens, 0.3, 1)
    table = _upload_table(T, tab)
    rng = np.random.default_rng(9)
    states = np.array([0, 1, 2, 3, 4, 0, 1], dtype=np.int32)
    B = len(states)
    cases = [np.full((B, n_tokens), 1.25, np.float32)]                                 # the noise alone decides
    x = rng.normal(0, 2, size=(B, n_tokens)).astype(np.float32)
    x[:, rng.integers(0, n_tokens, 200)] = np.nan
    x[:, rng.integers(0, n_tokens, 50)] = -np.inf
    cases.append(x.copy())
    x[:, rng.integers(0, n_tokens, 50)] = np.inf                                       # several +inf: lowest allowed id
    cases.append(x)
    y = np.full((B, n_tokens), -np.inf, np.float32)                                    # no mass anywhere
    y[:, rng.integers(0, n_tokens, 500)] = np.nan
    cases.append(y)
    cases.append(np.full((B, n_tokens), 3.0e38, np.float32))                           # l / T overflows at T < 1
    cases.append(rng.normal(0, 1e-30, size=(B, n_tokens)).astype(np.float32))          # tiny logits
    for i, x in enumerate(cases):
        lg = x if dtype == F32 else LG.f32_to_bf16_bits(x)
        if dtype == BF16 and np.isnan(x).any():
            lg = lg.copy()
            nan_pos = np.argwhere(np.isnan(x))
            lg[nan_pos[::2, 0], nan_pos[::2, 1]] = 0xFFFF
            lg[nan_pos[1::2, 0], nan_pos[1::2, 1]] = 0x7F81
        for temperature in (1.0, 0.01, 100.0):
            _step_and_check(T, oracle, table, tab, lg, dtype, states, temperature, 5 + i, i)
    with pytest.raises(T.TdfaError):
        T.sample_step(table, _to_dev(cases[0], F32), torch.from_numpy(states).cuda(), 0.0, 1, 0,
                      torch.empty(B, dtype=torch.int32, device="cuda"), torch.empty(B, dtype=torch.int32, device="cuda"))


def _decode(T, oracle, table, table_np, w, start_states, steps, check_steps, seed, temperature, noise_seed):
    """Chained sampled steps on the device, offset = step number; the listed steps are checked
    against the oracle fed with the device's own input states."""
    m = w.mask
    B, V = m.batch, w.vocab.n_tokens
    tdt = torch.float32 if m.dtype == "f32" else torch.bfloat16
    dt = F32 if m.dtype == "f32" else BF16
    hist_states = torch.empty((steps + 1, B), dtype=torch.int32, device="cuda")
    hist_tok = torch.empty((steps, B), dtype=torch.int32, device="cuda")
    hist_states[0] = torch.from_numpy(start_states.astype(np.int32)).cuda()
    logits = torch.empty((B, V), dtype=tdt, device="cuda")
    kept = {}
    stream = torch.cuda.current_stream().cuda_stream
    for s in range(steps):
        LG.gen_logits_device(logits.data_ptr(), seed, s, B, V, V, m.sigma, m.dtype, stream)
        if s in check_steps:
            kept[s] = logits.clone()
        T.sample_step(table, logits, hist_states[s], temperature, noise_seed, s, hist_tok[s], hist_states[s + 1])
    torch.cuda.synchronize()
    hs, ht = hist_states.cpu().numpy(), hist_tok.cpu().numpy()
    for s in sorted(check_steps):
        lg_np = _bits(kept[s]) if dt == BF16 else kept[s].cpu().numpy()
        tok, new = oracle.sample_step(table_np, lg_np, dt, hs[s], temperature, noise_seed, s, n_threads=16)
        assert np.array_equal(ht[s], tok), f"step {s}: tokens differ"
        assert np.array_equal(hs[s + 1], new), f"step {s}: states differ"
    return hs, ht


def test_c2_sampled_decode(T, oracle):
    """JSON-like constraint: 64 sequences, 128 sampled steps, every step checked; what was generated
    stays inside the language (the states never go DEAD) and differs between sequences."""
    w = configs.get("c2")
    d = w.dfas[0]
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    table = T.compile_token_dfa(v, T.CharDFA(d.trans, d.accept, d.start))
    tab = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=8)
    hs, ht = _decode(T, oracle, table, tab, w, np.full(64, d.start), 128, set(range(128)), configs.logits_seed(2), 1.0, 42)
    assert (hs >= 0).all()
    stopped = ht[-1] < 0
    assert d.accept[hs[-1][stopped]].all()
    assert len({tuple(r) for r in ht.T.tolist()}) > 32


def test_c3_sampled_full_size(T, oracle):
    """The API-call union at its full shape (128,256 tokens, batch 256, one workgroup per row), 40
    steps of a sampled decode, every step checked."""
    w = configs.get("c3")
    d = w.dfas[0]
    v = T.Vocab(w.vocab.data, w.vocab.offsets)
    table = T.compile_token_dfa(v, T.CharDFA(d.trans, d.accept, d.start))
    tab = oracle.compile_walk(d.trans, w.vocab.data, w.vocab.offsets, n_threads=16)
    hs, ht = _decode(T, oracle, table, tab, w, np.full(256, d.start), 40, set(range(40)), configs.logits_seed(3),
                     0.8, 7)
    assert len(np.unique(hs)) > 50


def test_offset_from_device_memory_in_a_graph(T, oracle):
    """tdfa_sample_step_at: a recorded decode loop whose offset lives in device memory and is
    advanced by the loop itself; every replay, with eager work between the replays, gives what
    the eager loop with explicit offsets gives (and step 0 what the oracle gives)."""
    n_tokens, B, S = 5003, 16, 6
    tab = _rand_table(9, n_tokens, 0.3, 21)
    table = _upload_table(T, tab)
    rng = np.random.default_rng(2)
    stride = (n_tokens + 7) // 8 * 8
    xs = [np.zeros((B, stride), dtype=np.float32) for _ in range(S)]
    for x in xs:
        x[:, :n_tokens] = rng.normal(0, 2, size=(B, n_tokens))
    lgs = [_to_dev(LG.f32_to_bf16_bits(x), BF16) for x in xs]
    start_np = rng.integers(0, 9, size=B).astype(np.int32)
    start = torch.from_numpy(start_np).cuda()
    seed, first = 77, 1000

    def loop(states, tokens, offset):
        states[0].copy_(start)
        for s in range(S):
            off = offset if isinstance(offset, torch.Tensor) else offset + s
            T.sample_step(table, lgs[s], states[s], 0.9, seed, off, tokens[s], states[s + 1], top_k=40)
            if isinstance(offset, torch.Tensor):
                offset.add_(1)

    ref_states = torch.empty((S + 1, B), dtype=torch.int32, device="cuda")
    ref_tokens = torch.empty((S, B), dtype=torch.int32, device="cuda")
    loop(ref_states, ref_tokens, first)
    torch.cuda.synchronize()
    tok0, new0 = oracle.sample_step(tab, LG.f32_to_bf16_bits(xs[0]), BF16, start_np, 0.9, seed, first, row_stride=stride, top_k=40)
    assert np.array_equal(ref_tokens[0].cpu().numpy(), tok0) and np.array_equal(ref_states[1].cpu().numpy(), new0)
    assert len({tuple(r) for r in ref_tokens.cpu().numpy().tolist()}) > 1          # the steps do differ

    counter = torch.full((1,), first, dtype=torch.int64, device="cuda")
    g_states = torch.empty_like(ref_states)
    g_tokens = torch.empty_like(ref_tokens)
    loop(g_states, g_tokens, counter)                                            # eager, device offset
    torch.cuda.synchronize()
    assert torch.equal(g_tokens, ref_tokens) and torch.equal(g_states, ref_states)
    assert int(counter.item()) == first + S
    graph = torch.cuda.CUDAGraph()
    counter.fill_(first)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        loop(g_states, g_tokens, counter)
    for replay in range(3):
        g_tokens.fill_(-5)
        counter.fill_(first)
        scratch = (torch.arange(1000, device="cuda") * (replay + 1)).sum()      # the program's own eager work
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_tokens, ref_tokens) and torch.equal(g_states, ref_states), f"replay {replay}"
        assert int(counter.item()) == first + S and int(scratch.item()) >= 0


@pytest.mark.parametrize("batch,n_tokens", [(3, 3000), (250, 40000)])
def test_masked_row_in_place(T, oracle, batch, n_tokens):
    """masked_out may be the logits themselves, states may be advanced in place, with a top-k cut."""
    tab = _rand_table(7, n_tokens, 0.2, 2)
    table = _upload_table(T, tab)
    rng = np.random.default_rng(batch)
    x = rng.normal(0, 2, size=(batch, n_tokens)).astype(np.float32)
    bits = LG.f32_to_bf16_bits(x)
    states = rng.integers(0, 7, size=batch).astype(np.int32)
    want_tok, want_new, want_masked = oracle.sample_step(tab, bits, BF16, states, 1.3, 8, 4, want_masked=True, top_k=25,
                                                         n_threads=16)
    lg = _to_dev(bits, BF16)
    st = torch.from_numpy(states).cuda()
    tok = torch.empty(batch, dtype=torch.int32, device="cuda")
    T.sample_step(table, lg, st, 1.3, 8, 4, tok, st, lg, top_k=25)
    torch.cuda.synchronize()
    assert np.array_equal(tok.cpu().numpy(), want_tok) and np.array_equal(st.cpu().numpy(), want_new)
    assert np.array_equal(_bits(lg), want_masked)
