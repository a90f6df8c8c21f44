"""tdfa_mask_step_noalloc (the decode step on the library's fixed scratch array, for callers that
cannot allocate) against tdfa_mask_step, through the C ABI, bit for bit."""
import numpy as np
import pytest
import torch

from workloads import logits as LG
import gpu_util as G

pytestmark = pytest.mark.gpu
DEAD = -1


@pytest.fixture(scope="module")
def T():
    import paper_2407_08103_amd as T
    assert torch.cuda.is_available()
    return T


def _table(T, n_rows, n_tokens, p_live, seed):
    rng = np.random.default_rng(seed)
    t = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
    t[rng.random((n_rows, n_tokens)) > p_live] = DEAD
    t[1] = DEAD                                                  # a state that allows nothing
    delta = torch.from_numpy(t).cuda()
    allow = torch.from_numpy(G.bits_from_table(t, T.allow_row_words(n_tokens)).view(np.int32)).cuda()
    return T.table_wrap(delta, allow), t


def _both(T, table, n_rows, batch, n_tokens, dtype, seed, masked):
    rng = np.random.default_rng(seed)
    stride = (n_tokens + 7) // 8 * 8
    x = np.zeros((batch, stride), dtype=np.float32)
    x[:, :n_tokens] = rng.normal(0, 2, size=(batch, n_tokens))
    if dtype == "bf16":
        lg = torch.from_numpy(LG.f32_to_bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        lg = torch.from_numpy(x).cuda()
    states = torch.from_numpy(rng.integers(-1, n_rows + 1, size=batch).astype(np.int32)).cuda()
    out = []
    for fn in (T.mask_step, T.mask_step_noalloc):
        tok = torch.full((batch,), -9, dtype=torch.int32, device="cuda")
        new = torch.full((batch,), -9, dtype=torch.int32, device="cuda")
        m = torch.zeros_like(lg) if masked else None
        fn(table, lg, states, tok, new, m)
        torch.cuda.synchronize()
        out.append((tok, new, m))
    (t0, n0, m0), (t1, n1, m1) = out
    assert torch.equal(t0, t1), "tokens differ"
    assert torch.equal(n0, n1), "states differ"
    if masked:
        assert torch.equal(m0.view(torch.int16 if dtype == "bf16" else torch.int32),
                           m1.view(torch.int16 if dtype == "bf16" else torch.int32)), "masked rows differ"
    assert int((t0 >= 0).sum()) > 0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_two_calls_second_smaller(T, dtype):
    """Rows split over several workgroups (the scratch is in use); the second call has a smaller
    batch and a shorter vocabulary than the first and runs on what the first left behind."""
    big, _ = _table(T, 9, 40003, 0.05, 1)
    small, _ = _table(T, 5, 9001, 0.3, 2)
    _both(T, big, 9, 64, 40003, dtype, 3, masked=True)
    _both(T, small, 5, 7, 9001, dtype, 4, masked=False)
    _both(T, big, 9, 1, 40003, dtype, 5, masked=False)


def test_chained_steps_and_one_workgroup_per_row(T):
    """A chained decode (states advanced in place) on both entry points, at a batch where each row
    has its own workgroup (the scratch is idle) and at one where rows are split."""
    for batch in (256, 48):
        table, _ = _table(T, 50, 50021, 0.2, 10 + batch)
        rng = np.random.default_rng(batch)
        stride = (50021 + 7) // 8 * 8
        runs = []
        for fn in (T.mask_step, T.mask_step_noalloc):
            st = torch.from_numpy((np.arange(batch) % 50).astype(np.int32)).cuda()
            toks = torch.empty((6, batch), dtype=torch.int32, device="cuda")
            r = np.random.default_rng(7)
            for s in range(6):
                x = np.zeros((batch, stride), dtype=np.float32)
                x[:, :50021] = r.normal(0, 2, size=(batch, 50021))
                lg = torch.from_numpy(LG.f32_to_bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)
                fn(table, lg, st, toks[s], st)
            torch.cuda.synchronize()
            runs.append((toks, st))
        assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])


def test_batch_beyond_the_array_is_refused(T):
    table, _ = _table(T, 3, 64, 0.5, 3)
    batch = 4097
    lg = torch.zeros((batch, 64), dtype=torch.bfloat16, device="cuda")
    st = torch.zeros(batch, dtype=torch.int32, device="cuda")
    tok = torch.full((batch,), -9, dtype=torch.int32, device="cuda")
    with pytest.raises(T.TdfaError) as e:
        T.mask_step_noalloc(table, lg, st, tok, st)
    assert e.value.code == -4 and "4096" in str(e.value)
    torch.cuda.synchronize()
    assert int((tok != -9).sum()) == 0                           # nothing was launched
    T.mask_step_noalloc(table, lg[:4096], st[:4096], tok[:4096], st[:4096])
    torch.cuda.synchronize()
    assert int((tok[:4096] == -9).sum()) == 0
