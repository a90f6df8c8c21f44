"""Pins for the oracle's decode step (Algorithm 2 loop body): closed forms, special cases that
reduce to numpy's argmax, the no-touch property of Appendix B.2.2, and an end-to-end decode
checked against Python's `re`."""
import re

import numpy as np
import pytest

from workloads import configs, logits as LG, vocab as V
from workloads.regex_dfa import compile_regex

DEAD = -1
F32, BF16 = 0, 1
NEG_INF_F32 = np.uint32(0xFF800000)
NEG_INF_BF16 = np.uint16(0xFF80)


def _table(n_rows=6, n_tokens=37, p_live=0.3, seed=0):
    rng = np.random.default_rng(seed)
    t = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
    t[rng.random((n_rows, n_tokens)) > p_live] = DEAD
    return t


def _as(dtype, x):
    x = np.asarray(x, dtype=np.float32)
    return x if dtype == F32 else LG.f32_to_bf16_bits(x)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_closed_forms(oracle, dtype):
    table = _table()
    table[3, :] = DEAD                      # state 3: nothing allowed (a sink)
    table[4, :] = DEAD
    table[4, 11] = 2                        # state 4: exactly one allowed token
    n_rows, n_tok = table.shape
    states = np.array([0, 1, 2, 3, 4, 5, DEAD, n_rows, -7], dtype=np.int32)
    B = len(states)
    # ascending ramp: the winner is the largest allowed id
    ramp = _as(dtype, np.tile(np.arange(n_tok, dtype=np.float32) * 0.5 - 4.0, (B, 1)))
    tok, new = oracle.mask_step(table, ramp, dtype, states)
    for b, q in enumerate(states):
        if 0 <= q < n_rows and (table[q] >= 0).any():
            want = int(np.nonzero(table[q] >= 0)[0].max())
            assert tok[b] == want and new[b] == table[q, want]
    # all equal: the winner is the smallest allowed id
    flat = _as(dtype, np.full((B, n_tok), 1.25, dtype=np.float32))
    tok, new = oracle.mask_step(table, flat, dtype, states)
    for b, q in enumerate(states):
        if 0 <= q < n_rows and (table[q] >= 0).any():
            want = int(np.nonzero(table[q] >= 0)[0].min())
            assert tok[b] == want and new[b] == table[q, want]
    assert tok[4] == 11 and new[4] == 2                 # single allowed token
    assert tok[3] == -1 and new[3] == 3                 # sink: no token, state held
    for b in (6, 7, 8):                                 # DEAD or out of range
        assert tok[b] == -1 and new[b] == DEAD


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_matches_numpy_argmax(oracle, dtype):
    rng = np.random.default_rng(5)
    table = _table(n_rows=9, n_tokens=301, p_live=0.2, seed=3)
    for trial in range(20):
        states = rng.integers(0, 9, size=7).astype(np.int32)
        x = rng.normal(0, 2, size=(7, 301)).astype(np.float32)
        lg = _as(dtype, x)
        vals = x if dtype == F32 else LG.bf16_bits_to_f32(lg)
        tok, new, masked = oracle.mask_step(table, lg, dtype, states, want_masked=True)
        allowed = table[states] >= 0
        ref = np.where(allowed, vals, -np.inf)
        want = np.argmax(ref, axis=1)                    # numpy: first index of the maximum
        has = allowed.any(axis=1)
        assert np.array_equal(tok[has], want[has]) and (tok[~has] == -1).all()
        assert np.array_equal(new[has], table[states[has], want[has]])
        # Appendix B.2.2: allowed logits untouched bit for bit, the rest exactly -inf
        assert np.array_equal(masked[allowed], lg[allowed])
        ninf = NEG_INF_F32 if dtype == F32 else NEG_INF_BF16
        assert (masked.view(np.uint32 if dtype == F32 else np.uint16)[~allowed] == ninf).all()


def test_bf16_ties_lowest_id(oracle):
    table = np.zeros((1, 64), dtype=np.int32)
    table[0, :5] = DEAD
    x = np.full((1, 64), 3.0, dtype=np.float32)
    x[0, [9, 20, 41]] = 8.03125      # 8.03125 and 8.0 round to the same bf16 value (spacing 1/16)
    x[0, 30] = 8.0
    x[0, 2] = 50.0                   # larger, but not allowed
    tok, new = oracle.mask_step(table, LG.f32_to_bf16_bits(x), BF16, np.zeros(1, np.int32))
    assert tok[0] == 9
    tok, _ = oracle.mask_step(table, x, F32, np.zeros(1, np.int32))
    assert tok[0] == 9
    x[0, 30] = 8.04
    tok, _ = oracle.mask_step(table, x, F32, np.zeros(1, np.int32))
    assert tok[0] == 30


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_nan_and_inf(oracle, dtype):
    table = np.zeros((1, 16), dtype=np.int32)
    table[0, 0] = DEAD
    st = np.zeros(1, np.int32)
    x = np.full((1, 16), -1.0, dtype=np.float32)
    x[0, 3] = np.nan
    x[0, 5] = 2.0
    x[0, 0] = np.inf                  # not allowed
    assert oracle.mask_step(table, _as(dtype, x), dtype, st)[0][0] == 5     # NaN never beats a number
    x[0, 7] = np.inf
    assert oracle.mask_step(table, _as(dtype, x), dtype, st)[0][0] == 7
    # only -inf and NaN among the allowed: they rank equal, lowest id wins, and a token is still chosen
    y = np.full((1, 16), -np.inf, dtype=np.float32)
    y[0, 2] = np.nan
    assert oracle.mask_step(table, _as(dtype, y), dtype, st)[0][0] == 1
    y[0, 1] = np.nan
    y[0, 0] = 1.0
    assert oracle.mask_step(table, _as(dtype, y), dtype, st)[0][0] == 1
    if dtype == BF16:                 # negative-sign NaN pattern
        z = LG.f32_to_bf16_bits(np.full((1, 16), -np.inf, dtype=np.float32))
        z[0, 1] = 0xFFFF
        z[0, 4] = 0x7FC1
        assert oracle.mask_step(table, z, dtype, st)[0][0] == 1


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_signed_zeros_tie(oracle, dtype):
    """-0 and +0 are the same value, so the lowest id among them wins."""
    table = np.zeros((1, 8), dtype=np.int32)
    x = np.array([[-1.0, -0.0, 0.0, -0.0, 0.0, -2.0, 0.0, -0.0]], dtype=np.float32)
    assert oracle.mask_step(table, _as(dtype, x), dtype, np.zeros(1, np.int32))[0][0] == 1
    assert int(np.argmax(x)) == 1                         # numpy agrees: first index of the maximum


def test_row_stride_and_empty(oracle):
    table = _table(n_rows=4, n_tokens=10, p_live=0.5, seed=2)
    rng = np.random.default_rng(0)
    wide = rng.normal(size=(3, 16)).astype(np.float32)
    st = np.array([0, 1, 2], dtype=np.int32)
    tok_w, new_w = oracle.mask_step(table, wide, F32, st, row_stride=16)
    tok_n, new_n = oracle.mask_step(table, np.ascontiguousarray(wide[:, :10]), F32, st)
    assert np.array_equal(tok_w, tok_n) and np.array_equal(new_w, new_n)
    tok, new = oracle.mask_step(table, np.zeros((0, 10), np.float32), F32, np.zeros(0, np.int32))
    assert len(tok) == 0 and len(new) == 0


def test_decode_loop_generates_members(oracle):
    """Algorithm 2 end to end on the Figure 3/4 example and on c1: whatever the logits say, the
    detokenized output is a viable prefix and, once the automaton stops, a member of the language."""
    cases = [(r"(foo)+d", V.from_tokens([b"f", b"oo", b"foo", b"for", b"food"])),
             (configs.C1_PATTERN, configs.get("c1").vocab)]
    for pattern, vocab in cases:
        d = compile_regex(pattern)
        cre = re.compile(pattern.encode())
        table = oracle.compile_compose(d.trans, vocab.data, vocab.offsets)
        toks = vocab.tokens()
        B = 16
        states = np.full(B, d.start, dtype=np.int32)
        texts = [b""] * B
        done_at_accept = 0
        for step in range(24):
            lg = LG.gen_logits(1234, step, B, vocab.n_tokens, 1.0, "f32")
            tok, new = oracle.mask_step(table, lg, F32, states)
            for b in range(B):
                if tok[b] >= 0:
                    assert table[states[b], tok[b]] == new[b] >= 0
                    texts[b] += toks[tok[b]]
                    assert bool(d.accept[new[b]]) == (cre.fullmatch(texts[b]) is not None)
                else:                                   # nothing allowed: must be a final state
                    assert new[b] == states[b] and d.accept[states[b]]
                    assert cre.fullmatch(texts[b]) is not None
                    done_at_accept += 1
            states = new
        if pattern == configs.C1_PATTERN:
            assert done_at_accept > 0


def test_concat_tables(oracle):
    a, b, c = _table(3, 11, 0.5, 1), _table(5, 11, 0.5, 2), _table(2, 11, 0.5, 3)
    out, offs = oracle.concat_tables([a, b, c])
    assert offs.tolist() == [0, 3, 8, 10] and out.shape == (10, 11)
    for t, o in zip((a, b, c), offs[:-1]):
        blk = out[o:o + t.shape[0]]
        assert np.array_equal(blk == DEAD, t == DEAD)
        assert np.array_equal(blk[t >= 0], t[t >= 0] + o)
