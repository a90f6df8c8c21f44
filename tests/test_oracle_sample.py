"""Pins for the oracle's sampling step (SampleNextToken of Algorithm 2 read as a draw from
softmax(l / T) over the allowed set, by the Gumbel-max rule): the generator's published
known-answer vectors, the binary32 logarithm against the exact one, the distribution of the
noise and of the chosen tokens against their closed forms, the greedy limit, and the handling of
the mask, which must be that of the greedy step."""
import math
import os

import numpy as np
import pytest
from scipy import stats

from workloads import logits as LG

DEAD = -1
F32, BF16 = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _table(n_rows=6, n_tokens=37, p_live=0.3, seed=0):
    rng = np.random.default_rng(seed)
    t = rng.integers(0, n_rows, size=(n_rows, n_tokens), dtype=np.int32)
    t[rng.random((n_rows, n_tokens)) > p_live] = DEAD
    return t


def test_philox_known_answers(oracle):
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]


def test_ln32_against_exact_logarithm(oracle):
    """Within 3 units in the last place of the exact logarithm wherever the result is not close to
    zero, and within 2.5e-7 relative near x = 1 (where f = x - 1 is exact and small)."""
    rng = np.random.default_rng(1)
    x = np.concatenate([
        np.exp(rng.uniform(math.log(2.0 ** -24), math.log(17.0), 20000)),     # the range the sampler uses
        rng.uniform(0.5, 2.0, 20000),
        1.0 + rng.uniform(-1e-3, 1e-3, 5000),
        np.float32(2.0) ** np.arange(-120, 120),
        [np.nextafter(np.float32(1), np.float32(0)), np.nextafter(np.float32(1), np.float32(2)),
         np.sqrt(2.0), np.nextafter(np.float32(np.sqrt(2.0)), np.float32(2)), np.sqrt(0.5), 0.5, 2.0, 1.0],
    ]).astype(np.float32)
    got = oracle.ln32(x).astype(np.float64)
    want = np.log(x.astype(np.float64))
    assert got[-1] == 0.0                                                     # ln 1 = 0 exactly
    err = np.abs(got - want)
    ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
    far = np.abs(want) > 0.1
    assert (err[far] <= 3.0 * ulp[far]).all()
    nz = want != 0
    assert (err[nz] / np.abs(want[nz])).max() < 2.5e-7
    # powers of two: e * ln 2 rounded once
    p2 = np.float32(2.0) ** np.arange(-120, 120)
    assert np.array_equal(oracle.ln32(p2), (np.arange(-120, 120) * np.float32(math.log(2))).astype(np.float32))


def test_uniform_grid_and_gumbel_law(oracle):
    """u lies on the grid (k + 1/2) 2^-23 inside (0, 1); g = -ln(-ln u) within rounding; the
    empirical law of g is the standard Gumbel one (Kolmogorov-Smirnov)."""
    n = 20000
    u = np.array([oracle.uniform(7, 3, t % 5, t) for t in range(n)], dtype=np.float64)
    k = u * 2 ** 23 - 0.5
    assert np.array_equal(k, np.round(k)) and k.min() >= 0 and k.max() < 2 ** 23
    g = np.array([oracle.gumbel(7, 3, t % 5, t) for t in range(n)], dtype=np.float64)
    assert np.abs(g - (-np.log(-np.log(u)))).max() < 4e-6
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    assert stats.kstest(g, "gumbel_r").pvalue > 1e-3
    # the four words of one generator block serve four neighbouring tokens; blocks differ by
    # token quad, sequence, offset and seed
    base = oracle.uniform(7, 3, 2, 40)
    others = [oracle.uniform(7, 3, 2, 41), oracle.uniform(7, 3, 2, 44), oracle.uniform(7, 3, 3, 40),
              oracle.uniform(7, 4, 2, 40), oracle.uniform(8, 3, 2, 40), oracle.uniform(7 + (1 << 32), 3, 2, 40),
              oracle.uniform(7, 3 + (1 << 32), 2, 40)]
    assert len({base, *others}) == 8
    want = oracle.philox4x32_10([10, 2, 3, 0], [7, 0])
    for j in range(4):
        assert oracle.uniform(7, 3, 2, 40 + j) == ((int(want[j]) >> 9) + 0.5) * 2.0 ** -23


@pytest.mark.parametrize("dtype,temperature", [(F32, 1.0), (F32, 0.5), (BF16, 2.0)])
def test_distribution_is_masked_softmax(oracle, dtype, temperature):
    """Chi-square test of the drawn tokens against softmax(l / T) over the allowed set."""
    n_tok = 23
    table = np.full((2, n_tok), DEAD, dtype=np.int32)
    allowed = [1, 4, 5, 9, 16, 22]
    table[1, allowed] = 0
    rng = np.random.default_rng(5)
    l = rng.normal(0, 1.5, n_tok).astype(np.float32)
    l[[0, 2, 3]] = 30.0                                   # large, but masked out
    bits = l if dtype == F32 else LG.f32_to_bf16_bits(l)
    lv = l if dtype == F32 else LG.bf16_bits_to_f32(bits)
    B, n_off = 500, 40
    logits = np.tile(bits, (B, 1))
    states = np.ones(B, dtype=np.int32)
    counts = np.zeros(n_tok, dtype=np.int64)
    for off in range(n_off):
        tok, new = oracle.sample_step(table, logits, dtype, states, temperature, 99, off)
        assert (new == 0).all()
        counts += np.bincount(tok, minlength=n_tok)
    assert counts.sum() == B * n_off and counts[[t for t in range(n_tok) if t not in allowed]].sum() == 0
    p = np.exp(lv[allowed].astype(np.float64) / temperature)
    p /= p.sum()
    chi = stats.chisquare(counts[allowed], p * counts.sum())
    assert chi.pvalue > 1e-3, (counts[allowed], p * counts.sum())
    # a wrong temperature (T in place of 1/T, or none) is rejected by the same test
    if temperature != 1.0:
        for wrong in (1.0, 1.0 / temperature):
            pw = np.exp(lv[allowed].astype(np.float64) / wrong)
            pw /= pw.sum()
            assert stats.chisquare(counts[allowed], pw * counts.sum()).pvalue < 1e-6


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_greedy_limit_and_mask(oracle, dtype):
    """With a small temperature the draw is the greedy choice; the masked row, the handling of
    sinks, DEAD and out-of-range states are those of the greedy step at any temperature."""
    table = _table(seed=3)
    table[3, :] = DEAD
    n_rows, n_tok = table.shape
    states = np.array([0, 1, 2, 3, 4, 5, DEAD, n_rows, -7, 0, 1], dtype=np.int32)
    rng = np.random.default_rng(8)
    x = rng.permutation(len(states) * n_tok).reshape(len(states), n_tok).astype(np.float32) * 0.25 - 20.0
    logits = x if dtype == F32 else LG.f32_to_bf16_bits(x)
    if dtype == BF16:                                     # keep the values distinct after rounding
        logits = LG.f32_to_bf16_bits(np.argsort(np.argsort(x, axis=1), axis=1).astype(np.float32) - 10.0)
    gt, gn, gm = oracle.mask_step(table, logits, dtype, states, want_masked=True)
    st, sn, sm = oracle.sample_step(table, logits, dtype, states, 1e-3, 1, 0, want_masked=True)
    assert np.array_equal(st, gt) and np.array_equal(sn, gn) and np.array_equal(sm, gm)
    for T in (0.7, 5.0):
        st, sn, sm = oracle.sample_step(table, logits, dtype, states, T, 2, 11, want_masked=True)
        assert np.array_equal(sm, gm)
        for b, q in enumerate(states):
            if 0 <= q < n_rows and (table[q] >= 0).any():
                assert table[q, st[b]] >= 0 and sn[b] == table[q, st[b]]
            else:
                assert st[b] == gt[b] and sn[b] == gn[b]
    # at a high temperature the draws do differ from the greedy choice somewhere
    st, _ = oracle.sample_step(table, np.tile(logits[:1], (64, 1)), dtype, np.zeros(64, np.int32), 50.0, 3, 0)
    assert len(set(st.tolist())) > 1


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_special_values(oracle, dtype):
    """-inf has probability zero, +inf is certain, NaN counts as -inf; when every allowed logit is
    -inf the lowest allowed id is taken, as in the greedy step."""
    n_tok = 12
    table = np.full((1, n_tok), DEAD, dtype=np.int32)
    table[0, [2, 3, 7, 8]] = 0
    ninf, pinf, nan = -np.inf, np.inf, np.nan
    rows = np.zeros((4, n_tok), dtype=np.float32)
    rows[0, [2, 3, 7, 8]] = [ninf, 1.0, ninf, nan]       # only token 3 has mass
    rows[1, [2, 3, 7, 8]] = [0.0, 5.0, pinf, 3.0]        # +inf wins
    rows[2, [2, 3, 7, 8]] = [ninf, nan, ninf, nan]       # nothing has mass: lowest allowed id
    rows[3, [2, 3, 7, 8]] = [0.0, pinf, pinf, 1.0]       # two +inf: the lower id
    logits = np.tile(rows, (16, 1))
    bits = logits if dtype == F32 else LG.f32_to_bf16_bits(logits)
    for off in range(8):
        tok, new = oracle.sample_step(table, bits, dtype, np.zeros(64, np.int32), 1.0, 5, off)
        assert tok.reshape(16, 4).tolist() == [[3, 7, 2, 3]] * 16


def test_reproducible_and_seeded(oracle):
    table = _table(n_rows=4, n_tokens=300, p_live=0.5, seed=4)
    rng = np.random.default_rng(6)
    logits = rng.normal(0, 2, (32, 300)).astype(np.float32)
    states = rng.integers(0, 4, 32).astype(np.int32)
    a = oracle.sample_step(table, logits, F32, states, 1.0, 10, 0)
    b = oracle.sample_step(table, logits, F32, states, 1.0, 10, 0, n_threads=4)
    c = oracle.sample_step(table, logits, F32, states, 1.0, 11, 0)
    d = oracle.sample_step(table, logits, F32, states, 1.0, 10, 1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[0], c[0]) and not np.array_equal(a[0], d[0])
    # the noise of sequence b does not depend on the batch it is in
    e = oracle.sample_step(table, logits[:5], F32, states[:5], 1.0, 10, 0)
    assert np.array_equal(e[0], a[0][:5])
    for bad in (0.0, -1.0, float("nan"), 1e-45):
        with pytest.raises(RuntimeError):
            oracle.sample_step(table, logits, F32, states, bad, 1, 0)


def test_noise_is_monotonic_and_bounded_by_leading_zeros(oracle):
    """Over all 2^23 values of the uniform grid: the noise does not decrease with the word, matches
    orc_gumbel, and stays below (clz(n) - 7) ln 2 + 0.001 with n = 2^23 - (x >> 9).  The GPU kernel
    discards tokens by that bound before it computes their noise, so the bound must hold for the
    noise as rounded, not only for the real-valued function."""
    k = np.arange(2 ** 23, dtype=np.uint32)
    g = oracle.gumbel_of_words(k << np.uint32(9))
    assert np.isfinite(g).all() and g[0] < -2.81 and 16.63 < g[-1] < 16.64
    assert (np.diff(g.astype(np.float64)) >= -2e-6).all()          # monotonic up to rounding
    n = (2 ** 23 - k.astype(np.int64))
    clz = 32 - np.floor(np.log2(n)).astype(np.int64) - 1
    assert clz.min() == 8 and clz.max() == 31
    ub = ((clz - 7).astype(np.float32) * np.float32(0.693147180559945309) + np.float32(1.0e-3)).astype(np.float32)
    assert (ub.astype(np.float64) >= g.astype(np.float64) + 5e-4).all()       # half the slack is still unused
    # the low nine bits of the word do not count
    assert np.array_equal(oracle.gumbel_of_words((k[::4097] << np.uint32(9)) | np.uint32(0x1FF)), g[::4097])
    ks = [0, 1, 12345, 2 ** 22, 2 ** 23 - 2, 2 ** 23 - 1]
    want = -np.log(-np.log((np.array(ks) + 0.5) * 2.0 ** -23))
    assert np.abs(g[ks] - want).max() < 4e-6


def test_top_k(oracle):
    """k = 1 is the greedy step; k at least the size of the allowed set changes nothing; the drawn
    tokens never fall below the cut, tokens tied with the k-th are kept, and among the kept tokens
    the law is the softmax (chi-square)."""
    n_tok = 40
    table = np.full((2, n_tok), DEAD, dtype=np.int32)
    allowed = [1, 4, 5, 9, 16, 22, 23, 30, 31, 39]
    table[1, allowed] = 0
    rng = np.random.default_rng(11)
    l = rng.normal(0, 1.0, n_tok).astype(np.float32)
    l[[0, 2, 3]] = 30.0                                               # masked out: must not count towards k
    l[[4, 22]] = 0.75                                                 # a tie inside the allowed set
    order = sorted(allowed, key=lambda t: (-l[t], t))
    B = 400
    logits = np.tile(l, (B, 1))
    states = np.ones(B, dtype=np.int32)
    g_tok, g_new = oracle.mask_step(table, logits, F32, states)
    tok, new = oracle.sample_step(table, logits, F32, states, 1.0, 3, 0, top_k=1)
    assert np.array_equal(tok, g_tok) and np.array_equal(new, g_new)
    a = oracle.sample_step(table, logits, F32, states, 1.0, 3, 0)
    for k in (len(allowed), len(allowed) + 5, 10 ** 6):
        b = oracle.sample_step(table, logits, F32, states, 1.0, 3, 0, top_k=k)
        assert np.array_equal(a[0], b[0])
    for k in range(1, len(allowed)):
        cut = l[order[k - 1]]
        kept = [t for t in allowed if l[t] >= cut]                    # ties with the k-th stay
        assert len(kept) >= k
        counts = np.zeros(n_tok, dtype=np.int64)
        for off in range(25):
            tok, _ = oracle.sample_step(table, logits, F32, states, 1.0, 17, off, top_k=k)
            counts += np.bincount(tok, minlength=n_tok)
        assert counts[[t for t in range(n_tok) if t not in kept]].sum() == 0
        if len(kept) > 1:
            p = np.exp(l[kept].astype(np.float64))
            p /= p.sum()
            assert stats.chisquare(counts[kept], p * counts.sum()).pvalue > 1e-4, (k, counts[kept])
    pos = {t: i for i, t in enumerate(order)}
    k_tie = max(pos[4], pos[22])                                      # k that ends between the two tied tokens
    tok, _ = oracle.sample_step(table, np.tile(l, (4000, 1)), F32, np.ones(4000, np.int32), 5.0, 1, 0, top_k=k_tie)
    assert {4, 22} <= set(tok.tolist())
    # NaN counts as -inf for the cut as well; an all -inf allowed set still yields its lowest id
    l2 = l.copy()
    l2[allowed] = np.nan
    l2[9] = -1.0
    tok, _ = oracle.sample_step(table, np.tile(l2, (8, 1)), F32, np.ones(8, np.int32), 1.0, 1, 0, top_k=3)
    assert (tok == 9).all()                                           # the other nine are -inf: probability zero
    l2[9] = np.nan
    tok, _ = oracle.sample_step(table, np.tile(l2, (8, 1)), F32, np.ones(8, np.int32), 1.0, 1, 0, top_k=3)
    assert (tok == 1).all()
    with pytest.raises(RuntimeError):
        oracle.sample_step(table, logits, F32, states, 1.0, 1, 0, top_k=-1)
