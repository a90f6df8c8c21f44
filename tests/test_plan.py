"""Host logic of the compile stage: the lane order and the default-chain jump tables that
tdfa_plan_describe reports are checked against their definition by walking the automaton byte by
byte (no GPU: the call is host only)."""
import numpy as np
import pytest

from workloads import configs
from workloads.regex_dfa import compile_regex, random_dfa


@pytest.fixture(scope="module")
def T():
    import paper_2407_08103_amd as T
    return T


def _walk(trans, q, data):
    for b in data:
        if q < 0:
            return -1
        q = int(trans[q, b])
    return q


def _check_plan(T, trans, rng, expect_classes=None):
    n = trans.shape[0]
    order, group_class, sets, jump = T.plan_describe(trans)
    # order: every state exactly once, idle lanes only as padding, whole groups per class
    states = order[order >= 0]
    assert np.array_equal(np.sort(states), np.arange(n))
    assert len(group_class) == (len(order) + 63) // 64
    n_classes = len(sets)
    if expect_classes is not None:
        assert n_classes == expect_classes
    seen = -1
    for g, c in enumerate(group_class):
        assert -1 <= c < n_classes
        if c >= 0:
            assert c >= seen, "groups of a class are contiguous, classes in order"
            seen = c
        else:
            seen = n_classes                       # after the classes only plain groups
    in_class = np.full(n, -1)
    for g, c in enumerate(group_class):
        for q in order[g * 64:(g + 1) * 64]:
            if q >= 0:
                in_class[q] = c
        if c >= 0:
            assert len(order) >= (g + 1) * 64      # a class group is always a whole group
    # jump tables against the definition: any string of m clean bytes takes q to jump[m-1][q]
    for c in range(n_classes):
        clean = [b for b in range(256) if (int(sets[c][b >> 5]) >> (b & 31)) & 1]
        assert len(clean) >= 2
        members = np.nonzero(in_class == c)[0]
        assert len(members) >= 24
        for q in rng.choice(members, size=min(len(members), 40), replace=False):
            assert all(trans[q, b] == trans[q, clean[0]] for b in clean), "clean bytes share one target"
            for m in (1, 2, 3, 7, 16, 31, 32):
                for _ in range(3):
                    s = rng.choice(clean, size=m)
                    assert _walk(trans, int(q), s) == jump[m - 1, q], (c, q, m)
    assert (jump[:, in_class < 0] == -1).all()
    return n_classes, in_class


@pytest.mark.parametrize("pattern,n_classes", [
    (r'"[^"\\]{0,40}"', 1),
    (r'[a-c_][a-c0-2_]{0,45}=[0-2]{1,40};', 2),
    (r'[ab]{70}[bc]{70}d', 2),
    (r'([ab]{26}[cd]{26}[ef]{26}[gh]{26}[ij]{26}[kl]{26}[mn]{26}[op]{26}[qr]{26}[st]{26})?u', 8),
    (r'(foo)+d', 0),
])
def test_plan_of_counters(T, pattern, n_classes):
    d = compile_regex(pattern)
    _check_plan(T, d.trans, np.random.default_rng(1), expect_classes=n_classes)


def test_plan_partial_chain(T):
    """[ab]{70}[bc]{70}d: a state of the first counter jumps only if 32 more clean bytes keep it
    inside that counter; the others are left to the byte-by-byte walk."""
    d = compile_regex(r'[ab]{70}[bc]{70}d')
    n_classes, in_class = _check_plan(T, d.trans, np.random.default_rng(2), expect_classes=2)
    # walk the first counter: state after k bytes 'a'
    q, chain = d.start, []
    for _ in range(70):
        chain.append(q)
        q = int(d.trans[q, ord("a")])
    first = [in_class[s] for s in chain]
    assert all(c >= 0 for c in first[:38]) and all(c < 0 for c in first[39:])


def test_plan_random_and_configs(T):
    rng = np.random.default_rng(3)
    assert _check_plan(T, random_dfa(300, 0.5, 0.2, rng).trans, rng)[0] == 0
    for name in ("c1", "c2", "c3"):
        w = configs.get(name)
        k, _ = _check_plan(T, w.dfas[0].trans, rng)
        assert k >= 1 or name == "c1"
    w = configs.get("c5")
    for d in w.dfas[:6]:
        _check_plan(T, d.trans, rng)


def test_plan_bad_arguments(T):
    with pytest.raises(T.TdfaError):
        T.plan_describe(np.full((2, 256), 9, dtype=np.int32))
