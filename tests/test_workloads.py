"""Input tooling: regex compiler against Python's `re`, vocabulary recipes, logits definition."""
import re

import numpy as np
import pytest
import torch

from workloads import configs, logits as LG
from workloads.regex_dfa import compile_regex, regex_alphabet

PATTERNS = [
    r"a+|ab", r"(a|b)*abb", r"x{2,}y{0,2}z{3}", configs.C1_PATTERN, r"-?[0-9]{1,9}", r'"[^"\\]{0,32}"',
    # the constraint regexes printed in Appendix C.4 (multiple choice, ISO date-time, IPv4, quoted text)
    r"Red|Orange|Yellow|Green|Blue|Indigo|Violet",
    r"\d{4}-[01]\d-[0-3]\dT[0-2]\d:[0-5]\d:[0-5]\d([+-][0-2]\d:[0-5]\d|Z)",
    r"((25[0-5]|2[0-4]\d|[01]?\d\d?)\.){3}(25[0-5]|2[0-4]\d|[01]?\d\d?)",
    r'" *(?:[^\s"\\]|\\["n\\])(?: |[^\s"\\]|\\["n\\])*"',
]


@pytest.mark.parametrize("pattern", PATTERNS + [configs.c2_pattern(), configs.c5_pattern(3)])
def test_regex_compiler_matches_re(pattern):
    d = compile_regex(pattern)
    cre = re.compile(pattern.encode())
    rng = np.random.default_rng(len(pattern))
    alpha = np.nonzero((d.trans >= 0).any(axis=0))[0]
    members = 0
    for _ in range(600):
        q, s = d.start, bytearray()
        for _ in range(int(rng.integers(0, 60 + 8 * len(pattern)))):
            nxt = np.nonzero(d.trans[q] >= 0)[0]
            if len(nxt) == 0 or (d.accept[q] and rng.random() < 0.3):
                break
            b = int(rng.choice(nxt))
            s.append(b)
            q = int(d.trans[q, b])
        if s and rng.random() < 0.5:
            s[int(rng.integers(0, len(s)))] = int(rng.choice(np.concatenate([alpha, [0, 10, 255]])))
        s = bytes(s)
        m = cre.fullmatch(s) is not None
        assert m == d.accepts(s), s
        members += m
    assert members > 5
    # trim: every state reaches a final state; minimal: no two states are equivalent (spot check by signature)
    assert d.accept.any()
    sig = {(bool(d.accept[q]), tuple(d.trans[q].tolist())) for q in range(d.n_states)}
    assert len(sig) == d.n_states


def test_regex_alphabet():
    a = regex_alphabet(r'[a-c]+"[^"\\]*"\(x\)')
    assert bytes(a) == b'"()abcx'


def test_config_shapes():
    w1 = configs.get("c1")
    assert w1.vocab.n_tokens == 512 and w1.mask.batch == 4 and w1.mask.dtype == "f32" and w1.mask.steps == 16
    toks = w1.vocab.tokens()
    assert len(set(toks)) == 512 and sum(len(t) == 1 for t in toks) == 95
    assert all(2 <= len(t) <= 8 or len(t) == 1 for t in toks) and all(0x20 <= b < 0x7F for t in toks for b in t)
    w2 = configs.get("c2")
    assert w2.vocab.n_tokens == 32000 and 150 <= w2.dfas[0].n_states <= 450
    toks = w2.vocab.tokens()
    assert len(set(toks)) == 32000 and sum(len(t) == 1 for t in toks) == 256 and max(map(len, toks)) <= 16
    # ids are shuffled: single-byte tokens are not the first 256 ids
    assert sum(len(t) == 1 for t in toks[:256]) < 64
    # deterministic
    configs._MEMO.clear()
    assert configs.get("c2").vocab.tokens() == toks


def test_c4_statistics():
    """Random 20,000-state DFA with death probability 0.7; live fraction of entries is
    sum_L P(L) 0.3^L; mean lookups per entry is at most 1/0.7."""
    w = configs.get("c4")
    d = w.dfas[0]
    assert d.trans.shape == (20000, 256) and w.vocab.n_tokens == 256000
    assert abs((d.trans < 0).mean() - 0.7) < 0.005 and abs(d.accept.mean() - 0.1) < 0.01
    lens = np.diff(w.vocab.offsets.astype(np.int64))
    assert lens.min() >= 1 and lens.max() <= 32 and len(set(w.vocab.tokens())) == 256000
    assert (lens == 1).sum() == 256                          # length 1 saturates
    assert abs(np.bincount(w.vocab.data, minlength=256).std() / np.bincount(w.vocab.data).mean()) < 0.05


def test_logits_definition():
    x = LG.gen_logits(99, 3, 8, 50000, 2.0, "f32")
    assert abs(float(x.mean())) < 0.02 and abs(float(x.std()) - 2.0) < 0.02
    assert np.abs(x).max() <= 12.0
    # exact multiples of sigma / 65536
    assert np.array_equal(x * 32768.0, np.round(x * 32768.0))
    # counter-based: a row slice equals the same rows of the full draw; steps differ
    part = LG.gen_logits(99, 3, 8, 50000, 2.0, "f32", b_lo=5, b_hi=7)
    assert np.array_equal(part, x[5:7])
    assert not np.array_equal(LG.gen_logits(99, 4, 8, 50000, 2.0, "f32"), x)
    # bf16 rounding is round-to-nearest-even: same bits as torch's conversion
    b = LG.gen_logits(99, 3, 8, 50000, 2.0, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, ref)
    assert np.array_equal(LG.bf16_bits_to_f32(b), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    # near the maximum many values collide in bf16 (ties are routine)
    top = np.sort(LG.bf16_bits_to_f32(LG.gen_logits(1, 0, 1, 128256, 2.0, "bf16"))[0])[-64:]
    assert len(np.unique(top)) < 40


def test_splitmix_reference_values():
    """First outputs of splitmix64 seeded with 0 (published test vector of the generator)."""
    with np.errstate(over="ignore"):
        z = LG._mix(np.uint64(0) + np.arange(1, 4, dtype=np.uint64) * LG.GOLDEN)
    assert [hex(int(v)) for v in z] == ["0xe220a8397b1dcdaf", "0x6e789e6aa1b965f4", "0x6c45d188009454f"]
