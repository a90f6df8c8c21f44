"""The five seeded synthetic workloads (input tooling only; no method arithmetic).

They stand in for the paper's own workloads (a production LM vocabulary and the
constraint regexes of Appendix C.4), none of which is available offline:

  c1  tiny API-call regex, 512-token vocabulary, fp32 logits
  c2  JSON-schema-like object with five typed fields, 32,000 tokens
  c3  union of 50 function signatures, 128,256 tokens
  c4  random 20,000-state DFA, 256,000 tokens of uniform bytes (compile stress)
  c5  64 JSON-like constraints bound to 1,024 sequences, 128,256 tokens

Every draw comes from numpy generators seeded from MASTER_SEED + config number
with a separate sub-stream per purpose (regex, vocabulary, binding).
"""
from __future__ import annotations

import hashlib
import os
from dataclasses import dataclass, field

import numpy as np

from . import regex_dfa, vocab as V
from .regex_dfa import CharDFA

MASTER_SEED = 0x240708103

STREAM_REGEX, STREAM_VOCAB, STREAM_BIND, STREAM_LOGITS = 1, 2, 3, 4


def rng_for(config: int, stream: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng([MASTER_SEED + config, stream, extra])


def logits_seed(config: int) -> int:
    return (MASTER_SEED + config) * 0x9E3779B1 % (1 << 63)


@dataclass
class MaskWorkload:
    batch: int
    dtype: str          # "f32" | "bf16"
    sigma: float        # standard deviation of the logits
    steps: int


@dataclass
class Workload:
    name: str
    config: int
    dfas: list[CharDFA]              # one per constraint (c5 has 64)
    patterns: list[str | None]
    vocab: V.Vocab
    mask: MaskWorkload | None
    binding: np.ndarray | None = None  # c5: constraint index of each sequence
    notes: dict = field(default_factory=dict)


# --------------------------------------------------------------------------- DFA cache
_CACHE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), ".cache")


def _source_tag() -> str:
    with open(regex_dfa.__file__, "rb") as f:
        return hashlib.sha1(f.read()).hexdigest()[:12]


def cached_regex_dfa(pattern: str) -> CharDFA:
    """compile_regex with an on-disk cache keyed by the pattern and the compiler's source."""
    key = hashlib.sha1((_source_tag() + "\0" + pattern).encode("latin-1")).hexdigest()[:24]
    path = os.path.join(_CACHE_DIR, key + ".npz")
    if os.path.exists(path):
        try:
            z = np.load(path)
            return CharDFA(trans=z["trans"], accept=z["accept"], start=int(z["start"]))
        except Exception:
            pass
    dfa = regex_dfa.compile_regex(pattern)
    try:
        os.makedirs(_CACHE_DIR, exist_ok=True)
        tmp = path + f".{os.getpid()}.tmp.npz"
        np.savez_compressed(tmp, trans=dfa.trans, accept=dfa.accept, start=np.int64(dfa.start))
        os.replace(tmp, path)
    except OSError:
        pass
    return dfa


# --------------------------------------------------------------------------- regex recipes
WS = r"[ \n]*"
_WORDS = ["alpha", "bravo", "charlie", "delta", "echo", "foxtrot", "golf", "hotel", "india",
          "juliet", "kilo", "lima", "mike", "november", "oscar", "papa", "quebec", "romeo",
          "sierra", "tango", "uniform", "victor", "whiskey", "xray", "yankee", "zulu",
          "amber", "birch", "cedar", "dune", "ember", "fjord", "grove", "heath", "islet"]


def _value_regex(kind: str, rng: np.random.Generator | None, p: dict) -> str:
    if kind == "int":
        return r"-?[0-9]{1,%d}" % p.get("int_digits", 9)
    if kind == "string":
        return r'"[^"\\]{0,%d}"' % p.get("str_len", 32)
    if kind == "bool":
        return r"(true|false)"
    if kind == "enum":
        return '"(' + "|".join(p["enum_words"]) + ')"'
    if kind == "float":
        return r"-?[0-9]{1,%d}\.[0-9]{1,%d}([eE][+-]?[0-9]{1,2})?" % (p.get("int_digits", 9),
                                                                   p.get("frac_digits", 6))
    raise ValueError(kind)


def json_object_regex(keys: list[tuple[str, str]], p: dict) -> str:
    """Object with the given (key, type) fields in fixed order and optional whitespace."""
    parts = []
    for name, kind in keys:
        parts.append(WS + '"' + name + '"' + WS + ":" + WS + _value_regex(kind, None, p) + WS)
    return r"\{" + ",".join(parts) + r"\}"


def c2_pattern() -> str:
    keys = [("record_identifier", "int"), ("display_name", "string"), ("is_active", "bool"),
            ("category_label", "enum"), ("confidence_score", "float")]
    p = {"enum_words": ["pending_manual_review", "approved_automatically",
                        "rejected_by_policy_engine", "escalated_to_operator"]}
    return json_object_regex(keys, p)


def c5_pattern(i: int) -> str:
    """Seeded schema variation i: field count, order, names, bounds all vary."""
    rng = rng_for(5, STREAM_REGEX, i)
    n_keys = int(rng.integers(4, 11))
    kinds = ["int", "string", "bool", "enum", "float"]
    names = rng.choice(len(_WORDS), size=n_keys, replace=False)
    keys = []
    for j in range(n_keys):
        kind = kinds[int(rng.integers(0, 5))] if j >= 2 else ["int", "string"][j]
        suffix = "_" + _WORDS[int(rng.integers(0, len(_WORDS)))] if rng.random() < 0.5 else ""
        keys.append((_WORDS[int(names[j])] + suffix, kind))
    ew = rng.choice(len(_WORDS), size=4, replace=False)
    p = {"int_digits": int(rng.integers(1, 13)), "str_len": int(rng.choice([16, 32, 64, 96])),
         "frac_digits": int(rng.integers(1, 9)), "enum_words": [_WORDS[int(k)] for k in ew]}
    return json_object_regex(keys, p)


def _ident(rng: np.random.Generator, lo: int, hi: int) -> str:
    n = int(rng.integers(lo, hi + 1))
    return "".join(chr(0x61 + int(c)) for c in rng.integers(0, 26, size=n))


def c3_pattern() -> str:
    """Alternation of 50 seeded signatures name(arg1=VAL,...,argk=VAL), k in 1..6."""
    rng = rng_for(3, STREAM_REGEX)
    vals = [r"-?[0-9]{1,9}", r'"[^"\\]{0,32}"', r"[a-z_][a-z0-9_]{0,19}"]
    names: set[str] = set()
    sigs = []
    while len(sigs) < 50:
        name = _ident(rng, 4, 10)
        if name in names:
            continue
        names.add(name)
        k = int(rng.integers(1, 7))
        args = []
        for _ in range(k):
            args.append(_ident(rng, 3, 8) + "=" + vals[int(rng.integers(0, 3))])
        sigs.append(name + r"\(" + ",".join(args) + r"\)")
    return "|".join(sigs)


C1_PATTERN = r'[a-z]{1,8}\(x="[a-z]*"\)'


def _alphabet_of(patterns: list[str]) -> np.ndarray:
    """Regex alphabet: bytes the patterns name positively (a negated class such as the
    string body does not make every byte part of it)."""
    used = np.zeros(256, dtype=bool)
    for p in patterns:
        used[regex_dfa.regex_alphabet(p)] = True
    return np.nonzero(used)[0].astype(np.uint8)


def _mixed_vocab(config: int, n_tokens: int, max_len: int, zipf_a: float,
                 patterns: list[str]) -> V.Vocab:
    """256 single bytes + strings of length 2..max_len, Zipf lengths, 70 % regex alphabet."""
    rng = rng_for(config, STREAM_VOCAB)
    alpha = _alphabet_of(patterns)
    other = np.setdiff1d(V.PRINTABLE, alpha)
    ls, ps = V.zipf_lengths(2, max_len, zipf_a)
    return V.make_vocab(rng, n_tokens, np.arange(256, dtype=np.uint8), ls, ps, alpha, 0.7, other)


# --------------------------------------------------------------------------- the five configs
_MEMO: dict[str, Workload] = {}


def get(name: str) -> Workload:
    """Workload by name: 'c1' .. 'c5' (memoised per process)."""
    if name in _MEMO:
        return _MEMO[name]
    if name == "c1":
        dfa = cached_regex_dfa(C1_PATTERN)
        rng = rng_for(1, STREAM_VOCAB)
        ls = np.arange(2, 9)
        vocab = V.make_vocab(rng, 512, V.PRINTABLE, ls, np.full(len(ls), 1.0 / len(ls)),
                             V.PRINTABLE, 1.0, None)
        w = Workload("c1", 1, [dfa], [C1_PATTERN], vocab, MaskWorkload(4, "f32", 1.0, 16))
    elif name == "c2":
        pat = c2_pattern()
        dfa = cached_regex_dfa(pat)
        w = Workload("c2", 2, [dfa], [pat], _mixed_vocab(2, 32000, 16, 1.1, [pat]),
                     MaskWorkload(64, "bf16", 2.0, 256))
    elif name == "c3":
        pat = c3_pattern()
        dfa = cached_regex_dfa(pat)
        w = Workload("c3", 3, [dfa], [pat], _mixed_vocab(3, 128256, 24, 1.1, [pat]),
                     MaskWorkload(256, "bf16", 2.0, 512))
    elif name == "c4":
        dfa = regex_dfa.random_dfa(20000, 0.7, 0.1, rng_for(4, STREAM_REGEX))
        rng = rng_for(4, STREAM_VOCAB)
        ls, ps = V.zipf_lengths(1, 32, 1.05)
        vocab = V.make_vocab(rng, 256000, np.zeros(0, dtype=np.uint8), ls, ps,
                             np.arange(256, dtype=np.uint8), 1.0, None)
        w = Workload("c4", 4, [dfa], [None], vocab, None)
    elif name == "c5":
        pats = [c5_pattern(i) for i in range(64)]
        dfas = [cached_regex_dfa(p) for p in pats]
        vocab = _mixed_vocab(5, 128256, 24, 1.1, pats)
        binding = (np.arange(1024) % 64).astype(np.int32)
        w = Workload("c5", 5, dfas, pats, vocab, MaskWorkload(1024, "bf16", 2.0, 512),
                     binding=binding)
    else:
        raise KeyError(name)
    _MEMO[name] = w
    return w


def small(seed: int, n_states_hint: int = 12, n_tokens: int = 300, max_len: int = 6) -> Workload:
    """A small seeded workload for parity tests that span tiles and ragged tails."""
    rng = np.random.default_rng([MASTER_SEED, 99, seed])
    pats = [r"(ab|cd)*e{0,3}(f|gh)+", r'[a-d]{1,5}\(x="[a-c]*"\)', r"-?[0-9]{1,4}(\.[0-9]{1,3})?",
            r"(a|b|c|d|e|f|g|h){0,9}xyz"]
    pat = pats[seed % len(pats)]
    dfa = cached_regex_dfa(pat)
    alpha = _alphabet_of([pat])
    other = np.setdiff1d(V.PRINTABLE, alpha)
    ls, ps = V.zipf_lengths(1, max_len, 1.1)
    vocab = V.make_vocab(rng, n_tokens, alpha, ls, ps, alpha, 0.8, other)
    return Workload(f"small{seed}", 0, [dfa], [pat], vocab, MaskWorkload(5, "bf16", 2.0, 12))
