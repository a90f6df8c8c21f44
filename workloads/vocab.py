"""Seeded synthetic token vocabularies (input tooling only; no method arithmetic).

A vocabulary is a pair (bytes, offsets): token t detokenizes to
bytes[offsets[t]:offsets[t+1]] (the d(v) of Appendix B.1).  Tokens are distinct
byte strings and token ids are a seeded shuffle of the generation order, so
id order is unrelated to lexicographic order (as in real tokenizers).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Vocab:
    data: np.ndarray      # uint8 [total_bytes]
    offsets: np.ndarray   # uint64 [n_tokens + 1]

    @property
    def n_tokens(self) -> int:
        return int(self.offsets.shape[0] - 1)

    def token(self, t: int) -> bytes:
        return self.data[int(self.offsets[t]):int(self.offsets[t + 1])].tobytes()

    def tokens(self) -> list[bytes]:
        o = self.offsets.astype(np.int64)
        raw = self.data.tobytes()
        return [raw[o[i]:o[i + 1]] for i in range(self.n_tokens)]


def from_tokens(tokens: list[bytes]) -> Vocab:
    lens = np.fromiter((len(t) for t in tokens), dtype=np.uint64, count=len(tokens))
    offsets = np.zeros(len(tokens) + 1, dtype=np.uint64)
    np.cumsum(lens, out=offsets[1:])
    data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy()
    return Vocab(data=data, offsets=offsets)


PRINTABLE = np.arange(0x20, 0x7F, dtype=np.uint8)       # the 95 printable ASCII bytes


def zipf_lengths(lo: int, hi: int, a: float) -> tuple[np.ndarray, np.ndarray]:
    """Rank-based Zipf over lengths lo..hi: P(L) proportional to (L - lo + 1)^(-a)."""
    ls = np.arange(lo, hi + 1)
    w = (ls - lo + 1.0) ** (-a)
    return ls, w / w.sum()


def make_vocab(rng: np.random.Generator, n_tokens: int, singles: np.ndarray,
               len_values: np.ndarray, len_probs: np.ndarray,
               alphabet_a: np.ndarray, p_a: float, alphabet_b: np.ndarray | None) -> Vocab:
    """`singles` as one-byte tokens, then distinct random strings up to n_tokens in total.

    Each string draws a length from (len_values, len_probs) and each of its bytes
    independently: with probability p_a uniform from alphabet_a, else uniform from
    alphabet_b.  A string that collides with an earlier token is dropped and both its
    length and bytes are drawn again.  Ids are shuffled at the end.
    """
    toks: list[bytes] = [bytes([int(b)]) for b in singles]
    seen = set(toks)
    need = n_tokens - len(toks)
    maxlen = int(len_values.max())
    while need > 0:
        m = int(need * 1.3) + 64
        lens = rng.choice(len_values, size=m, p=len_probs)
        pick_a = rng.random((m, maxlen)) < p_a
        ia = rng.integers(0, len(alphabet_a), size=(m, maxlen))
        mat = alphabet_a[ia]
        if alphabet_b is not None and len(alphabet_b):
            ib = rng.integers(0, len(alphabet_b), size=(m, maxlen))
            mat = np.where(pick_a, mat, alphabet_b[ib])
        mat = mat.astype(np.uint8)
        for i in range(m):
            s = mat[i, :lens[i]].tobytes()
            if s in seen:
                continue
            seen.add(s)
            toks.append(s)
            need -= 1
            if need == 0:
                break
    perm = rng.permutation(len(toks))
    return from_tokens([toks[i] for i in perm])
