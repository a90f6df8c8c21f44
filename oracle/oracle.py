"""ctypes front end of the C oracle in tdfa_oracle.c (test infrastructure only).

Argument marshalling only: every computation is in the C file, whose header states
which passages of the paper each function follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

DEAD = -1
F32, BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tdfa_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "pda_oracle.c")]
# TDFA_ORACLE_SANITIZE=1 (set by tests/test_oracle_sanitized.py for a child process) selects a build
# with AddressSanitizer and UndefinedBehaviorSanitizer; the process must then have libasan preloaded.
_SANITIZE = os.environ.get("TDFA_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libtdfa_oracle_san.so" if _SANITIZE else "libtdfa_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        tmp = _LIB + f".{os.getpid()}.tmp"
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
            if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *opt, "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-Wall",
                               "-Wextra", "-o", tmp, *_SRCS, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _FstEdge(C.Structure):
    _fields_ = [("src", C.c_int32), ("in_", C.c_int32), ("out", C.c_int32), ("dst", C.c_int32)]


class _Fst(C.Structure):
    _fields_ = [("n_states", C.c_int32), ("root", C.c_int32), ("n_edges", C.c_int64),
                ("edges", C.POINTER(_FstEdge))]


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
        _lib.orc_fst_transduce.restype = C.c_int64
    return _lib


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _vocab_arrays(data, offsets):
    data = np.ascontiguousarray(data, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    return data, offsets


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def max_threads() -> int:
    return int(_load().orc_max_threads())


class DetokFST:
    """T_V of Algorithm 1 as an edge list: rows (src, in, out, dst), -1 = epsilon."""

    def __init__(self, data, offsets):
        lib = _load()
        self._data, self._off = _vocab_arrays(data, offsets)
        self._fst = _Fst()
        _check(lib.orc_build_detok_fst(_p(self._data), _p(self._off), C.c_int32(len(self._off) - 1),
                                       C.byref(self._fst)), "build_detok_fst")
        self.n_states = int(self._fst.n_states)
        self.root = int(self._fst.root)
        n = int(self._fst.n_edges)
        buf = np.ctypeslib.as_array(C.cast(self._fst.edges, C.POINTER(C.c_int32)), shape=(max(n, 1), 4))
        self.edges = buf[:n].copy()

    def __del__(self):
        try:
            _load().orc_fst_free(C.byref(self._fst))
        except Exception:
            pass


def build_detok_fst(data, offsets) -> DetokFST:
    return DetokFST(data, offsets)


def fst_transduce(fst: DetokFST, token_ids, out_cap: int = 4096) -> bytes | None:
    """Output of T_V on a token sequence; None if it is not accepted."""
    x = np.ascontiguousarray(token_ids, dtype=np.int32)
    out = np.zeros(out_cap + 1, dtype=np.uint8)
    n = int(_load().orc_fst_transduce(C.byref(fst._fst), _p(x), C.c_int32(len(x)), _p(out),
                                      C.c_int64(out_cap)))
    if n == -1:
        return None
    if n < 0:
        raise RuntimeError(f"oracle transduce failed with code {n}")
    return out[:n].tobytes()


def _compile(fn_name, trans, data, offsets, q_lo, q_hi, extra):
    lib = _load()
    trans = np.ascontiguousarray(trans, dtype=np.int32)
    n_states = trans.shape[0]
    data, offsets = _vocab_arrays(data, offsets)
    n_tokens = len(offsets) - 1
    q_lo = 0 if q_lo is None else q_lo
    q_hi = n_states if q_hi is None else q_hi
    out = np.empty((q_hi - q_lo, n_tokens), dtype=np.int32)
    rc = getattr(lib, fn_name)(_p(trans), C.c_int32(n_states), _p(data), _p(offsets),
                               C.c_int32(n_tokens), C.c_int32(q_lo), C.c_int32(q_hi), *extra, _p(out))
    _check(rc, fn_name)
    return out


def compile_compose(trans, data, offsets, q_lo=None, q_hi=None, block: int = 16,
                    n_threads: int = 1) -> np.ndarray:
    """delta_T rows [q_lo, q_hi) by explicit composition with T_V and epsilon removal."""
    return _compile("orc_compile_compose", trans, data, offsets, q_lo, q_hi,
                    (C.c_int32(block), C.c_int32(n_threads)))


def compile_walk(trans, data, offsets, q_lo=None, q_hi=None, n_threads: int = 1) -> np.ndarray:
    """delta_T rows [q_lo, q_hi) by the closed form delta*(q, d(t))."""
    return _compile("orc_compile_walk", trans, data, offsets, q_lo, q_hi, (C.c_int32(n_threads),))


def mask_step(table, logits, dtype: int, states, row_stride: int | None = None,
              want_masked: bool = False, n_threads: int = 1):
    """One decode step.  logits: float32 array (F32) or uint16 bit patterns (BF16), [batch, >=V]."""
    lib = _load()
    table = np.ascontiguousarray(table, dtype=np.int32)
    n_rows, n_tokens = table.shape
    logits = np.ascontiguousarray(logits, dtype=np.float32 if dtype == F32 else np.uint16)
    batch = logits.shape[0]
    stride = logits.shape[1] if row_stride is None else row_stride
    states = np.ascontiguousarray(states, dtype=np.int32)
    tokens = np.empty(batch, dtype=np.int32)
    new_states = np.empty(batch, dtype=np.int32)
    masked = np.array(logits, copy=True) if want_masked else None
    rc = lib.orc_mask_step(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), _p(logits), C.c_int(dtype),
                           C.c_int32(batch), C.c_int64(stride), _p(states), _p(tokens), _p(new_states),
                           _p(masked), C.c_int32(n_threads))
    _check(rc, "mask_step")
    return (tokens, new_states, masked) if want_masked else (tokens, new_states)


def philox4x32_10(ctr, key) -> np.ndarray:
    """One block of Philox4x32-10: ctr (4 words), key (2 words) -> 4 words."""
    lib = _load()
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib.orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def ln32(x) -> np.ndarray:
    """The binary32 logarithm the sampler is defined with, element by element."""
    lib = _load()
    lib.orc_ln32.restype = C.c_float
    x = np.asarray(x, dtype=np.float32)
    return np.array([lib.orc_ln32(C.c_float(float(v))) for v in x.ravel()], dtype=np.float32).reshape(x.shape)


def uniform(seed: int, offset: int, b: int, t: int) -> float:
    lib = _load()
    lib.orc_uniform.restype = C.c_float
    return float(lib.orc_uniform(C.c_uint64(seed), C.c_uint64(offset), C.c_int32(b), C.c_int32(t)))


def gumbel(seed: int, offset: int, b: int, t: int) -> float:
    lib = _load()
    lib.orc_gumbel.restype = C.c_float
    return float(lib.orc_gumbel(C.c_uint64(seed), C.c_uint64(offset), C.c_int32(b), C.c_int32(t)))


def gumbel_of_words(x) -> np.ndarray:
    """The noise as a function of the generator word (only its upper 23 bits count)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.uint32)
    out = np.empty(x.shape, dtype=np.float32)
    _check(lib.orc_gumbel_of_words(_p(x), C.c_int64(x.size), _p(out)), "gumbel_of_words")
    return out


def sample_noise(batch: int, n_tokens: int, seed: int, offset: int) -> np.ndarray:
    lib = _load()
    out = np.empty((batch, n_tokens), dtype=np.float32)
    _check(lib.orc_sample_noise(C.c_int32(batch), C.c_int32(n_tokens), C.c_uint64(seed), C.c_uint64(offset), _p(out)),
           "sample_noise")
    return out


def sample_step(table, logits, dtype: int, states, temperature: float, seed: int, offset: int,
                row_stride: int | None = None, want_masked: bool = False, n_threads: int = 1, top_k: int = 0):
    """One decode step with the token drawn from softmax(logits / temperature) over the allowed set
    (top_k > 0: over the allowed tokens whose logit reaches the k-th largest allowed logit)."""
    lib = _load()
    table = np.ascontiguousarray(table, dtype=np.int32)
    n_rows, n_tokens = table.shape
    logits = np.ascontiguousarray(logits, dtype=np.float32 if dtype == F32 else np.uint16)
    batch = logits.shape[0]
    stride = logits.shape[1] if row_stride is None else row_stride
    states = np.ascontiguousarray(states, dtype=np.int32)
    tokens = np.empty(batch, dtype=np.int32)
    new_states = np.empty(batch, dtype=np.int32)
    masked = np.array(logits, copy=True) if want_masked else None
    rc = lib.orc_sample_step(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), _p(logits), C.c_int(dtype),
                             C.c_int32(batch), C.c_int64(stride), _p(states), C.c_float(temperature),
                             C.c_int32(top_k), C.c_uint64(seed), C.c_uint64(offset), _p(tokens), _p(new_states), _p(masked),
                             C.c_int32(n_threads))
    _check(rc, "sample_step")
    return (tokens, new_states, masked) if want_masked else (tokens, new_states)


def advance_tokens(table, states, tokens):
    """Speculated runs: (history [batch, k + 1], n_valid [batch]) for tokens [batch, k]."""
    lib = _load()
    table = np.ascontiguousarray(table, dtype=np.int32)
    n_rows, n_tokens = table.shape
    states = np.ascontiguousarray(states, dtype=np.int32)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(states.shape[0], -1)
    batch, k = tokens.shape
    history = np.empty((batch, k + 1), dtype=np.int32)
    n_valid = np.empty(batch, dtype=np.int32)
    _check(lib.orc_advance_tokens(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), C.c_int32(batch), C.c_int32(k),
                                  _p(states), _p(tokens), _p(history), _p(n_valid)), "advance_tokens")
    return history, n_valid


def apply_terminals(table, edges, masks):
    """Terminal labels: a copy of `table` with the terminal edges [(state, label, target), ...]
    (in precedence order) applied; masks is [n_labels, n_tokens] of 0/1."""
    lib = _load()
    out = np.array(table, dtype=np.int32, copy=True, order="C")
    n_rows, n_tokens = out.shape
    ed = np.ascontiguousarray(edges, dtype=np.int32).reshape(-1, 3)
    st, lb, to = (np.ascontiguousarray(ed[:, i]) for i in range(3))
    masks = np.ascontiguousarray(masks, dtype=np.uint8).reshape(-1, n_tokens)
    _check(lib.orc_apply_terminals(_p(out), C.c_int64(n_rows), C.c_int32(n_tokens), C.c_int32(len(ed)), _p(st), _p(lb),
                                   _p(to), C.c_int32(masks.shape[0]), _p(masks)), "apply_terminals")
    return out


def minimize(table, accept, starts):
    """Token-level optimisation: (new table, new accept flags, map old state -> new state or DEAD)."""
    lib = _load()
    table = np.ascontiguousarray(table, dtype=np.int32)
    n_rows, n_tokens = table.shape
    accept = np.ascontiguousarray(accept, dtype=np.uint8)
    starts = np.ascontiguousarray(starts, dtype=np.int32).reshape(-1)
    out = np.empty((n_rows, n_tokens), dtype=np.int32)
    acc = np.empty(n_rows, dtype=np.uint8)
    mp = np.empty(n_rows, dtype=np.int32)
    n_new = C.c_int64()
    _check(lib.orc_minimize(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), _p(accept), _p(starts),
                            C.c_int32(len(starts)), _p(mp), C.byref(n_new), _p(out), _p(acc)), "minimize")
    k = n_new.value
    return out[:k].copy(), acc[:k].copy(), mp


def compact(table):
    """Edge-list form of a table: (row_begin [n_rows + 1] int64, targets [n_edges] int32)."""
    lib = _load()
    table = np.ascontiguousarray(table, dtype=np.int32)
    n_rows, n_tokens = table.shape
    row_begin = np.empty(n_rows + 1, dtype=np.int64)
    _check(lib.orc_compact(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), _p(row_begin), None), "compact")
    targets = np.empty(int(row_begin[-1]), dtype=np.int32)
    _check(lib.orc_compact(_p(table), C.c_int64(n_rows), C.c_int32(n_tokens), _p(row_begin), _p(targets)), "compact")
    return row_begin, targets


def expand(allowed, row_begin, targets) -> np.ndarray:
    """The dense table of an edge list; allowed: bool [n_rows, n_tokens]."""
    lib = _load()
    allowed = np.ascontiguousarray(allowed, dtype=np.uint8)
    n_rows, n_tokens = allowed.shape
    row_begin = np.ascontiguousarray(row_begin, dtype=np.int64)
    targets = np.ascontiguousarray(targets, dtype=np.int32)
    table = np.empty((n_rows, n_tokens), dtype=np.int32)
    _check(lib.orc_expand(_p(allowed), C.c_int64(n_rows), C.c_int32(n_tokens), _p(row_begin), _p(targets), _p(table)),
           "expand")
    return table


def concat_tables(tables: list[np.ndarray]):
    lib = _load()
    tabs = [np.ascontiguousarray(t, dtype=np.int32) for t in tables]
    n = len(tabs)
    n_tokens = tabs[0].shape[1]
    rows = np.array([t.shape[0] for t in tabs], dtype=np.int32)
    out = np.empty((int(rows.sum()), n_tokens), dtype=np.int32)
    offs = np.zeros(n + 1, dtype=np.int64)
    ptrs = (C.c_void_p * n)(*[t.ctypes.data for t in tabs])
    _check(lib.orc_concat_tables(ptrs, _p(rows), C.c_int32(n), C.c_int32(n_tokens), _p(out), _p(offs)),
           "concat_tables")
    return out, offs


# ---- push-down constraints (pda_oracle.c)

PDA_STR = 12


def _pda_args(pda):
    """pda: an object with n_states, src, input, dst, pop_begin, pop_syms, push_begin, push_syms (edges sorted by src)."""
    arrs = [np.ascontiguousarray(getattr(pda, k), dtype=np.int32) for k in
            ("src", "input", "dst", "pop_begin", "pop_syms", "push_begin", "push_syms")]
    return arrs, (C.c_int32(pda.n_states), C.c_int32(len(arrs[0])), *[_p(a) for a in arrs])


def pda_check_deterministic(pda) -> int:
    """0 if deterministic, else 1 + the index of the first edge that has a rival."""
    arrs, args = _pda_args(pda)
    return int(_load().orc_pda_check_deterministic(*args))


class TokenEdges:
    """Token edges of P_{G o V}: arrays src, token, dst, n_pops, pops [n, 12], n_push, pushes [n, 12] (unused -1)."""

    def __init__(self, src, token, dst, n_pops, pops, n_push, pushes):
        self.src, self.token, self.dst, self.n_pops, self.pops, self.n_push, self.pushes = src, token, dst, n_pops, pops, n_push, pushes

    def __len__(self):
        return len(self.src)

    def as_set(self):
        """{(src, token, pops tuple, dst, pushes tuple)}: what is unique about the result."""
        return {(int(self.src[i]), int(self.token[i]), tuple(self.pops[i, :self.n_pops[i]].tolist()), int(self.dst[i]),
                 tuple(self.pushes[i, :self.n_push[i]].tolist())) for i in range(len(self))}

    def edge_first(self, n_states: int) -> np.ndarray:
        first = np.zeros(n_states + 1, dtype=np.int64)
        np.add.at(first, self.src.astype(np.int64) + 1, 1)
        return np.cumsum(first)


def pda_compile(pda, data, offsets, q_lo=None, q_hi=None, cap: int = 1 << 22) -> TokenEdges:
    """Token edges of P_G o T_V leaving states [q_lo, q_hi), by explicit composition and removal of
    epsilon-input edges.  Raises RuntimeError (code -3) for a non-deterministic automaton."""
    lib = _load()
    arrs, args = _pda_args(pda)
    data, offsets = _vocab_arrays(data, offsets)
    q_lo = 0 if q_lo is None else q_lo
    q_hi = pda.n_states if q_hi is None else q_hi
    out = [np.empty(cap, dtype=np.int32) for _ in range(5)]
    pops = np.empty((cap, PDA_STR), dtype=np.int32)
    pushes = np.empty((cap, PDA_STR), dtype=np.int32)
    n = C.c_int64()
    rc = lib.orc_pda_compile(*args, _p(data), _p(offsets), C.c_int32(len(offsets) - 1), C.c_int32(q_lo), C.c_int32(q_hi),
                             C.c_int64(cap), _p(out[0]), _p(out[1]), _p(out[2]), _p(out[3]), _p(pops), _p(out[4]), _p(pushes),
                             C.byref(n))
    _check(rc, "pda_compile")
    k = n.value
    return TokenEdges(out[0][:k].copy(), out[1][:k].copy(), out[2][:k].copy(), out[3][:k].copy(), pops[:k].copy(),
                      out[4][:k].copy(), pushes[:k].copy())


def pda_accepting(pda, accept, q: int, stack) -> bool:
    lib = _load()
    arrs, args = _pda_args(pda)
    acc = np.ascontiguousarray(accept, dtype=np.uint8)
    st = np.ascontiguousarray(stack, dtype=np.int32)
    rc = lib.orc_pda_accepting(*args, _p(acc), C.c_int32(q), _p(st), C.c_int32(len(st)))
    if rc < 0:
        raise RuntimeError(f"oracle pda_accepting failed with code {rc}")
    return bool(rc)


def pda_step(n_states: int, n_tokens: int, edges: TokenEdges, logits, dtype: int, states, stacks, depths,
             row_stride: int | None = None, want_masked: bool = False):
    """One decode step of Algorithm 3.  edges sorted by src; stacks [batch, cap] and depths [batch] are updated in place.
    Returns (tokens, new_states[, masked])."""
    lib = _load()
    logits = np.ascontiguousarray(logits, dtype=np.float32 if dtype == F32 else np.uint16)
    batch = logits.shape[0]
    stride = logits.shape[1] if row_stride is None else row_stride
    states = np.ascontiguousarray(states, dtype=np.int32)
    assert stacks.dtype == np.int32 and depths.dtype == np.int32 and stacks.flags.c_contiguous and depths.flags.c_contiguous
    first = np.ascontiguousarray(edges.edge_first(n_states), dtype=np.int64)
    arr = [np.ascontiguousarray(a, dtype=np.int32) for a in (edges.token, edges.dst, edges.n_pops, edges.pops, edges.n_push, edges.pushes)]
    tokens = np.empty(batch, dtype=np.int32)
    new_states = np.empty(batch, dtype=np.int32)
    masked = np.array(logits, copy=True) if want_masked else None
    rc = lib.orc_pda_step(C.c_int32(n_states), C.c_int32(n_tokens), _p(first), *[_p(a) for a in arr], _p(logits), C.c_int(dtype),
                          C.c_int32(batch), C.c_int64(stride), _p(states), _p(stacks), _p(depths), C.c_int32(stacks.shape[1]),
                          _p(tokens), _p(new_states), _p(masked))
    _check(rc, "pda_step")
    return (tokens, new_states, masked) if want_masked else (tokens, new_states)


def pda_sample_step(n_states: int, n_tokens: int, edges: TokenEdges, logits, dtype: int, states, stacks, depths,
                    temperature: float, seed: int, offset: int, top_k: int = 0, row_stride: int | None = None,
                    want_masked: bool = False):
    """The step of Algorithm 3 with the token drawn from softmax(logits / temperature) over the allowed set (top_k as
    in sample_step).  Same arrays as pda_step; stacks and depths are updated in place."""
    lib = _load()
    logits = np.ascontiguousarray(logits, dtype=np.float32 if dtype == F32 else np.uint16)
    batch = logits.shape[0]
    stride = logits.shape[1] if row_stride is None else row_stride
    states = np.ascontiguousarray(states, dtype=np.int32)
    assert stacks.dtype == np.int32 and depths.dtype == np.int32 and stacks.flags.c_contiguous and depths.flags.c_contiguous
    first = np.ascontiguousarray(edges.edge_first(n_states), dtype=np.int64)
    arr = [np.ascontiguousarray(a, dtype=np.int32) for a in (edges.token, edges.dst, edges.n_pops, edges.pops, edges.n_push, edges.pushes)]
    tokens = np.empty(batch, dtype=np.int32)
    new_states = np.empty(batch, dtype=np.int32)
    masked = np.array(logits, copy=True) if want_masked else None
    rc = lib.orc_pda_sample_step(C.c_int32(n_states), C.c_int32(n_tokens), _p(first), *[_p(a) for a in arr], _p(logits),
                                 C.c_int(dtype), C.c_int32(batch), C.c_int64(stride), _p(states), _p(stacks), _p(depths),
                                 C.c_int32(stacks.shape[1]), C.c_float(temperature), C.c_int32(top_k), C.c_uint64(seed),
                                 C.c_uint64(offset), _p(tokens), _p(new_states), _p(masked))
    _check(rc, "pda_sample_step")
    return (tokens, new_states, masked) if want_masked else (tokens, new_states)
