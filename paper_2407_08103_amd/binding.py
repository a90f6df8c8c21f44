"""Thin ctypes binding of the C ABI in include/tdfa.h.

Argument marshalling only: every step of the method runs in the library's HIP kernels.
PyTorch is used for device memory (torch.empty on "cuda") and for the current stream.
There is no CPU fallback: loading fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

DEAD = -1
NO_TOKEN = -1
F32, BF16 = 0, 1
PATH_AUTO, PATH_WALK, PATH_PAIRS, PATH_STAGED = 0, 1, 2, 3
OK = 0

_lib = None


class TdfaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"tdfa error {code}: {message}")
        self.code = code


def lib():
    """The loaded shared library (built on first use if no built copy exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = C.CDLL(_build.LIB)
        L.tdfa_last_error.restype = C.c_char_p
        L.tdfa_allow_row_words.restype = C.c_int64
        L.tdfa_allow_row_words.argtypes = [C.c_int32]
        L.tdfa_vocab_create.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tdfa_vocab_destroy.argtypes = [C.c_void_p]
        L.tdfa_vocab_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.tdfa_dfa_create.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tdfa_dfa_destroy.argtypes = [C.c_void_p]
        L.tdfa_dfa_union.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_dfa_union_host.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                          C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_plan_describe.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        L.tdfa_compile_token_dfa.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.POINTER(C.c_void_p)]
        L.tdfa_compile_token_dfa_at.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.POINTER(C.c_void_p)]
        L.tdfa_compile_stacked.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_table_concat.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_table_wrap.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_void_p)]
        L.tdfa_table_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_void_p),
                                      C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_table_destroy.argtypes = [C.c_void_p]
        L.tdfa_mask_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.tdfa_mask_step_noalloc.argtypes = L.tdfa_mask_step.argtypes
        L.tdfa_dfa_workspace_limit.argtypes = [C.c_void_p, C.c_int64]
        L.tdfa_dfa_compile_path.argtypes = [C.c_void_p, C.c_int]
        L.tdfa_dfa_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_int64)]
        L.tdfa_sample_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64, C.c_void_p, C.c_float,
                                       C.c_int32, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tdfa_sample_step_at.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64, C.c_void_p, C.c_float,
                                          C.c_int32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tdfa_table_pack.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tdfa_table_pack_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_void_p),
                                           C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
        L.tdfa_sample_noise.argtypes = [C.c_int32, C.c_int32, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p]
        L.tdfa_table_apply_terminals.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                 C.c_void_p, C.c_void_p]
        L.tdfa_table_minimize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p),
                                          C.c_void_p, C.c_void_p]
        L.tdfa_advance_tokens.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
        L.tdfa_pda_create.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tdfa_pda_destroy.argtypes = [C.c_void_p]
        L.tdfa_compile_token_pda.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tdfa_ptable_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int64)] + \
            [C.POINTER(C.c_void_p)] * 7
        L.tdfa_ptable_destroy.argtypes = [C.c_void_p]
        L.tdfa_pda_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tdfa_pda_sample_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int32, C.c_float, C.c_int32, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != OK:
        raise TdfaError(rc, lib().tdfa_last_error().decode("utf-8", "replace"))


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def allow_row_words(n_tokens: int) -> int:
    return int(lib().tdfa_allow_row_words(n_tokens))


def trim() -> None:
    """tdfa_trim: gives the workspace blocks kept from destroyed automata back to the device."""
    _check(lib().tdfa_trim())


def plan_describe(trans):
    """tdfa_plan_describe: (order, group_class, clean_sets [n_classes][8] uint32, jump [32][n_states] int32)."""
    tr = np.ascontiguousarray(trans, dtype=np.int32)
    n = tr.shape[0]
    cap = (n + 64 * 9 + 63) // 64 * 64
    order = np.empty(cap, dtype=np.int32)
    group_class = np.empty(cap // 64, dtype=np.int8)
    sets = np.zeros(64, dtype=np.uint32)
    jump = np.empty((32, n), dtype=np.int32)
    n_order, n_classes = C.c_int32(), C.c_int32()
    _check(lib().tdfa_plan_describe(tr.ctypes.data, n, order.ctypes.data, cap, C.byref(n_order), group_class.ctypes.data,
                                    sets.ctypes.data, jump.ctypes.data, C.byref(n_classes)))
    k = n_order.value
    return order[:k].copy(), group_class[:(k + 63) // 64].copy(), sets.reshape(8, 8)[:n_classes.value].copy(), jump


class Vocab:
    """tdfa_vocab handle."""

    def __init__(self, data, offsets, stream=None):
        data = np.ascontiguousarray(data, dtype=np.uint8)
        offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.n_tokens = len(offsets) - 1
        self._h = C.c_void_p()
        _check(lib().tdfa_vocab_create(data.ctypes.data, offsets.ctypes.data, self.n_tokens, _stream(stream),
                                       C.byref(self._h)))

    def info(self):
        n, nb, ml = C.c_int32(), C.c_int64(), C.c_int32()
        _check(lib().tdfa_vocab_info(self._h, C.byref(n), C.byref(nb), C.byref(ml)))
        return n.value, nb.value, ml.value

    def close(self):
        if self._h:
            lib().tdfa_vocab_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close


class CharDFA:
    """tdfa_dfa handle."""

    def __init__(self, trans, accept, start: int, stream=None):
        trans = np.ascontiguousarray(trans, dtype=np.int32)
        if trans.ndim != 2 or trans.shape[1] != 256:
            raise ValueError("trans must be [n_states, 256]")
        self.n_states = trans.shape[0]
        self.start = int(start)
        acc = None if accept is None else np.ascontiguousarray(accept, dtype=np.uint8)
        self._h = C.c_void_p()
        _check(lib().tdfa_dfa_create(trans.ctypes.data, None if acc is None else acc.ctypes.data, self.n_states,
                                     self.start, _stream(stream), C.byref(self._h)))

    def info(self):
        """tdfa_dfa_info: (n_states, start, compile path taken, pair-list workspace bytes or -1)."""
        n, st, pth, ws = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
        _check(lib().tdfa_dfa_info(self._h, C.byref(n), C.byref(st), C.byref(pth), C.byref(ws)))
        return n.value, st.value, pth.value, ws.value

    def compile_path(self, path: int) -> None:
        """tdfa_dfa_compile_path (PATH_AUTO, PATH_WALK, PATH_PAIRS, PATH_STAGED)."""
        _check(lib().tdfa_dfa_compile_path(self._h, int(path)))

    def workspace_limit(self, max_bytes: int) -> None:
        """tdfa_dfa_workspace_limit."""
        _check(lib().tdfa_dfa_workspace_limit(self._h, int(max_bytes)))

    def close(self):
        if self._h:
            lib().tdfa_dfa_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close


def dfa_union(dfas: list[CharDFA], stream=None):
    """tdfa_dfa_union: (CharDFA of the disjoint union, row offsets [n + 1])."""
    n = len(dfas)
    hs = (C.c_void_p * n)(*[d._h for d in dfas])
    offs = np.zeros(n + 1, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().tdfa_dfa_union(hs, n, _stream(stream), C.byref(h), offs.ctypes.data_as(C.POINTER(C.c_int64))))
    u = CharDFA.__new__(CharDFA)
    u._h = h
    u.n_states = int(offs[-1])
    u.start = dfas[0].start
    return u, offs


def dfa_union_host(automata, stream=None):
    """tdfa_dfa_union_host: `automata` is a list of (trans [n, 256] int32, accept [n] or None, start);
    returns (CharDFA of the disjoint union, row offsets [n + 1]) without uploading each automaton."""
    n = len(automata)
    tr = [np.ascontiguousarray(a[0], dtype=np.int32).reshape(-1, 256) for a in automata]
    ac = [None if a[1] is None else np.ascontiguousarray(a[1]).astype(np.uint8) for a in automata]
    tp = (C.c_void_p * n)(*[t.ctypes.data for t in tr])
    ap = (C.c_void_p * n)(*[None if a is None else a.ctypes.data for a in ac])
    ns = np.array([t.shape[0] for t in tr], dtype=np.int32)
    offs = np.zeros(n + 1, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().tdfa_dfa_union_host(tp, ap, ns.ctypes.data_as(C.c_void_p), n, int(automata[0][2]), _stream(stream), C.byref(h),
                                     offs.ctypes.data_as(C.POINTER(C.c_int64))))
    u = CharDFA.__new__(CharDFA)
    u._h = h
    u.n_states = int(offs[-1])
    u.start = int(automata[0][2])
    return u, offs


class Table:
    """tdfa_table handle.  `delta` / `allow` are torch views of the device buffers when the
    caller supplied them; otherwise the library owns the memory and device_ptrs() gives it."""

    def __init__(self, handle, keep=()):
        self._h = handle
        self._keep = keep          # tensors the table points into
        n_rows, n_tok, dp, ap, rw = C.c_int64(), C.c_int32(), C.c_void_p(), C.c_void_p(), C.c_int64()
        _check(lib().tdfa_table_info(self._h, C.byref(n_rows), C.byref(n_tok), C.byref(dp), C.byref(ap), C.byref(rw)))
        self.n_rows, self.n_tokens, self.row_words = n_rows.value, n_tok.value, rw.value
        self.delta_ptr, self.allow_ptr = dp.value, ap.value
        self.delta = keep[0] if keep else None
        self.allow = keep[1] if keep else None

    def close(self):
        if self._h:
            lib().tdfa_table_destroy(self._h)
            self._h = C.c_void_p()
            self._keep = ()

    __del__ = close


def _table_buffers(n_rows: int, n_tokens: int, device):
    delta = torch.empty((n_rows, n_tokens), dtype=torch.int32, device=device)
    allow = torch.empty((n_rows, allow_row_words(n_tokens)), dtype=torch.int32, device=device)
    return delta, allow


def compile_token_dfa(vocab: Vocab, dfa: CharDFA, stream=None, out=None, device="cuda", row_base: int = 0) -> Table:
    """tdfa_compile_token_dfa (row_base = 0) or tdfa_compile_token_dfa_at, into torch-owned buffers
    (out = (delta, allow) to reuse buffers or to write a slice of a stacked table)."""
    delta, allow = out if out is not None else _table_buffers(dfa.n_states, vocab.n_tokens, device)
    h = C.c_void_p()
    if row_base == 0:
        _check(lib().tdfa_compile_token_dfa(vocab._h, dfa._h, delta.data_ptr(), allow.data_ptr(), _stream(stream),
                                            C.byref(h)))
    else:
        _check(lib().tdfa_compile_token_dfa_at(vocab._h, dfa._h, row_base, delta.data_ptr(), allow.data_ptr(),
                                               _stream(stream), C.byref(h)))
    return Table(h, (delta, allow))


def compile_stacked(vocab: Vocab, dfas: list[CharDFA], stream=None, out=None, device="cuda"):
    """tdfa_compile_stacked: all constraints into one table whose states are global row ids.
    Returns (table, row_offsets as int64 numpy array)."""
    n = len(dfas)
    rows = sum(d.n_states for d in dfas)
    delta, allow = out if out is not None else _table_buffers(rows, vocab.n_tokens, device)
    arr = (C.c_void_p * n)(*[d._h for d in dfas])
    offs = np.zeros(n + 1, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().tdfa_compile_stacked(vocab._h, arr, n, delta.data_ptr(), allow.data_ptr(), _stream(stream), C.byref(h),
                                      offs.ctypes.data_as(C.POINTER(C.c_int64))))
    return Table(h, (delta, allow)), offs


def table_concat(tables: list[Table], stream=None, out=None, device="cuda"):
    """tdfa_table_concat; returns (table, row_offsets as int64 numpy array)."""
    n = len(tables)
    rows = sum(t.n_rows for t in tables)
    delta, allow = out if out is not None else _table_buffers(rows, tables[0].n_tokens, device)
    arr = (C.c_void_p * n)(*[t._h for t in tables])
    offs = np.zeros(n + 1, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().tdfa_table_concat(arr, n, delta.data_ptr(), allow.data_ptr(), _stream(stream), C.byref(h),
                                   offs.ctypes.data_as(C.POINTER(C.c_int64))))
    return Table(h, (delta, allow)), offs


def table_wrap(delta: torch.Tensor, allow: torch.Tensor) -> Table:
    h = C.c_void_p()
    _check(lib().tdfa_table_wrap(delta.data_ptr(), allow.data_ptr(), delta.shape[0], delta.shape[1], C.byref(h)))
    return Table(h, (delta, allow))


def _step_args(logits, states, tokens, new_states, masked_out):
    if logits.dtype == torch.float32:
        dtype = F32
    elif logits.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("logits must be float32 or bfloat16")
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [batch, n] with unit inner stride")
    if masked_out is not None and (masked_out.dtype != logits.dtype or masked_out.stride() != logits.stride()):
        raise ValueError("masked_out must have the dtype and strides of logits")
    for t in (states, tokens, new_states):
        if t.dtype != torch.int32 or not t.is_contiguous() or t.numel() < logits.shape[0]:
            raise ValueError("states, tokens, new_states must be contiguous int32 of length batch")
    return dtype


def mask_step(table: Table, logits: torch.Tensor, states: torch.Tensor, tokens: torch.Tensor,
              new_states: torch.Tensor, masked_out: torch.Tensor | None = None, stream=None) -> None:
    """tdfa_mask_step.  logits: [batch, >= n_tokens] float32 or bfloat16 on the GPU."""
    dtype = _step_args(logits, states, tokens, new_states, masked_out)
    _check(lib().tdfa_mask_step(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0),
                                states.data_ptr(), tokens.data_ptr(), new_states.data_ptr(),
                                None if masked_out is None else masked_out.data_ptr(), _stream(stream)))


def mask_step_noalloc(table: Table, logits: torch.Tensor, states: torch.Tensor, tokens: torch.Tensor,
                      new_states: torch.Tensor, masked_out: torch.Tensor | None = None, stream=None) -> None:
    """tdfa_mask_step_noalloc: the same step on the library's fixed scratch array (batch <= 4096)."""
    dtype = _step_args(logits, states, tokens, new_states, masked_out)
    _check(lib().tdfa_mask_step_noalloc(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0),
                                        states.data_ptr(), tokens.data_ptr(), new_states.data_ptr(),
                                        None if masked_out is None else masked_out.data_ptr(), _stream(stream)))


def sample_step(table: Table, logits: torch.Tensor, states: torch.Tensor, temperature: float, seed: int,
                offset: int, tokens: torch.Tensor, new_states: torch.Tensor,
                masked_out: torch.Tensor | None = None, stream=None, top_k: int = 0) -> None:
    """tdfa_sample_step.  Arguments as mask_step, plus the temperature, the generator's seed / offset
    and the top-k cut (0: none)."""
    dtype = _step_args(logits, states, tokens, new_states, masked_out)
    if isinstance(offset, torch.Tensor):
        # tdfa_sample_step_at: the offset is a one-element int64 tensor on the GPU, read when the step runs
        if offset.dtype != torch.int64 or offset.numel() != 1 or not offset.is_cuda:
            raise ValueError("a device offset must be a one-element int64 tensor on the GPU")
        _check(lib().tdfa_sample_step_at(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0),
                                         states.data_ptr(), float(temperature), int(top_k), int(seed) & (2 ** 64 - 1),
                                         offset.data_ptr(), tokens.data_ptr(), new_states.data_ptr(),
                                         None if masked_out is None else masked_out.data_ptr(), _stream(stream)))
        return
    _check(lib().tdfa_sample_step(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0),
                                  states.data_ptr(), float(temperature), int(top_k), int(seed) & (2 ** 64 - 1),
                                  int(offset) & (2 ** 64 - 1), tokens.data_ptr(), new_states.data_ptr(),
                                  None if masked_out is None else masked_out.data_ptr(), _stream(stream)))


def sample_noise(noise: torch.Tensor, seed: int, offset: int, stream=None) -> None:
    """tdfa_sample_noise.  noise: contiguous float32 [batch, n_tokens] on the GPU, written."""
    if noise.dtype != torch.float32 or noise.dim() != 2 or not noise.is_contiguous():
        raise ValueError("noise must be contiguous float32 [batch, n_tokens]")
    _check(lib().tdfa_sample_noise(noise.shape[0], noise.shape[1], int(seed) & (2 ** 64 - 1),
                                   int(offset) & (2 ** 64 - 1), noise.data_ptr(), _stream(stream)))


def advance_tokens(table: Table, states: torch.Tensor, tokens: torch.Tensor, history: torch.Tensor,
                   n_valid: torch.Tensor | None = None, stream=None) -> None:
    """tdfa_advance_tokens.  tokens: [batch, k] int32; history: [batch, k + 1] int32, written."""
    batch = states.numel()
    k = tokens.numel() // batch if batch else 0
    for t in (states, tokens, history) + (() if n_valid is None else (n_valid,)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError("states, tokens, history, n_valid must be contiguous int32")
    if tokens.numel() != batch * k or history.numel() != batch * (k + 1) or (n_valid is not None and n_valid.numel() != batch):
        raise ValueError("shapes: tokens [batch, k], history [batch, k + 1], n_valid [batch]")
    _check(lib().tdfa_advance_tokens(table._h, batch, k, states.data_ptr(), tokens.data_ptr(), history.data_ptr(),
                                     None if n_valid is None else n_valid.data_ptr(), _stream(stream)))


def table_apply_terminals(table: Table, edges, masks: torch.Tensor, stream=None) -> None:
    """tdfa_table_apply_terminals.  edges: [(state, label, target), ...] in precedence order;
    masks: int32 [n_labels, allow_row_words(n_tokens)] on the GPU, bit rows like the allowed bits."""
    ed = np.ascontiguousarray(edges, dtype=np.int32).reshape(-1, 3)
    st, lb, to = (np.ascontiguousarray(ed[:, i]) for i in range(3))
    if masks.dtype != torch.int32 or not masks.is_contiguous() or masks.dim() != 2:
        raise ValueError("masks must be contiguous int32 [n_labels, row_words]")
    _check(lib().tdfa_table_apply_terminals(table._h, len(ed), st.ctypes.data, lb.ctypes.data, to.ctypes.data,
                                            masks.shape[0], masks.data_ptr(), _stream(stream)))


def table_pack(table: Table, stream=None) -> Table:
    """tdfa_table_pack: the edge-list form of a dense table (library-owned; `delta` is None)."""
    h = C.c_void_p()
    _check(lib().tdfa_table_pack(table._h, _stream(stream), C.byref(h)))
    return Table(h)


_hip = None


def _copy_from_device(ptr: int, count: int, dtype: torch.dtype) -> torch.Tensor:
    """A torch tensor holding a copy of `count` elements at a device address the library owns."""
    global _hip
    out = torch.empty(count, dtype=dtype, device="cuda")
    if count:
        if _hip is None:
            _hip = C.CDLL("libamdhip64.so")
            _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        torch.cuda.synchronize()
        if _hip.hipMemcpy(out.data_ptr(), ptr, count * out.element_size(), 3) != 0:      # 3: device to device
            raise TdfaError(-3, "hipMemcpy from a library-owned array failed")
    return out


def table_pack_arrays(table: Table):
    """tdfa_table_pack_info, with the arrays copied into torch tensors: (targets int32 [n_edges],
    row_begin int64 [n_rows + 1], dir int32 bit patterns [n_rows, row_words / 4], allow int32 [n_rows, row_words])."""
    n_edges, tp, bp, dp, de = C.c_int64(), C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_int64()
    _check(lib().tdfa_table_pack_info(table._h, C.byref(n_edges), C.byref(tp), C.byref(bp), C.byref(dp), C.byref(de)))
    targets = _copy_from_device(tp.value, n_edges.value, torch.int32)
    row_begin = _copy_from_device(bp.value, table.n_rows + 1, torch.int64)
    dirs = _copy_from_device(dp.value, table.n_rows * de.value, torch.int32).view(table.n_rows, de.value)
    allow = _copy_from_device(table.allow_ptr, table.n_rows * table.row_words, torch.int32).view(table.n_rows, table.row_words)
    return targets, row_begin, dirs, allow


def table_minimize(table: Table, accept, starts, stream=None):
    """tdfa_table_minimize: (new Table, its accept flags, map old state -> new state or DEAD)."""
    acc = np.ascontiguousarray(accept, dtype=np.uint8)
    st = np.ascontiguousarray(starts, dtype=np.int32).reshape(-1)
    if len(acc) != table.n_rows:
        raise ValueError("accept must have one entry per row of the table")
    mp = np.empty(len(acc), dtype=np.int32)
    acc_out = np.empty(len(acc), dtype=np.uint8)
    h = C.c_void_p()
    _check(lib().tdfa_table_minimize(table._h, acc.ctypes.data, st.ctypes.data, len(st), _stream(stream), C.byref(h),
                                     mp.ctypes.data, acc_out.ctypes.data))
    new = Table(h)
    return new, acc_out[:new.n_rows].copy(), mp


PDA_STRING = 12


class CharPDA:
    """tdfa_pda handle.  Arguments: the arrays of tdfa_pda_create (edges sorted by source state)."""

    def __init__(self, n_states: int, start: int, accept, src, input, dst, pop_begin, pop_syms, push_begin, push_syms, stream=None):
        i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
        arrs = [i32(a) for a in (src, input, dst, pop_begin, pop_syms, push_begin, push_syms)]
        acc = None if accept is None else np.ascontiguousarray(accept, dtype=np.uint8)
        self.n_states = int(n_states)
        self.start = int(start)
        self._h = C.c_void_p()
        ptr = lambda a: a.ctypes.data if a.size else None
        _check(lib().tdfa_pda_create(self.n_states, self.start, None if acc is None else acc.ctypes.data, len(arrs[0]),
                                     ptr(arrs[0]), ptr(arrs[1]), ptr(arrs[2]), arrs[3].ctypes.data, ptr(arrs[4]),
                                     arrs[5].ctypes.data, ptr(arrs[6]), _stream(stream), C.byref(self._h)))

    def close(self):
        if self._h:
            lib().tdfa_pda_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close


class TokenPDA:
    """tdfa_ptable handle: the token edges of P_{G o V}, resident on the device."""

    def __init__(self, handle):
        self._h = handle
        n_states, n_tokens, n_edges = C.c_int32(), C.c_int32(), C.c_int64()
        ptrs = [C.c_void_p() for _ in range(7)]
        _check(lib().tdfa_ptable_info(self._h, C.byref(n_states), C.byref(n_tokens), C.byref(n_edges), *[C.byref(p) for p in ptrs]))
        self.n_states, self.n_tokens, self.n_edges = n_states.value, n_tokens.value, n_edges.value
        self._ptrs = [p.value for p in ptrs]

    def arrays(self):
        """Host copies: (edge_first, token, dst, n_pops, pops [n, 12], n_push, pushes [n, 12])."""
        n = self.n_edges

        def fetch(ptr, count, dtype):
            out = torch.empty(count, dtype=dtype, device="cuda")
            if count:
                _hip_copy(out.data_ptr(), ptr, out.numel() * out.element_size())
            return out.cpu().numpy()

        torch.cuda.synchronize()
        first = fetch(self._ptrs[0], self.n_states + 1, torch.int64)
        token, dst, n_pops = (fetch(self._ptrs[i], n, torch.int32) for i in (1, 2, 3))
        pops = fetch(self._ptrs[4], n * PDA_STRING, torch.int32).reshape(n, PDA_STRING)
        n_push = fetch(self._ptrs[5], n, torch.int32)
        pushes = fetch(self._ptrs[6], n * PDA_STRING, torch.int32).reshape(n, PDA_STRING)
        return first, token, dst, n_pops, pops, n_push, pushes

    def close(self):
        if self._h:
            lib().tdfa_ptable_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close


def _hip_copy(dst_ptr: int, src_ptr: int, n_bytes: int) -> None:
    """Device-to-device copy out of a library-owned array into a torch tensor."""
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    rc = hip.hipMemcpy(dst_ptr, src_ptr, n_bytes, 3)           # hipMemcpyDeviceToDevice
    if rc != 0:
        raise TdfaError(-3, f"hipMemcpy failed with {rc}")


def compile_token_pda(vocab: Vocab, pda: CharPDA, stream=None) -> TokenPDA:
    """tdfa_compile_token_pda."""
    h = C.c_void_p()
    _check(lib().tdfa_compile_token_pda(vocab._h, pda._h, _stream(stream), C.byref(h)))
    return TokenPDA(h)


def pda_step(table: TokenPDA, logits: torch.Tensor, states: torch.Tensor, stacks: torch.Tensor, depths: torch.Tensor,
             tokens: torch.Tensor, new_states: torch.Tensor, masked_out: torch.Tensor | None = None, stream=None) -> None:
    """tdfa_pda_step.  stacks: int32 [batch, stack_cap], depths: int32 [batch], both updated in place."""
    dtype = _step_args(logits, states, tokens, new_states, masked_out)
    assert stacks.dtype == torch.int32 and depths.dtype == torch.int32 and stacks.is_contiguous() and depths.is_contiguous()
    _check(lib().tdfa_pda_step(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0), states.data_ptr(),
                               stacks.data_ptr(), depths.data_ptr(), stacks.shape[1], tokens.data_ptr(), new_states.data_ptr(),
                               None if masked_out is None else masked_out.data_ptr(), _stream(stream)))


def pda_sample_step(table: TokenPDA, logits: torch.Tensor, states: torch.Tensor, stacks: torch.Tensor, depths: torch.Tensor,
                    temperature: float, seed: int, offset: int, tokens: torch.Tensor, new_states: torch.Tensor,
                    masked_out: torch.Tensor | None = None, stream=None, top_k: int = 0) -> None:
    """tdfa_pda_sample_step: pda_step with the token drawn at a temperature (seed, offset, top_k as sample_step)."""
    dtype = _step_args(logits, states, tokens, new_states, masked_out)
    assert stacks.dtype == torch.int32 and depths.dtype == torch.int32 and stacks.is_contiguous() and depths.is_contiguous()
    _check(lib().tdfa_pda_sample_step(table._h, logits.data_ptr(), dtype, logits.shape[0], logits.stride(0), states.data_ptr(),
                                      stacks.data_ptr(), depths.data_ptr(), stacks.shape[1], float(temperature), int(top_k),
                                      int(seed) & (2 ** 64 - 1), int(offset) & (2 ** 64 - 1), tokens.data_ptr(),
                                      new_states.data_ptr(), None if masked_out is None else masked_out.data_ptr(),
                                      _stream(stream)))
