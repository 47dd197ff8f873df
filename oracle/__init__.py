"""ctypes binding of the CPU oracle (oracle/pre3_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU-baseline leg
import this package.  It shares nothing with the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pre3_oracle.c")
_LIB = os.path.join(_HERE, "libpre3_oracle.so")

A_ERROR, A_SHIFT, A_REDUCE, A_ACCEPT = 0, 1, 2, 3
T_END = 256


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C + OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    vp, i32, i64 = c.c_void_p, c.c_int, c.c_int64
    lib.pre3o_build.restype = vp
    lib.pre3o_build.argtypes = [c.POINTER(c.c_char_p), i32, c.c_char_p, i32]
    lib.pre3o_free.argtypes = [vp]
    for name, args in [
        ("pre3o_n_grammars", [vp]),
        ("pre3o_n_states", [vp, i32]),
        ("pre3o_n_states_total", [vp]),
        ("pre3o_n_productions", [vp, i32]),
        ("pre3o_n_nonterminals", [vp, i32]),
        ("pre3o_initial_state", [vp, i32]),
        ("pre3o_n_items", [vp, i32, i32]),
        ("pre3o_production_lhs", [vp, i32, i32]),
        ("pre3o_production_len", [vp, i32, i32]),
        ("pre3o_action", [vp, i32, i32, i32, c.POINTER(i32)]),
        ("pre3o_goto", [vp, i32, i32, i32]),
        ("pre3o_allowed", [vp, vp, i32, vp, i32]),
        ("pre3o_eos_allowed", [vp, vp, i32]),
        ("pre3o_advance", [vp, vp, vp, i32, vp, i32]),
        ("pre3o_n_cycles", [vp, i32]),
        ("pre3o_cycle", [vp, i32, i32, vp]),
        ("pre3o_compact", [vp, vp, i32]),
    ]:
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = args
    lib.pre3o_nonterminal_name.restype = c.c_char_p
    lib.pre3o_nonterminal_name.argtypes = [vp, i32, i32]
    lib.pre3o_mask_row.restype = None
    lib.pre3o_mask_row.argtypes = [vp, vp, i32, i32, vp, vp, i32, i32, vp]
    lib.pre3o_fill_mask.restype = None
    lib.pre3o_fill_mask.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, i32, i32, vp]
    lib.pre3o_allowed_many.restype = None
    lib.pre3o_allowed_many.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp]
    lib.pre3o_apply_mask.restype = None
    lib.pre3o_apply_mask.argtypes = [vp, vp, i32, i32, i64]
    lib.pre3o_masked_argmax.restype = None
    lib.pre3o_masked_argmax.argtypes = [vp, vp, i32, i32, i64, vp]
    lib.pre3o_masked_topk.restype = None
    lib.pre3o_masked_topk.argtypes = [vp, vp, i32, i32, i64, i32, vp, vp]
    lib.pre3o_jump_forward.restype = i32
    lib.pre3o_jump_forward.argtypes = [vp, vp, vp, i32, i32, vp]
    lib.pre3o_jump_forward_batch.restype = None
    lib.pre3o_jump_forward_batch.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.pre3o_compact_batch.restype = None
    lib.pre3o_compact_batch.argtypes = [vp, vp, vp, i32, i32]
    lib.pre3o_advance_batch.restype = None
    lib.pre3o_advance_batch.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp]
    _lib = lib
    return lib


class GrammarError(ValueError):
    pass


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


class Oracle:
    """Canonical LR(1) tables of one or several grammars (disjoint union of state ids)."""

    def __init__(self, grammars, compact_cycles: bool = False):
        """compact_cycles: every advance (single, batched, jump-forward) is followed by the
        compaction of Sec. 3.2.3 (`compact`), as a library compiled with that option does."""
        if isinstance(grammars, str):
            grammars = [grammars]
        self.compact_cycles = bool(compact_cycles)
        lib = _load()
        arr = (ctypes.c_char_p * len(grammars))(*[g.encode("latin-1") for g in grammars])
        err = ctypes.create_string_buffer(512)
        self._h = lib.pre3o_build(arr, len(grammars), err, 512)
        if not self._h:
            raise GrammarError(err.value.decode())
        self._lib = lib
        self.n_grammars = len(grammars)

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.pre3o_free(self._h)
            self._h = None

    # ---- table queries (local state ids of grammar g)
    def n_states(self, g=0):
        return self._lib.pre3o_n_states(self._h, g)

    def n_states_total(self):
        return self._lib.pre3o_n_states_total(self._h)

    def n_productions(self, g=0):
        return self._lib.pre3o_n_productions(self._h, g)

    def n_nonterminals(self, g=0):
        return self._lib.pre3o_n_nonterminals(self._h, g)

    def initial_state(self, g=0):
        return self._lib.pre3o_initial_state(self._h, g)

    def n_items(self, s, g=0):
        return self._lib.pre3o_n_items(self._h, g, s)

    def production(self, p, g=0):
        """(lhs name, rhs length) of production p (production 0 is the augmented one)."""
        a = self._lib.pre3o_production_lhs(self._h, g, p)
        return self._lib.pre3o_nonterminal_name(self._h, g, a).decode(), self._lib.pre3o_production_len(self._h, g, p)

    def nonterminal_index(self, name, g=0):
        for a in range(self.n_nonterminals(g)):
            if self._lib.pre3o_nonterminal_name(self._h, g, a).decode() == name:
                return a
        raise KeyError(name)

    def action(self, s, a, g=0):
        arg = ctypes.c_int(0)
        kind = self._lib.pre3o_action(self._h, g, s, a, ctypes.byref(arg))
        return kind, arg.value

    def goto(self, s, A, g=0):
        return self._lib.pre3o_goto(self._h, g, s, A)

    # ---- per-stack queries (global state ids)
    def initial_stack(self, g=0):
        return [self.initial_state(g)]

    def allowed(self, stack, data: bytes) -> bool:
        st = np.asarray(stack, dtype=np.int32)
        buf = np.frombuffer(bytes(data) + b"\0", dtype=np.uint8)
        return bool(self._lib.pre3o_allowed(self._h, _ptr(st), len(st), _ptr(buf), len(data)))

    def eos_allowed(self, stack) -> bool:
        st = np.asarray(stack, dtype=np.int32)
        return bool(self._lib.pre3o_eos_allowed(self._h, _ptr(st), len(st)))

    def advance(self, stack, data: bytes, cap: int = 1 << 20):
        """Returns (rc, new stack list); rc 0 ok, 1 not allowed, 2 overflow of `cap`."""
        n = len(stack)
        cap = int(min(cap, n + 8 * len(data) + 64))
        st = np.zeros(cap, dtype=np.int32)
        st[:n] = stack
        ln = np.array([n], dtype=np.int32)
        buf = np.frombuffer(bytes(data) + b"\0", dtype=np.uint8)
        rc = self._lib.pre3o_advance(self._h, _ptr(st), _ptr(ln), cap, _ptr(buf), len(data))
        if rc == 0 and self.compact_cycles:
            ln[0] = self._lib.pre3o_compact(self._h, _ptr(st), int(ln[0]))
        return rc, st[: ln[0]].tolist()

    def jump_forward(self, stack, max_bytes: int = 64, cap: int = 1 << 20):
        """(forced bytes, advanced stack): the bytes every continuation must start with."""
        n = len(stack)
        cap = int(min(cap, n + 8 * max_bytes + 64))
        st = np.zeros(cap, dtype=np.int32)
        st[:n] = stack
        ln = np.array([n], dtype=np.int32)
        out = np.zeros(max(1, max_bytes), dtype=np.uint8)
        k = self._lib.pre3o_jump_forward(self._h, _ptr(st), _ptr(ln), cap, int(max_bytes), _ptr(out))
        if self.compact_cycles:
            ln[0] = self._lib.pre3o_compact(self._h, _ptr(st), int(ln[0]))
        return out[:k].tobytes(), st[: ln[0]].tolist()

    def jump_forward_batch(self, states, data, length, max_bytes: int):
        """In place on states/data/length (as advance_batch); returns (bytes [B, max_bytes] u8, counts [B])."""
        B, cap = data.shape
        assert data.flags.c_contiguous and data.dtype == np.int32 and length.dtype == np.int32 and states.dtype == np.int32
        out = np.zeros((B, max(1, max_bytes)), dtype=np.uint8)
        cnt = np.zeros(B, dtype=np.int32)
        self._lib.pre3o_jump_forward_batch(self._h, _ptr(states), _ptr(data), _ptr(length), cap, B, int(max_bytes),
                                           _ptr(out), _ptr(cnt))
        if self.compact_cycles:
            self.compact_batch(data, length)
        return out[:, :max_bytes], cnt

    def cycles(self, g=0):
        """Reduction cycles of grammar g (Sec. 3.2.3), each a list of GLOBAL state ids v1..vn."""
        out, buf = [], np.zeros(64, dtype=np.int32)
        off = self.initial_state(g)
        for k in range(self._lib.pre3o_n_cycles(self._h, g)):
            n = self._lib.pre3o_cycle(self._h, g, k, _ptr(buf))
            out.append((buf[:n] + off).tolist())
        return out

    def compact(self, stack):
        """The stack without the complete cycle traversals it need not keep (Alg. 1 step 1)."""
        st = np.array(stack, dtype=np.int32)
        n = self._lib.pre3o_compact(self._h, _ptr(st), len(st))
        return st[:n].tolist()

    def compact_batch(self, data, length):
        """In place on data/length: every stack of the batch in normal form."""
        B, cap = data.shape
        assert data.flags.c_contiguous and data.dtype == np.int32 and length.dtype == np.int32
        self._lib.pre3o_compact_batch(self._h, _ptr(data), _ptr(length), cap, B)

    def accepts(self, text: bytes, g=0) -> bool:
        """Is `text` a sentence of grammar g?"""
        st = self.initial_stack(g)
        if len(text):
            rc, st = self.advance(st, text)
            if rc != 0:
                return False
        return self.eos_allowed(st)

    def mask_row(self, stack, vocab, done: bool = False) -> np.ndarray:
        st = np.asarray(stack, dtype=np.int32)
        row = np.zeros(vocab.words, dtype=np.uint32)
        self._lib.pre3o_mask_row(self._h, _ptr(st), len(st), int(done), _ptr(vocab.bytes),
                                 _ptr(vocab.offsets), vocab.n_tokens, vocab.eos_id, _ptr(row))
        return row

    def allowed_many(self, stack, vocab, ids) -> np.ndarray:
        st = np.asarray(stack, dtype=np.int32)
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        out = np.zeros(len(ids), dtype=np.uint8)
        self._lib.pre3o_allowed_many(self._h, _ptr(st), len(st), _ptr(vocab.bytes),
                                     _ptr(vocab.offsets), _ptr(ids), len(ids), _ptr(out))
        return out.astype(bool)

    # ---- batched calls mirroring the device entry points
    def fill_mask(self, states, data, length, vocab) -> np.ndarray:
        states = np.ascontiguousarray(states, dtype=np.int32)
        data = np.ascontiguousarray(data, dtype=np.int32)
        length = np.ascontiguousarray(length, dtype=np.int32)
        batch, cap = data.shape
        out = np.zeros((batch, vocab.words), dtype=np.uint32)
        self._lib.pre3o_fill_mask(self._h, _ptr(states), _ptr(data), _ptr(length), cap, batch,
                                  _ptr(vocab.bytes), _ptr(vocab.offsets), vocab.n_tokens,
                                  vocab.eos_id, _ptr(out))
        return out

    def advance_batch(self, states, data, length, tokens, vocab) -> np.ndarray:
        """Mutates states, data, length in place; returns err[B]."""
        for a in (states, data, length):
            assert a.dtype == np.int32 and a.flags.c_contiguous
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        batch, cap = data.shape
        err = np.zeros(batch, dtype=np.int32)
        self._lib.pre3o_advance_batch(self._h, _ptr(states), _ptr(data), _ptr(length), cap, batch,
                                      _ptr(tokens), _ptr(vocab.bytes), _ptr(vocab.offsets),
                                      vocab.n_tokens, vocab.eos_id, _ptr(err))
        if self.compact_cycles:
            self.compact_batch(data, length)
        return err


def apply_mask(logits_u16: np.ndarray, bitmask: np.ndarray, n_tokens: int) -> None:
    """bf16 select on raw bit patterns, in place: masked entries become 0xFF80 (-inf)."""
    assert logits_u16.dtype == np.uint16 and logits_u16.flags.c_contiguous and logits_u16.ndim == 2
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    _load().pre3o_apply_mask(_ptr(logits_u16), _ptr(bm), bm.shape[0], int(n_tokens), logits_u16.shape[1])


def masked_argmax(logits_u16: np.ndarray, bitmask: np.ndarray, n_tokens: int) -> np.ndarray:
    """Greedy choice per row: id of the largest allowed, non-NaN bf16 logit (first of equals), -1 if none."""
    assert logits_u16.dtype == np.uint16 and logits_u16.flags.c_contiguous and logits_u16.ndim == 2
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    out = np.empty(bm.shape[0], dtype=np.int32)
    _load().pre3o_masked_argmax(_ptr(logits_u16), _ptr(bm), bm.shape[0], int(n_tokens), logits_u16.shape[1], _ptr(out))
    return out


def masked_topk(logits_u16: np.ndarray, bitmask: np.ndarray, n_tokens: int, k: int):
    """Per row the k largest allowed, non-NaN bf16 logits, largest first, equal values by ascending
    id: (ids [B, k] int32, padded with -1; bf16 patterns [B, k] uint16, padded with 0xFF80)."""
    assert logits_u16.dtype == np.uint16 and logits_u16.flags.c_contiguous and logits_u16.ndim == 2
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    ids = np.empty((bm.shape[0], k), dtype=np.int32)
    vals = np.empty((bm.shape[0], k), dtype=np.uint16)
    _load().pre3o_masked_topk(_ptr(logits_u16), _ptr(bm), bm.shape[0], int(n_tokens), logits_u16.shape[1], int(k),
                              _ptr(ids), _ptr(vals))
    return ids, vals
