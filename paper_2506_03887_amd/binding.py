"""Thin ctypes binding of libpre3.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  Device buffers are torch tensors
(PyTorch is used for device memory and streams only); their data_ptr() and the current
stream's handle are passed through the C ABI declared in include/pre3.h.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpre3.so")

PRE3_OK = 0
E_BADARG, E_PARSE, E_NOT_LR1, E_TOKEN_TOO_LONG, E_NOMEM, E_HIP, E_LIMIT = -1, -2, -3, -4, -5, -6, -7
FLAG_HOST_ONLY = 1
FLAG_NO_TOKEN_EDGES = 2
FLAG_STEPWISE_REDUCTIONS = 4
FLAG_COMPACT_CYCLES = 8
FLAG_NO_TOKEN_EFFECTS = 16
ADVANCE_RESTART_ON_EOS = 1
STEP_ONE_KERNEL = 2
STATE_DONE = -1

EXPORTS = [
    "pre3_compile", "pre3_free", "pre3_last_error", "pre3_initial_state", "pre3_bind_state",
    "pre3_fill_mask", "pre3_apply_mask", "pre3_fill_apply_mask", "pre3_advance", "pre3_advance_fill_mask", "pre3_advance_fill_apply_mask", "pre3_advance_fill_argmax", "pre3_step_is_one_kernel", "pre3_apply_mask_argmax", "pre3_apply_mask_topk", "pre3_jump_forward", "pre3_n_grammars", "pre3_n_states",
    "pre3_n_byte_classes", "pre3_byte_class", "pre3_edge", "pre3_goto_target", "pre3_walk_depth_bound",
    "pre3_token_edge_stats", "pre3_debug_resolve_row", "pre3_symbol_edge_stats", "pre3_debug_advance", "pre3_debug_validate_tables",
    "pre3_forced_run", "pre3_n_reduction_cycles", "pre3_reduction_cycle", "pre3_debug_compact", "pre3_debug_fault_count", "pre3_debug_timestamp", "pre3_advance_static", "pre3_token_effect_stats", "pre3_debug_token_effect",
]


class Pre3Error(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"pre3 status {status}: {text}")
        self.status = status


class _Vocab(ctypes.Structure):
    _fields_ = [("bytes", ctypes.c_void_p), ("offsets", ctypes.c_void_p),
                ("n_tokens", ctypes.c_int32), ("eos_id", ctypes.c_int32)]


class _Options(ctypes.Structure):
    _fields_ = [("max_token_len", ctypes.c_int32), ("stack_cap", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("max_condition_depth", ctypes.c_int32), ("row_threshold", ctypes.c_int32),
                ("effect_min_len", ctypes.c_int32)]


class _Stacks(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("len", ctypes.c_void_p),
                ("cap", ctypes.c_int32), ("batch", ctypes.c_int32)]


_lib = None


def load():
    """Loads the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime: it must be in the process before libpre3.so is
    # loaded, so that both resolve to the same runtime (two runtimes cannot share the GPU).
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with paper_2506_03887_amd.build.build()")
    lib = ctypes.CDLL(LIB_PATH)
    c, vp, i32 = ctypes, ctypes.c_void_p, ctypes.c_int32
    lib.pre3_compile.argtypes = [c.POINTER(c.c_char_p), i32, c.POINTER(_Vocab), c.POINTER(_Options), c.POINTER(vp)]
    lib.pre3_free.argtypes = [vp]
    lib.pre3_last_error.argtypes = [vp]
    lib.pre3_last_error.restype = c.c_char_p
    lib.pre3_initial_state.argtypes = [vp, i32]
    lib.pre3_bind_state.argtypes = [vp, vp, _Stacks, vp]
    lib.pre3_fill_mask.argtypes = [vp, vp, _Stacks, vp, vp]
    lib.pre3_apply_mask.argtypes = [vp, vp, i32, i32, c.c_int64, vp]
    lib.pre3_fill_apply_mask.argtypes = [vp, vp, _Stacks, vp, vp, c.c_int64, vp]
    lib.pre3_advance.argtypes = [vp, vp, vp]
    lib.pre3_advance_fill_mask.argtypes = [vp, vp, vp, i32, vp]
    lib.pre3_advance_fill_apply_mask.argtypes = [vp, vp, vp, vp, c.c_int64, i32, vp]
    lib.pre3_step_is_one_kernel.argtypes = [vp, vp, c.c_int64, i32]
    lib.pre3_advance_fill_argmax.argtypes = [vp, vp, vp, vp, c.c_int64, vp, i32, vp]
    lib.pre3_advance_static.argtypes = [vp, vp, vp, _Stacks, vp, vp]
    lib.pre3_apply_mask_argmax.argtypes = [vp, vp, c.c_int64, vp, vp, vp]
    lib.pre3_apply_mask_topk.argtypes = [vp, vp, c.c_int64, vp, i32, vp, vp, vp]
    lib.pre3_jump_forward.argtypes = [vp, vp, vp, i32, vp]
    lib.pre3_reduction_cycle.argtypes = [vp, i32, vp, i32]
    lib.pre3_forced_run.argtypes = [vp, i32, vp, vp, i32]
    lib.pre3_debug_compact.argtypes = [vp, vp, i32]
    lib.pre3_debug_fault_count.argtypes = [vp, c.POINTER(c.c_int64)]
    lib.pre3_debug_timestamp.argtypes = [vp, vp]
    for name in ("pre3_n_grammars", "pre3_n_states", "pre3_n_byte_classes", "pre3_walk_depth_bound",
                 "pre3_n_reduction_cycles"):
        getattr(lib, name).argtypes = [vp]
    lib.pre3_byte_class.argtypes = [vp, i32]
    lib.pre3_debug_validate_tables.argtypes = [vp]
    lib.pre3_edge.argtypes = [vp, i32, i32, c.POINTER(i32), c.POINTER(i32)]
    lib.pre3_goto_target.argtypes = [vp, i32, i32]
    lib.pre3_token_edge_stats.argtypes = [vp, vp]
    lib.pre3_symbol_edge_stats.argtypes = [vp, vp]
    lib.pre3_token_effect_stats.argtypes = [vp, vp]
    lib.pre3_debug_token_effect.argtypes = [vp, vp, i32, i32, vp, i32, vp]
    lib.pre3_debug_advance.argtypes = [vp, vp, vp, i32, vp, i32, i32]
    lib.pre3_debug_resolve_row.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp]
    for name in EXPORTS:
        if name != "pre3_last_error":
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t, dtype_name):
    """Device pointer of a contiguous torch tensor of the expected dtype."""
    import torch
    want = {"i32": torch.int32, "u16": (torch.bfloat16, torch.uint16, torch.int16), "u32": (torch.int32, torch.uint32),
            "u8": torch.uint8}[dtype_name]
    ok = t.dtype in want if isinstance(want, tuple) else t.dtype == want
    if not (t.is_cuda and ok):
        raise TypeError(f"expected a CUDA tensor of kind {dtype_name}, got {t.dtype} on {t.device}")
    return ctypes.c_void_p(t.data_ptr())


class Pre3:
    """Compiled grammar(s) + vocabulary.  Mirrors the C entry points one to one."""

    def __init__(self, grammars, vocab_bytes: np.ndarray, vocab_offsets: np.ndarray, eos_id: int,
                 max_token_len: int = 64, stack_cap: int = 1024, host_only: bool = False,
                 token_edges: bool = True, max_condition_depth: int = 0, merged_reductions: bool = True,
                 row_threshold: int = 0, compact_cycles: bool = False, token_effects: bool = True,
                 effect_min_len: int = 0):
        lib = load()
        if isinstance(grammars, str):
            grammars = [grammars]
        texts = (ctypes.c_char_p * len(grammars))(*[g.encode("latin-1") for g in grammars])
        vb = np.ascontiguousarray(vocab_bytes, dtype=np.uint8)
        vo = np.ascontiguousarray(vocab_offsets, dtype=np.int64)
        voc = _Vocab(vb.ctypes.data, vo.ctypes.data, len(vo) - 1, eos_id)
        opt = _Options(max_token_len, stack_cap,
                       (FLAG_HOST_ONLY if host_only else 0) | (0 if token_edges else FLAG_NO_TOKEN_EDGES)
                       | (0 if merged_reductions else FLAG_STEPWISE_REDUCTIONS)
                       | (FLAG_COMPACT_CYCLES if compact_cycles else 0) | (0 if token_effects else FLAG_NO_TOKEN_EFFECTS),
                       max_condition_depth, row_threshold, effect_min_len)
        h = ctypes.c_void_p()
        rc = lib.pre3_compile(texts, len(grammars), ctypes.byref(voc), ctypes.byref(opt), ctypes.byref(h))
        self._lib, self._h = lib, h
        if rc != PRE3_OK:
            text = lib.pre3_last_error(h).decode() if h else "allocation failed"
            lib.pre3_free(h)
            self._h = None
            raise Pre3Error(rc, text)
        self.n_tokens = len(vo) - 1
        self.words = (self.n_tokens + 31) // 32
        self.eos_id = eos_id
        self._bound = None

    def close(self):
        if getattr(self, "_h", None):
            self._lib.pre3_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def _check(self, rc):
        if rc != PRE3_OK:
            raise Pre3Error(rc, self._lib.pre3_last_error(self._h).decode())

    # ---- host queries
    def initial_state(self, g=0):
        s = self._lib.pre3_initial_state(self._h, g)
        if s < 0:
            raise Pre3Error(s, "bad grammar index")
        return s

    n_grammars = property(lambda self: self._lib.pre3_n_grammars(self._h))
    n_states = property(lambda self: self._lib.pre3_n_states(self._h))
    n_byte_classes = property(lambda self: self._lib.pre3_n_byte_classes(self._h))
    walk_depth_bound = property(lambda self: self._lib.pre3_walk_depth_bound(self._h))

    def byte_class(self, byte):
        return self._lib.pre3_byte_class(self._h, byte)

    def edge(self, state, symbol):
        a0, a1 = ctypes.c_int32(), ctypes.c_int32()
        kind = self._lib.pre3_edge(self._h, state, symbol, ctypes.byref(a0), ctypes.byref(a1))
        return kind, a0.value, a1.value

    def goto_target(self, state, nt):
        return self._lib.pre3_goto_target(self._h, state, nt)

    def token_edge_stats(self):
        out = (ctypes.c_int64 * 8)()
        self._check(self._lib.pre3_token_edge_stats(self._h, out))
        keys = ["built", "roots", "nodes", "dense_rows", "delta_ids", "walk_ids", "max_known", "device_bytes"]
        return dict(zip(keys, list(out)))

    def token_effect_stats(self):
        out = (ctypes.c_int64 * 4)()
        self._check(self._lib.pre3_token_effect_stats(self._h, out))
        return dict(zip(["records", "stored", "dropped", "device_bytes"], list(out)))

    def debug_token_effect(self, stack, token: int):
        """Host mirror of the effect look-up: (new stack list, k, peak, n_push) or None if no record covers it."""
        st = np.ascontiguousarray(stack, dtype=np.int32)
        out = np.zeros(len(st) + 256, dtype=np.int32)
        info = np.zeros(3, dtype=np.int32)
        n = self._lib.pre3_debug_token_effect(self._h, st.ctypes.data, len(st), int(token), out.ctypes.data, len(out), info.ctypes.data)
        if n < 0:
            raise Pre3Error(n, "debug_token_effect")
        return None if n == 0 else (out[:n].tolist(), int(info[0]), int(info[1]), int(info[2]))

    def symbol_edge_stats(self):
        out = (ctypes.c_int64 * 4)()
        self._check(self._lib.pre3_symbol_edge_stats(self._h, out))
        return dict(zip(["built", "nodes", "max_known", "device_bytes"], list(out)))

    def debug_advance(self, stack, data: bytes, cap: int = 1 << 20, merged: bool = True, end: bool = False):
        """Host mirror of advance on one stack: (rc, new stack list)."""
        n = len(stack)
        cap = int(min(cap, n + 8 * len(data) + 64))
        st = np.zeros(cap, dtype=np.int32)
        st[:n] = stack
        ln = ctypes.c_int32(n)
        buf = np.frombuffer(bytes(data) + b"\0", dtype=np.uint8)
        rc = self._lib.pre3_debug_advance(self._h, st.ctypes.data, ctypes.byref(ln), cap, buf.ctypes.data,
                                          -1 if end else len(data), int(merged))
        if rc < 0:
            raise Pre3Error(rc, "debug_advance")
        return rc, st[: ln.value].tolist()

    def reduction_cycles(self):
        """The registered reduction cycles, each a list of global state ids v1..vn."""
        out = []
        buf = np.zeros(64, dtype=np.int32)
        for i in range(self._lib.pre3_n_reduction_cycles(self._h)):
            n = self._lib.pre3_reduction_cycle(self._h, i, buf.ctypes.data, len(buf))
            if n < 0:
                raise Pre3Error(n, "reduction_cycle")
            out.append(buf[:n].tolist())
        return out

    def debug_compact(self, stack):
        """Host evaluation of the compaction normal form on the compiled cycle tables."""
        st = np.array(stack, dtype=np.int32)
        n = self._lib.pre3_debug_compact(self._h, st.ctypes.data, len(st))
        if n < 0:
            raise Pre3Error(n, "debug_compact")
        return st[:n].tolist()

    def forced_run(self, state: int):
        """(bytes, states) of the run of forced bytes that starts at `state` (empty if it forces nothing)."""
        out_b = (ctypes.c_uint8 * 64)()
        out_s = (ctypes.c_int32 * 64)()
        n = self._lib.pre3_forced_run(self._h, int(state), out_b, out_s, 64)
        if n < 0:
            raise Pre3Error(n, "forced_run")
        return bytes(out_b[:n]), list(out_s[:n])

    def fault_count(self) -> int:
        """Walks that a kernel stopped at an internal guard since compile (0 expected); synchronises first."""
        import torch
        torch.cuda.synchronize()
        n = ctypes.c_int64()
        self._check(self._lib.pre3_debug_fault_count(self._h, ctypes.byref(n)))
        return n.value

    def validate_tables(self) -> int:
        """Number of out-of-range indices in the compiled tables (0 expected)."""
        rc = self._lib.pre3_debug_validate_tables(self._h)
        if rc < 0:
            raise Pre3Error(rc, "validate_tables")
        return rc

    def debug_resolve_row(self, stack):
        """(resolved?, row bits uint32[W], walk token ids) from the host copy of the tables."""
        st = np.ascontiguousarray(stack, dtype=np.int32)
        row = np.zeros(self.words, dtype=np.uint32)
        walk = np.zeros(self.n_tokens, dtype=np.int32)
        n = ctypes.c_int32()
        info = np.zeros(4, dtype=np.int32)
        rc = self._lib.pre3_debug_resolve_row(self._h, st.ctypes.data, len(st), row.ctypes.data,
                                              walk.ctypes.data, len(walk), ctypes.byref(n), info.ctypes.data)
        self.last_resolve_info = dict(zip(["path_nodes", "dense_index", "delta_ids", "deepest_entry"], info.tolist()))
        if rc < 0:
            raise Pre3Error(rc, "debug_resolve_row")
        return bool(rc), row, walk[: n.value].copy()

    # ---- device calls (torch tensors in, nothing out: all results are written in place)
    @staticmethod
    def _stacks(data, length):
        batch, cap = data.shape
        assert data.is_contiguous() and length.is_contiguous() and length.numel() == batch
        return _Stacks(_dev(data, "i32"), _dev(length, "i32"), cap, batch)

    def bind_state(self, states, data, length, err):
        self._check(self._lib.pre3_bind_state(self._h, _dev(states, "i32"), self._stacks(data, length), _dev(err, "i32")))
        self._bound = (states, data, length, err)          # keep the tensors alive

    def fill_mask(self, states, data, length, bitmask, stream=None):
        assert bitmask.is_contiguous() and tuple(bitmask.shape) == (data.shape[0], self.words)
        self._check(self._lib.pre3_fill_mask(self._h, _dev(states, "i32"), self._stacks(data, length),
                                             _dev(bitmask, "u32"), _stream_ptr(stream)))

    def fill_apply_mask(self, states, data, length, bitmask, logits, stream=None):
        assert bitmask.is_contiguous() and tuple(bitmask.shape) == (data.shape[0], self.words)
        assert logits.dim() == 2 and logits.stride(1) == 1 and logits.shape[0] == data.shape[0]
        self._check(self._lib.pre3_fill_apply_mask(self._h, _dev(states, "i32"), self._stacks(data, length),
                                                   _dev(bitmask, "u32"), _dev(logits, "u16"), logits.stride(0),
                                                   _stream_ptr(stream)))

    def advance(self, tokens, stream=None):
        assert tokens.is_contiguous()
        self._check(self._lib.pre3_advance(self._h, _dev(tokens, "i32"), _stream_ptr(stream)))

    def advance_static(self, tokens, states, data, length, err, stream=None):
        """pre3_advance on the buffers passed in, with the library's static spill area (no allocation)."""
        assert tokens.is_contiguous() and tokens.numel() == data.shape[0] == states.numel() == err.numel()
        self._check(self._lib.pre3_advance_static(self._h, _dev(tokens, "i32"), _dev(states, "i32"),
                                                  self._stacks(data, length), _dev(err, "i32"), _stream_ptr(stream)))

    def advance_fill_mask(self, tokens, bitmask, restart_on_eos=False, stream=None):
        assert tokens.is_contiguous() and bitmask.is_contiguous() and bitmask.shape[1] == self.words
        self._check(self._lib.pre3_advance_fill_mask(self._h, _dev(tokens, "i32"), _dev(bitmask, "u32"),
                                                     ADVANCE_RESTART_ON_EOS if restart_on_eos else 0,
                                                     _stream_ptr(stream)))

    def advance_fill_apply_mask(self, tokens, bitmask, logits, restart_on_eos=False, one_kernel=False, stream=None):
        """The whole decode step: advance, next mask rows, and those rows applied to `logits` in place.
        one_kernel: ask for the one-kernel form at any batch size (the library chooses by itself otherwise)."""
        assert tokens.is_contiguous() and bitmask.is_contiguous() and bitmask.shape[1] == self.words
        assert logits.dim() == 2 and logits.stride(1) == 1 and logits.shape[0] == bitmask.shape[0]
        self._check(self._lib.pre3_advance_fill_apply_mask(self._h, _dev(tokens, "i32"), _dev(bitmask, "u32"),
                                                           _dev(logits, "u16"), logits.stride(0),
                                                           (ADVANCE_RESTART_ON_EOS if restart_on_eos else 0) |
                                                           (STEP_ONE_KERNEL if one_kernel else 0),
                                                           _stream_ptr(stream)))

    def advance_fill_argmax(self, tokens, bitmask, logits, out_tokens, restart_on_eos=False, one_kernel=False, stream=None):
        """The whole greedy step: advance, next mask rows, and out_tokens[b] = arg max of the allowed logits of
        row b (the logits are only read; out_tokens may be `tokens`)."""
        assert tokens.is_contiguous() and bitmask.is_contiguous() and bitmask.shape[1] == self.words and out_tokens.is_contiguous()
        assert logits.dim() == 2 and logits.stride(1) == 1 and logits.shape[0] == bitmask.shape[0] == out_tokens.numel()
        self._check(self._lib.pre3_advance_fill_argmax(self._h, _dev(tokens, "i32"), _dev(bitmask, "u32"),
                                                       _dev(logits, "u16"), logits.stride(0), _dev(out_tokens, "i32"),
                                                       (ADVANCE_RESTART_ON_EOS if restart_on_eos else 0) |
                                                       (STEP_ONE_KERNEL if one_kernel else 0), _stream_ptr(stream)))

    def step_kernel_launches(self, logits, one_kernel=False):
        """0 if advance_fill_apply_mask is two calls for the bound batch and these logits, else the number of launches
        of its one kernel (1 up to one sequence per compute unit, equal shares of the batch beyond)."""
        rc = self._lib.pre3_step_is_one_kernel(self._h, _dev(logits, "u16"), logits.stride(0), STEP_ONE_KERNEL if one_kernel else 0)
        if rc < 0:
            raise Pre3Error(rc, "step_is_one_kernel")
        return rc

    def step_is_one_kernel(self, logits, one_kernel=False):
        """Whether advance_fill_apply_mask runs as one kernel for the bound batch and these logits."""
        return self.step_kernel_launches(logits, one_kernel) > 0

    def apply_mask_argmax(self, logits, bitmask, out_tokens, stream=None):
        """out_tokens[b] = id of the largest allowed logit of row b (bound batch); the logits are only read."""
        assert logits.dim() == 2 and logits.stride(1) == 1 and bitmask.is_contiguous() and out_tokens.is_contiguous()
        assert bitmask.shape[1] == self.words and out_tokens.numel() == logits.shape[0] == bitmask.shape[0]
        self._check(self._lib.pre3_apply_mask_argmax(self._h, _dev(logits, "u16"), logits.stride(0), _dev(bitmask, "u32"),
                                                     _dev(out_tokens, "i32"), _stream_ptr(stream)))

    def apply_mask_topk(self, logits, bitmask, out_tokens, out_logits=None, stream=None):
        """out_tokens[b, j] = id of the (j+1)-th largest allowed logit of row b (k = out_tokens.shape[1], -1
        padded), out_logits[b, j] (optional, bf16/int16/uint16) its stored pattern; the logits are only read."""
        assert logits.dim() == 2 and logits.stride(1) == 1 and bitmask.is_contiguous() and out_tokens.is_contiguous()
        assert out_tokens.dim() == 2 and out_tokens.shape[0] == logits.shape[0] == bitmask.shape[0]
        assert bitmask.shape[1] == self.words
        if out_logits is not None:
            assert out_logits.is_contiguous() and out_logits.shape == out_tokens.shape
        self._check(self._lib.pre3_apply_mask_topk(self._h, _dev(logits, "u16"), logits.stride(0), _dev(bitmask, "u32"),
                                                   out_tokens.shape[1], _dev(out_tokens, "i32"),
                                                   None if out_logits is None else _dev(out_logits, "u16"),
                                                   _stream_ptr(stream)))

    def jump_forward(self, out_bytes, out_len, stream=None):
        """Forced bytes of every bound sequence into out_bytes [B, max_bytes] (uint8), their counts into
        out_len [B]; the stacks are advanced by them."""
        assert out_bytes.dim() == 2 and out_bytes.is_contiguous() and out_len.is_contiguous()
        assert out_bytes.shape[0] == out_len.numel()
        self._check(self._lib.pre3_jump_forward(self._h, _dev(out_bytes, "u8"), _dev(out_len, "i32"), out_bytes.shape[1],
                                                _stream_ptr(stream)))


def apply_mask(logits, bitmask, vocab: int, stream=None):
    """In place on a [B, >=vocab] bf16 tensor whose rows may be strided."""
    lib = load()
    assert logits.dim() == 2 and logits.stride(1) == 1 and bitmask.is_contiguous()
    rc = lib.pre3_apply_mask(_dev(logits, "u16"), _dev(bitmask, "u32"), logits.shape[0], vocab,
                             logits.stride(0), _stream_ptr(stream))
    if rc != PRE3_OK:
        raise Pre3Error(rc, "apply_mask: bad argument or launch failure")


def device_timestamp(out, index: int = 0, stream=None):
    """Enqueues a one-thread kernel that writes the device's 100 MHz wall clock to out[index]
    (out: int64 device tensor).  Between the calls of a captured step this times each kernel in place."""
    lib = load()
    assert out.dtype.itemsize == 8 and out.is_contiguous() and 0 <= index < out.numel()
    rc = lib.pre3_debug_timestamp(out.data_ptr() + 8 * index, _stream_ptr(stream))
    if rc != PRE3_OK:
        raise Pre3Error(rc, "device_timestamp: bad argument or launch failure")
