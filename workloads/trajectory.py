"""Seeded decode trajectories: which token every sequence samples at every step.

The driver draws, for each live sequence, one token uniformly at random from the tokens
that a *checker* (passed in by the caller; the tests pass the CPU oracle) allows, subject
to the workload's caps.  It holds no automaton logic of its own: it only asks the checker
"which of these token ids are allowed after this stack" and "advance this batch".

Rules of the recipe:
  * the end-of-sequence token is taken with probability 1/2 whenever it is allowed, and
    always on the last step if allowed; a finished sequence is reset to its initial
    stack at the next step (continuous-batching slot reuse) - recorded in `reset`;
  * tokens that would raise container nesting (unclosed { or [ outside strings, or
    unclosed parentheses) above `nest_cap`, or the stack above `len_cap` entries, are
    not drawn;
  * a workload of line-structured text sets `p_line_feed`: with that probability the draw is
    first tried among the allowed tokens that contain a line feed (uniformly), so that lines end;
  * otherwise the draw is uniform over the remaining allowed tokens: candidates are the tokens whose
    first byte is viable (found by asking the checker about the one-byte tokens), sampled
    by rejection, then by enumeration if rejection keeps failing.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Trajectory:
    tokens: np.ndarray            # [steps, B] int32 token drawn at each step
    reset: np.ndarray             # [steps, B] bool: sequence starts afresh at this step
    init_data: np.ndarray         # [B, cap] int32 initial stacks (step 0)
    init_len: np.ndarray          # [B] int32
    grammar_idx: np.ndarray       # [B] int32 grammar of each sequence
    cap: int
    depth_hist: dict = field(default_factory=dict)


class _Lexer:
    """Tracks container nesting of the emitted text: { [ ( outside JSON strings.  With a
    `marker`, nothing counts until the text has contained the marker's bytes (a workload whose
    documents open with free text that must not be read as containers)."""

    __slots__ = ("in_string", "escape", "depth", "marker", "matched")

    def __init__(self, marker: bytes = b""):
        self.in_string = False
        self.escape = False
        self.depth = 0
        self.marker = marker
        self.matched = 0              # bytes of the marker seen so far; len(marker) = counting

    def copy(self):
        c = _Lexer(self.marker)
        c.in_string, c.escape, c.depth, c.matched = self.in_string, self.escape, self.depth, self.matched
        return c

    def feed(self, data: bytes, strings: bool):
        """Returns the maximum depth reached while reading `data`."""
        peak = self.depth
        for c in data:
            if self.matched < len(self.marker):
                # the markers in use start with a byte that occurs nowhere else in them, so a
                # mismatch can only restart the match at that first byte
                self.matched = self.matched + 1 if c == self.marker[self.matched] else int(c == self.marker[0])
                continue
            if self.in_string:
                if self.escape:
                    self.escape = False
                elif c == 0x5C:
                    self.escape = True
                elif c == 0x22:
                    self.in_string = False
            elif c == 0x22 and strings:
                self.in_string = True
            elif c in (0x7B, 0x5B, 0x28):
                self.depth += 1
                peak = max(peak, self.depth)
            elif c in (0x7D, 0x5D, 0x29):
                self.depth -= 1
        return peak


def _first_byte_buckets(vocab):
    buckets = [[] for _ in range(256)]
    for t, tok in enumerate(vocab.tokens):
        if t != vocab.eos_id and len(tok) > 0:
            buckets[tok[0]].append(t)
    return [np.array(b, dtype=np.int32) for b in buckets]


class Driver:
    def __init__(self, checker, vocab, batch, cap, seed, grammar_idx=None, nest_cap=10,
                 len_cap=None, json_strings=True, p_eos=0.5, marker=b"", p_line_feed=0.0):
        self.ck, self.vocab, self.B, self.cap = checker, vocab, batch, cap
        self.rng = np.random.default_rng(seed)
        self.grammar_idx = (np.zeros(batch, dtype=np.int32) if grammar_idx is None
                            else np.asarray(grammar_idx, dtype=np.int32))
        self.nest_cap, self.len_cap = nest_cap, (cap if len_cap is None else len_cap)
        self.json_strings, self.p_eos, self.marker = json_strings, p_eos, marker
        self.buckets = _first_byte_buckets(vocab)
        self.p_line_feed = p_line_feed
        self.line_feed_tokens = (np.array([t for t, tok in enumerate(vocab.tokens) if b"\n" in tok and t != vocab.eos_id],
                                          dtype=np.int32) if p_line_feed > 0 else None)
        # does the vocabulary hold every single byte as ids 0..255 (byte fallback)?
        self.byte_fallback = vocab.n_tokens > 256 and all(vocab.tokens[b] == bytes([b]) for b in range(256))
        self.states = np.zeros(batch, dtype=np.int32)
        self.data = np.zeros((batch, cap), dtype=np.int32)
        self.len = np.ones(batch, dtype=np.int32)
        self.lex = [_Lexer(marker) for _ in range(batch)]
        for b in range(batch):
            self._reset(b)

    def _reset(self, b):
        s0 = self.ck.initial_state(int(self.grammar_idx[b]))
        self.data[b, 0] = s0
        self.len[b] = 1
        self.states[b] = s0
        self.lex[b] = _Lexer(self.marker)

    def _fits(self, b, t):
        tok = self.vocab.tokens[t]
        if self.lex[b].copy().feed(tok, self.json_strings) > self.nest_cap:
            return False
        stack = self.data[b, : self.len[b]]
        rc, new = self.ck.advance(stack, tok, cap=self.len_cap)
        return rc == 0

    def _draw(self, b, last_step):
        stack = self.data[b, : self.len[b]]
        if self.ck.eos_allowed(stack) and (last_step or self.rng.random() < self.p_eos):
            return self.vocab.eos_id
        if self.p_line_feed > 0 and self.rng.random() < self.p_line_feed:
            ok = self.line_feed_tokens[self.ck.allowed_many(stack, self.vocab, self.line_feed_tokens)]
            for t in self.rng.permutation(ok):
                if self._fits(b, int(t)):
                    return int(t)
        if self.byte_fallback:
            viable = np.flatnonzero(self.ck.allowed_many(stack, self.vocab, np.arange(256, dtype=np.int32)))
            cand = np.concatenate([self.buckets[c] for c in viable]) if len(viable) else np.zeros(0, np.int32)
        else:
            cand = np.array([t for t in range(self.vocab.n_tokens)
                             if t != self.vocab.eos_id and len(self.vocab.tokens[t])], dtype=np.int32)
        if len(cand) == 0:
            if self.ck.eos_allowed(stack):
                return self.vocab.eos_id
            raise RuntimeError("no viable token")
        for _ in range(64):                       # rejection sampling, uniform over cand
            t = int(cand[self.rng.integers(len(cand))])
            if self.ck.allowed(stack, self.vocab.tokens[t]) and self._fits(b, t):
                return t
        ok = cand[self.ck.allowed_many(stack, self.vocab, cand)]
        ok = self.rng.permutation(ok)
        for t in ok:
            if self._fits(b, int(t)):
                return int(t)
        if self.ck.eos_allowed(stack):
            return self.vocab.eos_id
        raise RuntimeError("no token satisfies the workload caps")

    def step(self, last_step=False):
        """Draw one token per sequence and advance.  Returns (tokens[B], reset[B])."""
        reset = np.zeros(self.B, dtype=bool)
        for b in range(self.B):
            if self.states[b] < 0:
                self._reset(b)
                reset[b] = True
        tokens = np.array([self._draw(b, last_step) for b in range(self.B)], dtype=np.int32)
        err = self.ck.advance_batch(self.states, self.data, self.len, tokens, self.vocab)
        assert not err.any(), "driver drew a token the checker refuses to advance by"
        for b in range(self.B):
            if tokens[b] != self.vocab.eos_id:
                self.lex[b].feed(self.vocab.tokens[tokens[b]], self.json_strings)
        return tokens, reset

    def warm_to_depths(self, target_depths, max_steps=400):
        """Advance sequence b along a random valid prefix until len-1 >= target_depths[b]
        (or keep the deepest stack seen).  Used to seed deep initial stacks."""
        best = [(self.data[b, : self.len[b]].copy(), self.lex[b].copy()) for b in range(self.B)]
        for b in range(self.B):
            d = int(target_depths[b])
            for _ in range(max_steps):
                if self.len[b] - 1 >= d:
                    break
                t = self._draw(b, False)
                if t == self.vocab.eos_id:
                    self._reset(b)
                    continue
                tok = self.vocab.tokens[t]
                rc, new = self.ck.advance(self.data[b, : self.len[b]], tok, cap=self.len_cap)
                assert rc == 0
                self.data[b, : len(new)] = new
                self.len[b] = len(new)
                self.states[b] = new[-1]
                self.lex[b].feed(tok, self.json_strings)
                if len(new) > len(best[b][0]):
                    best[b] = (np.array(new, dtype=np.int32), self.lex[b].copy())
            if self.len[b] - 1 < d:
                st, lx = best[b]
                self.data[b, : len(st)] = st
                self.len[b] = len(st)
                self.states[b] = st[-1]
                self.lex[b] = lx


def generate(checker, vocab, batch, steps, cap, seed, grammar_idx=None, nest_cap=10, len_cap=None,
             json_strings=True, target_depths=None, progress=None, marker=b"",
             p_line_feed=0.0) -> Trajectory:
    drv = Driver(checker, vocab, batch, cap, seed, grammar_idx, nest_cap, len_cap, json_strings, marker=marker,
                 p_line_feed=p_line_feed)
    if target_depths is not None:
        drv.warm_to_depths(target_depths)
    init_data, init_len = drv.data.copy(), drv.len.copy()
    depths, counts = np.unique(init_len - 1, return_counts=True)
    toks = np.zeros((steps, batch), dtype=np.int32)
    reset = np.zeros((steps, batch), dtype=bool)
    for s in range(steps):
        toks[s], reset[s] = drv.step(last_step=(s == steps - 1))
        if progress and (s % 16 == 15 or s == steps - 1):
            progress(s + 1, steps)
    return Trajectory(toks, reset, init_data, init_len, drv.grammar_idx.copy(), cap,
                      dict(zip(depths.tolist(), counts.tolist())))
