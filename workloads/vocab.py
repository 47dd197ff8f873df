"""Seeded synthetic vocabularies and logits (inputs only)."""
from __future__ import annotations

import numpy as np

BASE_SEED = 2506_03887 * 10


class Vocab:
    """token t = bytes[offsets[t]:offsets[t+1]]; the bytes of eos_id are ignored."""

    def __init__(self, tokens, eos_id: int):
        self.tokens = [bytes(t) for t in tokens]
        self.n_tokens = len(self.tokens)
        self.eos_id = int(eos_id)
        lens = np.array([len(t) for t in self.tokens], dtype=np.int64)
        self.offsets = np.zeros(self.n_tokens + 1, dtype=np.int64)
        np.cumsum(lens, out=self.offsets[1:])
        self.bytes = np.frombuffer(b"".join(self.tokens) + b"\0", dtype=np.uint8).copy()
        self.words = (self.n_tokens + 31) // 32
        self.max_len = int(lens.max()) if self.n_tokens else 0


def _byte_distribution():
    """JSON-text-like byte distribution: 40% letters (a-z 32%, A-Z 8%), 15% digits, 25%
    uniform over the seven bytes \"{}[]:, and 20% other (space 8%, newline 2%, 1% each of
    - . _ / \\ + e E t n)."""
    p = np.zeros(256)
    for c in range(ord("a"), ord("z") + 1):
        p[c] += 0.32 / 26
    for c in range(ord("A"), ord("Z") + 1):
        p[c] += 0.08 / 26
    for c in range(ord("0"), ord("9") + 1):
        p[c] += 0.15 / 10
    for c in b'"{}[]:,':
        p[c] += 0.25 / 7
    p[ord(" ")] += 0.08
    p[ord("\n")] += 0.02
    for c in b"-._/\\+eEtn":
        p[c] += 0.01
    return p / p.sum()


def bpe_like_vocab(n_tokens: int, max_len: int, seed: int) -> Vocab:
    """ids 0..255 are the 256 single bytes (byte fallback, as in real BPE vocabularies), id
    n_tokens-1 is the end-of-sequence token, every other token has length
    min(Geometric(p=0.25), max_len) (mean 4) and i.i.d. bytes from the distribution above.
    Duplicate strings are kept."""
    rng = np.random.default_rng(seed)
    p = _byte_distribution()
    n_rand = n_tokens - 257
    lens = np.minimum(rng.geometric(0.25, size=n_rand), max_len)
    flat = rng.choice(256, size=int(lens.sum()), p=p).astype(np.uint8)
    tokens = [bytes([b]) for b in range(256)]
    pos = 0
    for n in lens:
        tokens.append(flat[pos:pos + n].tobytes())
        pos += int(n)
    tokens.append(b"")                    # EOS
    return Vocab(tokens, n_tokens - 1)


def arithmetic_vocab(seed: int) -> Vocab:
    """512 tokens of length U{1..4} over the alphabet 'a+*()b- ', plus EOS as id 512.  The
    seed is bumped until each of the five grammar terminals occurs as a one-byte token."""
    alphabet = b"a+*()b- "
    while True:
        rng = np.random.default_rng(seed)
        lens = rng.integers(1, 5, size=512)
        tokens = [bytes(alphabet[int(i)] for i in rng.integers(0, len(alphabet), size=int(n))) for n in lens]
        if all(bytes([c]) in tokens for c in b"a+*()"):
            tokens.append(b"")
            return Vocab(tokens, 512)
        seed += 1000


def bf16_logits(rng: np.random.Generator, batch: int, n_tokens: int) -> np.ndarray:
    """N(0,1) float32 rounded to nearest-even bf16; returned as raw uint16 bit patterns."""
    x = rng.standard_normal((batch, n_tokens), dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)
