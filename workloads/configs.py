"""The seeded synthetic workload configurations (inputs only)."""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache

import numpy as np

from . import grammars as G
from .vocab import BASE_SEED, Vocab, arithmetic_vocab, bpe_like_vocab

STACK_CAP = 1024


@dataclass
class Config:
    idx: int
    name: str
    grammars: list            # grammar texts; several = disjoint union
    vocab: Vocab
    batch: int
    steps: int
    nest_cap: int
    cap: int = STACK_CAP
    json_strings: bool = True
    mixed: bool = False       # sequences on different grammars with deep seeded stacks
    seed: int = 0
    notes: dict = None
    marker: bytes = b""       # container nesting is counted only after these bytes (free text first)
    p_line_feed: float = 0.0  # chance that a draw prefers the tokens that hold a line feed
    compact: bool = False     # stacks are kept without complete traversals of reduction cycles


# (n_keys, depth, n_enum, extra_objects) of the eight schema grammars of config 5, chosen so the
# numbers of productions as written span roughly 50..400.
_CFG5_SHAPES = [(5, 1, 8, 0), (8, 2, 8, 0), (12, 2, 8, 0), (14, 3, 8, 1),
                (16, 3, 8, 2), (16, 3, 8, 3), (18, 3, 8, 3), (19, 3, 8, 3)]


@lru_cache(maxsize=None)
def get(idx: int) -> Config:
    seed = BASE_SEED + idx
    if idx == 1:
        return Config(1, "arithmetic-B4-V513", [G.ARITHMETIC], arithmetic_vocab(seed), 4, 32,
                      nest_cap=8, json_strings=False, seed=seed)
    if idx == 2:
        return Config(2, "json-B64-V32000", [G.JSON], bpe_like_vocab(32000, 16, seed), 64, 128,
                      nest_cap=6, seed=seed)
    if idx == 3:
        return Config(3, "json-B256-V128256", [G.JSON], bpe_like_vocab(128256, 32, seed), 256, 256,
                      nest_cap=10, seed=seed)
    if idx == 4:
        sg = G.schema_grammar(seed, n_keys=12, depth=3, n_enum=8)
        return Config(4, "schema-B512-V152064", [sg.text], bpe_like_vocab(152064, 32, seed), 512, 256,
                      nest_cap=10, seed=seed, notes=dict(alternatives=[sg.n_alternatives]))
    if idx == 5:
        sgs = [G.schema_grammar(seed * 100 + i, *shape) for i, shape in enumerate(_CFG5_SHAPES)]
        return Config(5, "mixed8-B256-V128256", [s.text for s in sgs],
                      bpe_like_vocab(128256, 32, seed), 256, 512, nest_cap=10, mixed=True, seed=seed,
                      notes=dict(alternatives=[s.n_alternatives for s in sgs]))
    if idx == 6:
        return Config(6, "thought-json-B256-V128256", [G.THOUGHT_THEN_JSON], bpe_like_vocab(128256, 32, seed),
                      256, 256, nest_cap=10, seed=seed, marker=G.THOUGHT_THEN_JSON_MARKER, p_line_feed=0.125)
    if idx == 7:
        return Config(7, "json-right-recursive-B256-V128256", [G.JSON_RIGHT_RECURSIVE],
                      bpe_like_vocab(128256, 32, seed), 256, 256, nest_cap=10, seed=seed, compact=True)
    raise KeyError(idx)


def sequence_setup(cfg: Config):
    """(grammar index per sequence, target stack depth per sequence or None)."""
    if not cfg.mixed:
        return np.zeros(cfg.batch, dtype=np.int32), None
    rng = np.random.default_rng(cfg.seed + 7)
    return (rng.integers(0, len(cfg.grammars), size=cfg.batch).astype(np.int32),
            rng.integers(0, 65, size=cfg.batch).astype(np.int32))
