"""Seeded random tiny grammars.  Those that both independent LR(1) builders accept are checked
three ways: the oracle against the LR-free brute-force recogniser (all strings up to length 6),
the library's compiled tables against the oracle's tables, and the library's merged reduction
edges and token-level edges (host evaluation of the same tables the GPU reads) against the
oracle's parse loop.  Both sides must also agree on WHICH grammars are LR(1)."""
import itertools
import random

import numpy as np

from cfg_brute import languages
from oracle import GrammarError, Oracle
from paper_2506_03887_amd.binding import E_NOT_LR1, E_PARSE, Pre3, Pre3Error
from workloads.vocab import Vocab

N = 6
ALPHABET = "abc"


def random_grammar(rnd):
    nts = ["S", "A", "B"][: rnd.randint(2, 3)]
    lines = []
    for nt in nts:
        alts = []
        for _ in range(rnd.randint(1, 3)):
            syms = []
            for _ in range(rnd.randint(0, 3)):
                if rnd.random() < 0.55:
                    syms.append('"%s"' % rnd.choice(ALPHABET))
                else:
                    syms.append(rnd.choice(nts))
            alts.append(" ".join(syms) if syms else '""')
        lines.append("%s ::= %s" % (nt, " | ".join(alts)))
    return "\n".join(lines)


def _vocab():
    toks = ["".join(t).encode() for k in (1, 2, 3) for t in itertools.product(ALPHABET + "x", repeat=k)] + [b""]
    return Vocab(toks, len(toks) - 1)


def _row_bits(row, V):
    return ((row[np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1).astype(bool)


def test_random_grammars_three_ways():
    rnd = random.Random(2506_03887)
    v = _vocab()
    V = v.n_tokens
    accepted = rejected = 0
    tried = 0
    while accepted < 40 and tried < 4000:
        tried += 1
        text = random_grammar(rnd)
        try:
            o = Oracle(text)
            oracle_status = "ok"
        except GrammarError as e:
            oracle_status = str(e)
        try:
            lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=3, stack_cap=64, host_only=True)
            lib_status = "ok"
        except Pre3Error as e:
            lib_status = e.status
        # the two builders agree on acceptance (not LR(1), useless or undefined symbols are refused by both)
        assert (oracle_status == "ok") == (lib_status == "ok"), (text, oracle_status, lib_status)
        if oracle_status != "ok":
            assert lib_status in (E_NOT_LR1, E_PARSE), (text, lib_status)
            rejected += 1
            continue
        sentences, viable = languages(text, N)
        if len(viable) < 4:
            continue
        accepted += 1
        assert lib.n_states == o.n_states(0), text
        assert lib.validate_tables() == 0, text
        for p in sorted(viable):
            rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p.encode())
            assert rc == 0, (text, p)
            # 1. oracle == brute force
            assert o.eos_allowed(st) == (p in sentences), (text, p)
            want = _row_bits(o.mask_row(st, v), V)
            for t in range(V - 1):
                tok = v.tokens[t].decode()
                if len(p) + len(tok) <= N:
                    assert want[t] == ((p + tok) in viable), (text, p, tok)
            assert want[V - 1] == (p in sentences)
            # 2. token-level edges == oracle row
            ok, row, walk = lib.debug_resolve_row(np.array(st, dtype=np.int32))
            if ok:
                got = _row_bits(row, V)
                left = np.zeros(V, dtype=bool)
                left[walk] = True
                assert (got[~left] == want[~left]).all() and not (got & left).any(), (text, p)
            # 3. merged reduction edges and per-step edges == oracle advance
            for t in rnd.sample(range(V - 1), 12):
                rc_o, st_o = o.advance(st, v.tokens[t], cap=64)
                for merged in (True, False):
                    rc_l, st_l = lib.debug_advance(st, v.tokens[t], cap=64, merged=merged)
                    assert rc_l == rc_o and (rc_o != 0 or list(st_l) == list(st_o)), (text, p, v.tokens[t], merged)
    assert accepted >= 40 and rejected >= 10, (accepted, rejected, tried)


def test_both_sides_read_the_same_grammar_texts():
    """The grammar text format is specified once and implemented twice: seeded random edits of valid
    texts (deleted, inserted, replaced characters: quotes, brackets, bars, escapes, comments, line
    breaks) must be accepted or refused by both, and where accepted give automata of the same size."""
    from workloads import grammars as G
    rnd = random.Random(2506_03887 + 9)
    v = Vocab([bytes([c]) for c in range(256)] + [b""], 256)
    bases = [G.ARITHMETIC, G.RIGHT_LIST, G.EPSILON_MIX, G.DYCK, 'S ::= [a-c] S | "x" # c\n',
             'S ::= A\n  | "q"\nA ::= [^a-y] | "\\x41\\n"\n', G.JSON]
    alphabet = '"[]|:=\\ \n#^-ax1S'
    accepted = refused = 0
    for _ in range(2500):
        t = list(rnd.choice(bases))
        for _ in range(rnd.randint(1, 3)):
            kind, pos = rnd.randrange(3), rnd.randrange(len(t) + 1)
            if kind == 0 and t:
                del t[min(pos, len(t) - 1)]
            elif kind == 1:
                t.insert(pos, rnd.choice(alphabet))
            elif t:
                t[min(pos, len(t) - 1)] = rnd.choice(alphabet)
        text = "".join(t)
        try:
            n_oracle = Oracle([text]).n_states(0)
        except GrammarError:
            n_oracle = None
        try:
            n_lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=1, host_only=True, token_edges=False).n_states
        except Pre3Error:
            n_lib = None
        assert n_oracle == n_lib, (text, n_oracle, n_lib)
        accepted += n_oracle is not None
        refused += n_oracle is None
    assert accepted > 150 and refused > 1500, (accepted, refused)
