"""Host logic of the library, checked on the CPU: the compiled DPDA edge tables against the
oracle's ACTION/GOTO tables, byte-class aggregation, error statuses, exported symbols."""
import ctypes
import os
import re

import pytest

from oracle import A_ACCEPT, A_ERROR, A_REDUCE, A_SHIFT, Oracle
from paper_2506_03887_amd import binding
from paper_2506_03887_amd.binding import Pre3, Pre3Error
from workloads import grammars as G
from workloads.vocab import BASE_SEED, bpe_like_vocab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def vocab():
    return bpe_like_vocab(2000, 12, BASE_SEED + 50)


def host_compile(grammars, vocab, **kw):
    return Pre3(grammars, vocab.bytes, vocab.offsets, vocab.eos_id, host_only=True, **kw)


def test_header_symbols_are_exported():
    header = open(os.path.join(ROOT, "include", "pre3.h")).read()
    declared = set(re.findall(r"\b(pre3_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("texts", [
    [G.JSON], [G.schema_grammar(11, 6, 2, 4).text, G.JSON], [G.JSON_RIGHT_RECURSIVE, G.schema_grammar(13, 8, 1, 5).text],
    ['S ::= "%s" T "%s"\nT ::= "x" | "y"' % ("abcdefghij" * 10, "0123456789" * 7)],
])
def test_forced_runs_are_the_shift_only_chains_of_the_oracle_tables(texts, vocab):
    """The multi-symbol edges of jump-forward (Sec. 3.3) against the oracle's ACTION table: a state starts a
    run exactly if its only action, over all 256 bytes and the end of input, is one shift; the run follows
    such shifts byte by byte and target by target, for at most 64 steps, and ends where the next state has
    another action (or the limit is reached)."""
    o = Oracle(texts)
    p = host_compile(texts, vocab)

    def only_shift(g, s):
        acts = [(a,) + o.action(s, a, g) for a in range(257)]
        live = [x for x in acts if x[1] != A_ERROR]
        return (live[0][0], live[0][2]) if len(live) == 1 and live[0][1] == A_SHIFT else None

    with_run = longest = 0
    for g in range(len(texts)):
        off = o.initial_state(g)
        for s in range(o.n_states(g)):
            want_bytes, want_states, at = [], [], s
            while len(want_bytes) < 64 and only_shift(g, at) is not None:
                a, at = only_shift(g, at)
                want_bytes.append(a)
                want_states.append(at + off)
            got_bytes, got_states = p.forced_run(off + s)
            assert list(got_bytes) == want_bytes and got_states == want_states, (g, s)
            with_run += bool(want_bytes)
            longest = max(longest, len(want_bytes))
    assert with_run > 0
    if len(texts) == 1 and texts[0].startswith("S ::="):
        assert longest == 64 and p.forced_run(p.initial_state(0))[0] == ("abcdefghij" * 10)[:64].encode()


@pytest.mark.parametrize("texts", [
    [G.ARITHMETIC], [G.JSON], [G.EPSILON_MIX, G.DYCK, G.ARITHMETIC],
    [G.schema_grammar(11, 6, 2, 4).text, G.JSON],
])
def test_edge_tables_equal_oracle_tables(texts, vocab):
    """Same canonical collection, same state numbering, same actions: every (state, symbol)
    cell and every goto of the library equals the oracle's."""
    o = Oracle(texts)
    p = host_compile(texts, vocab)
    assert p.n_grammars == len(texts) and p.n_states == o.n_states_total()
    for g in range(len(texts)):
        off = o.initial_state(g)
        assert p.initial_state(g) == off
        names = [o.production(q, g)[0] for q in range(o.n_productions(g))]
        lhs_index = {n: o.nonterminal_index(n, g) for n in set(names)}
        for s in range(o.n_states(g)):
            for a in range(257):
                kind, arg = o.action(s, a, g)
                got = p.edge(off + s, a)
                if kind == A_ERROR:
                    assert got[0] == 0
                elif kind == A_SHIFT:
                    assert got[:2] == (1, arg + off), (g, s, a)
                elif kind == A_REDUCE:
                    name, n = o.production(arg, g)
                    assert got == (2, n, lhs_index[name]), (g, s, a)
                else:
                    assert kind == A_ACCEPT and got[0] == 3 and a == 256
            for A in range(o.n_nonterminals(g)):
                t = o.goto(s, A, g)
                assert p.goto_target(off + s, A) == (t + off if t >= 0 else -1)


def test_byte_classes_aggregate_digits_and_plain_characters(vocab):
    """Sec. 3.3 edge aggregation: bytes with identical edges share a class - the digits of
    a number grammar collapse into one class, and so do the plain string characters."""
    p = host_compile(G.JSON, vocab)
    assert len({p.byte_class(c) for c in b"123456789"}) == 1
    assert p.byte_class(ord("0")) != p.byte_class(ord("1"))          # JSON forbids leading zeros
    n = host_compile('N ::= D | N D\nD ::= [0-9]\n', vocab)           # the paper's example: digits 0-9 -> one edge
    assert len({n.byte_class(c) for c in b"0123456789"}) == 1 and n.n_byte_classes == 2
    plain = [c for c in range(0x20, 0x100) if c not in b'"\\/bfnrtu0123456789abcdefABCDEF+-.eE{}[]:, truefalsn']
    assert len({p.byte_class(c) for c in plain}) == 1
    assert len({p.byte_class(c) for c in b"\t\n\r"}) == 1                         # white space only
    assert p.byte_class(ord(" ")) not in (p.byte_class(9), p.byte_class(ord("x")))  # also a string character
    assert len({p.byte_class(c) for c in range(0x20) if c not in b"\t\n\r"}) == 1  # control bytes: no edges
    assert p.n_byte_classes < 40
    a = host_compile(G.ARITHMETIC, vocab)
    assert a.n_byte_classes == 6                                      # a + * ( ) and "everything else"


@pytest.mark.parametrize("text,status", [
    (G.AMBIGUOUS, binding.E_NOT_LR1), (G.PALINDROME, binding.E_NOT_LR1),
    ('S ::= "a" | S B\nB ::= B "b"\n', binding.E_PARSE), ('S ::= "a"\nB ::= "b"\n', binding.E_PARSE),
    ('S ::= "a" C\n', binding.E_PARSE), ('S ::= "a" [bc]\n', binding.E_PARSE),
    ('S ::= "a\n', binding.E_PARSE), ('S ::= \n', binding.E_PARSE), ("", binding.E_PARSE),
    ('S ::= "\\q"\n', binding.E_PARSE),
])
def test_compile_errors(text, status, vocab):
    with pytest.raises(Pre3Error) as e:
        host_compile(text, vocab)
    assert e.value.status == status and len(str(e.value)) > 20


def test_argument_errors(vocab):
    with pytest.raises(Pre3Error) as e:
        host_compile(G.JSON, vocab, max_token_len=4)
    assert e.value.status == binding.E_TOKEN_TOO_LONG
    with pytest.raises(Pre3Error) as e:
        Pre3(G.JSON, vocab.bytes, vocab.offsets, vocab.n_tokens, host_only=True)       # eos out of range
    assert e.value.status == binding.E_BADARG
    p = host_compile(G.JSON, vocab)
    lib = binding.load()
    # device calls on a host-only handle are refused, as are null pointers
    st = binding._Stacks(1, 1, 8, 1)
    assert lib.pre3_fill_mask(p._h, 1, st, 1, None) == binding.E_BADARG
    assert lib.pre3_advance(p._h, 1, None) == binding.E_BADARG
    assert lib.pre3_bind_state(p._h, 1, st, 1) == binding.E_BADARG
    assert lib.pre3_apply_mask(None, None, 1, 1, 1, None) == binding.E_BADARG
    assert lib.pre3_apply_mask(None, None, 0, 1, 1, None) == 0                          # empty batch: nothing to do
    assert lib.pre3_apply_mask(16, 16, 1, 8, 4, None) == binding.E_BADARG               # stride < vocab
    assert lib.pre3_initial_state(p._h, 1) == binding.E_BADARG
    assert lib.pre3_free(None) == 0
    assert lib.pre3_last_error(None) == b"null handle"


def test_walk_depth_bound_covers_deep_tokens(vocab):
    """The private-stack bound must cover the deepest walk: '[' pushes two states ('[' and the
    empty white space), so k brackets need 2k entries."""
    o = Oracle(G.JSON)
    p = host_compile(G.JSON, vocab, max_token_len=12)
    rc, st = o.advance(o.initial_stack(), b"[" * vocab.max_len)
    assert rc == 0 and p.walk_depth_bound >= len(st) - 1


@pytest.mark.parametrize("texts,prefixes", [
    ([G.JSON], [b"", b'{"a', b"[1", b'{"k": [tr', b"[[[[", b'"x\\', b"12.5e", b" 7 ", b'{"a":{"b":[{},[[]],"', b"[[1,2],[3"]),
    ([G.ARITHMETIC, G.DYCK], [b"", b"(a+a", b"((a*(a", b"a+a*a"]),
])
def test_merged_reduction_edges_equal_oracle_advance(texts, prefixes, vocab):
    """Alg. 1 step 3: every reduction chain collapsed into one edge with a stack-matching
    condition.  The host mirror of the device walk, with merged edges and with one reduction
    step at a time, must reproduce the oracle's advance (result code and stack) and its EOS test."""
    import random
    o = Oracle(texts)
    p = host_compile(texts, vocab)
    stats = p.symbol_edge_stats()
    assert stats["built"] == 1 and stats["nodes"] >= p.n_states
    rnd = random.Random(4)
    n_ok = 0
    for prefix in prefixes:
        rc, st = (0, o.initial_stack()) if not prefix else o.advance(o.initial_stack(), prefix)
        assert rc == 0
        assert (p.debug_advance(st, b"", end=True)[0] == 0) == o.eos_allowed(st)
        toks = [vocab.tokens[rnd.randrange(vocab.n_tokens - 1)] for _ in range(300)]
        toks += [b"]", b"}", b"]]", b'"', b'",', b"1", b",", b" ", b"]]]]", b"[" * 12, b")", b"))", b"+a", b""]
        for tok in toks:
            for cap in (len(st) + 3, len(st) + 64):
                want = o.advance(st, tok, cap=cap) if tok else (1, st)
                for merged in (True, False):
                    got = p.debug_advance(st, tok, cap=cap, merged=merged)
                    assert got[0] == want[0], (prefix, tok, cap, merged)
                    if want[0] == 0:
                        assert got[1] == want[1], (prefix, tok, cap, merged)
                        n_ok += 1
    assert n_ok > 30


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, vocab):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "paper_2506_03887_amd", "no_such_libpre3.so"))
    with pytest.raises(ImportError):
        Pre3([G.ARITHMETIC], vocab.bytes, vocab.offsets, vocab.eos_id, host_only=True)


def test_device_calls_refuse_a_host_only_handle(vocab):
    p = host_compile([G.ARITHMETIC], vocab)
    lib = binding.load()
    null = ctypes.c_void_p(0)
    assert lib.pre3_advance(p._h, null, null) == binding.E_BADARG
    assert lib.pre3_advance_fill_mask(p._h, null, null, 0, null) == binding.E_BADARG
    assert lib.pre3_apply_mask_argmax(p._h, null, 0, null, null, null) == binding.E_BADARG


@pytest.mark.parametrize("cfg_idx", [1, 2, 3, 4, 5, 6, 7])
def test_compiled_tables_are_internally_consistent(cfg_idx):
    """The kernels follow table contents without range checks: every index in the tables of the
    workload configurations must stay inside its table (with each merging level on and off)."""
    from workloads import configs
    cfg = configs.get(cfg_idx)
    v = cfg.vocab
    for kw in (dict(), dict(max_condition_depth=2), dict(merged_reductions=False, token_edges=False)):
        p = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), host_only=True,
                 compact_cycles=cfg.compact, **kw)
        assert p.validate_tables() == 0
