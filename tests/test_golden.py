"""The statements of the paper that a fixture can hold (tests/golden/paper_statements.txt, each
with its citation), checked against the oracle and, where they concern the compiled automaton,
against the library's host tables."""
import os

import pytest

from oracle import A_ACCEPT, T_END, GrammarError, Oracle
from paper_2506_03887_amd.binding import E_NOT_LR1, Pre3, Pre3Error
from workloads import grammars as G
from workloads.vocab import BASE_SEED, bpe_like_vocab

HERE = os.path.dirname(os.path.abspath(__file__))


def _records():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_statements.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, where, fact, data = [x.strip() for x in line.split(" ; ")]
        assert where and fact
        out[key] = data
    return out


REC = _records()


def test_palindromes_are_refused_by_both_builders():
    text = REC["palindromes_not_deterministic"] + "\n"
    with pytest.raises(GrammarError, match="not LR\\(1\\)"):
        Oracle(text)
    v = bpe_like_vocab(300, 4, BASE_SEED + 3)
    with pytest.raises(Pre3Error) as e:
        Pre3([text], v.bytes, v.offsets, v.eos_id, host_only=True)
    assert e.value.status == E_NOT_LR1


def test_digits_share_one_edge_class():
    text = REC["digits_form_one_edge"].replace(" / ", "\n") + "\n"
    v = bpe_like_vocab(300, 4, BASE_SEED + 3)
    lib = Pre3([text], v.bytes, v.offsets, v.eos_id, host_only=True)
    classes = {lib.byte_class(b) for b in b"0123456789"}
    assert len(classes) == 1
    assert lib.byte_class(ord("a")) not in classes


def test_accept_appears_once_and_only_under_end_of_input():
    for name in REC["accept_only_at_end_item"].split():
        o = Oracle(getattr(G, name))
        start = o.goto(0, o.nonterminal_index(o.production(1)[0]))    # GOTO(I0, S): holds [S' -> S . , $]
        cells = [(s, a) for s in range(o.n_states()) for a in range(257) if o.action(s, a)[0] == A_ACCEPT]
        assert cells == [(start, T_END)], name


def test_stack_lengths_follow_the_parsing_loop():
    o = Oracle(G.ARITHMETIC)
    for item in REC["reduce_pops_rhs_length"].split():
        prefix, want = item.rsplit("=", 1)
        rc, st = o.advance(o.initial_stack(), prefix.encode())
        assert rc == 0 and len(st) == int(want), (prefix, len(st))


def test_the_stack_starts_with_the_start_state_only():
    for name in REC["start_state_only_initially"].split():
        o = Oracle(getattr(G, name))
        assert o.initial_stack() == [o.initial_state(0)] == [0]


def test_a_complete_cycle_traversal_leaves_no_trace_on_the_stack():
    o, plain = Oracle(G.RIGHT_LIST, compact_cycles=True), Oracle(G.RIGHT_LIST)
    for item in REC["cycle_traversal_is_popped"].split():
        prefix, want = item.rsplit("=", 1)
        rc, st = o.advance(o.initial_stack(), prefix.encode())
        rc_p, st_p = plain.advance(plain.initial_stack(), prefix.encode())
        assert rc == rc_p == 0 and len(st) == int(want), (prefix, st)
        assert len(st_p) == len(prefix) + 1                         # the plain stack keeps every element
        for tail in (b"", b",x", b",", b"x", b",x,x", b",,"):       # equivalent state: same continuations
            a, b = o.advance(st, tail) if tail else (0, st), plain.advance(st_p, tail) if tail else (0, st_p)
            assert a[0] == b[0] and (a[0] != 0 or o.eos_allowed(a[1]) == plain.eos_allowed(b[1])), (prefix, tail)
