"""Pins of the oracle's canonical LR(1) construction (paper App. A.2) against
hand-derived tables, textbook state counts and conflict detection."""
import pytest

from oracle import A_ACCEPT, A_ERROR, A_REDUCE, A_SHIFT, T_END, GrammarError, Oracle
from workloads import grammars as G

c, d = ord("c"), ord("d")


def test_dragon_cc_collection_by_hand():
    """S -> C C, C -> c C | d.  Derived by hand with CLOSURE/GOTO, numbering states breadth
    first with terminals ('c' < 'd') before nonterminals (S, C):
      I0 = {S'->.S,$  S->.CC,$  C->.cC,c/d  C->.d,c/d}            6 items
      I1 = GOTO(I0,c) = {C->c.C,c/d  C->.cC,c/d  C->.d,c/d}        6
      I2 = GOTO(I0,d) = {C->d.,c/d}                                2
      I3 = GOTO(I0,S) = {S'->S.,$}                                 1
      I4 = GOTO(I0,C) = {S->C.C,$  C->.cC,$  C->.d,$}              3
      GOTO(I1,c)=I1  GOTO(I1,d)=I2  I5 = GOTO(I1,C) = {C->cC.,c/d} 2
      I6 = GOTO(I4,c) = {C->c.C,$  C->.cC,$  C->.d,$}              3
      I7 = GOTO(I4,d) = {C->d.,$}                                  1
      I8 = GOTO(I4,C) = {S->CC.,$}                                 1
      GOTO(I6,c)=I6  GOTO(I6,d)=I7  I9 = GOTO(I6,C) = {C->cC.,$}   1
    Productions: 0 S'->S, 1 S->CC, 2 C->cC, 3 C->d."""
    o = Oracle(G.DRAGON_CC)
    assert o.n_states() == 10
    assert [o.n_items(s) for s in range(10)] == [6, 6, 2, 1, 3, 2, 3, 1, 1, 1]
    assert [o.production(p) for p in range(4)] == [("$accept", 1), ("S", 2), ("C", 2), ("C", 1)]
    S, C = o.nonterminal_index("S"), o.nonterminal_index("C")
    sh, rd, acc = A_SHIFT, A_REDUCE, A_ACCEPT
    expect = {
        0: {c: (sh, 1), d: (sh, 2)},
        1: {c: (sh, 1), d: (sh, 2)},
        2: {c: (rd, 3), d: (rd, 3)},
        3: {T_END: (acc, 0)},
        4: {c: (sh, 6), d: (sh, 7)},
        5: {c: (rd, 2), d: (rd, 2)},
        6: {c: (sh, 6), d: (sh, 7)},
        7: {T_END: (rd, 3)},
        8: {T_END: (rd, 1)},
        9: {T_END: (rd, 2)},
    }
    for s in range(10):
        for a in range(257):
            kind, arg = o.action(s, a)
            if a in expect[s]:
                assert (kind, arg) == expect[s][a], (s, a)
            else:
                assert kind == A_ERROR, (s, a)
    gotos = {(0, S): 3, (0, C): 4, (1, C): 5, (4, C): 8, (6, C): 9}
    for s in range(10):
        for A in (S, C):
            assert o.goto(s, A) == gotos.get((s, A), -1)


def test_arithmetic_has_22_canonical_states():
    """The expression grammar E->E+T|T, T->T*F|F, F->(E)|a has 22 canonical LR(1) item sets
    (its LALR/SLR automaton has 12): the textbook count for this grammar."""
    o = Oracle(G.ARITHMETIC)
    assert o.n_states() == 22
    assert o.n_productions() == 7
    # I0 by hand: S'->.E,$ ; E->.E+T and E->.T with lookaheads {$,+} ; T->.T*F, T->.F with
    # {$,+,*} ; F->.(E), F->.a with {$,+,*}  => 1 + 2*2 + 2*3 + 2*3 = 17 items
    assert o.n_items(0) == 17
    # shifts out of I0 in terminal order '(' (40) then 'a' (97), then GOTO on E, T, F
    assert o.action(0, ord("(")) == (A_SHIFT, 1)
    assert o.action(0, ord("a")) == (A_SHIFT, 2)
    assert [o.goto(0, o.nonterminal_index(n)) for n in "ETF"] == [3, 4, 5]
    assert o.action(3, T_END) == (A_ACCEPT, 0)
    # the state after 'a' at top level reduces F->a on $,+,* only
    for a in range(257):
        kind, arg = o.action(2, a)
        if a in (T_END, ord("+"), ord("*")):
            assert (kind, o.production(arg)) == (A_REDUCE, ("F", 1))
        else:
            assert kind == A_ERROR
    # the state after '(' 'a' is a different item set: it reduces on ')' instead of '$'
    inner_a = o.action(1, ord("a"))[1]
    assert inner_a != 2
    assert o.action(inner_a, ord(")"))[0] == A_REDUCE and o.action(inner_a, T_END)[0] == A_ERROR


def test_lr1_but_not_lalr_grammar_is_accepted():
    """S -> aEa | bEb | aFb | bFa, E -> e, F -> e is LR(1) but not LALR(1): merging item sets
    with equal cores would create a reduce/reduce conflict, so it pins that states are
    told apart by their lookaheads."""
    text = 'S ::= "a" E "a" | "b" E "b" | "a" F "b" | "b" F "a"\nE ::= "e"\nF ::= "e"\n'
    o = Oracle(text)
    for w, ok in [(b"aea", True), (b"beb", True), (b"aeb", True), (b"bea", True), (b"aee", False), (b"ae", False)]:
        assert o.accepts(w) == ok
    # after "ae" the reduction depends on the lookahead: 'a' -> E, 'b' -> F
    rc, st = o.advance(o.initial_stack(), b"ae")
    assert rc == 0
    ka, pa = o.action(st[-1], ord("a"))
    kb, pb = o.action(st[-1], ord("b"))
    assert ka == kb == A_REDUCE and o.production(pa)[0] == "E" and o.production(pb)[0] == "F"


@pytest.mark.parametrize("text", [G.AMBIGUOUS, G.PALINDROME,
                                  'S ::= A | B\nA ::= "x"\nB ::= "x"\n'])
def test_conflicts_are_reported(text):
    with pytest.raises(GrammarError, match="not LR\\(1\\)"):
        Oracle(text)


@pytest.mark.parametrize("text,msg", [
    ('S ::= "a" | S B\nB ::= B "b"\n', "derives no string"),
    ('S ::= "a"\nB ::= "b"\n', "unreachable"),
    ('S ::= "a" C\n', "undefined"),
    ('S ::= "a" [bc]\n', "whole alternative"),
    ('S ::= "a\n', "unterminated"),
    ('S ::= \n', "empty alternative"),
])
def test_malformed_grammars_are_rejected(text, msg):
    with pytest.raises(GrammarError, match=msg):
        Oracle(text)


def test_class_is_sugar_for_one_production_per_byte():
    a = Oracle('S ::= D | S D\nD ::= [0-2]\n')
    b = Oracle('S ::= D | S D\nD ::= "0" | "1" | "2"\n')
    assert a.n_states() == b.n_states() and a.n_productions() == b.n_productions() == 6
    for s in range(a.n_states()):
        for t in range(257):
            assert a.action(s, t) == b.action(s, t)
    neg = Oracle('S ::= [^\\x00-\\x2f\\x33-\\xff]\n')          # == [0-2]
    assert [neg.accepts(bytes([x])) for x in b"/0123"] == [False, True, True, True, False]


def test_multi_grammar_union_offsets_state_ids():
    o = Oracle([G.DRAGON_CC, G.ARITHMETIC, G.DYCK])
    assert [o.n_states(g) for g in range(3)] == [10, 22, 8]
    assert [o.initial_state(g) for g in range(3)] == [0, 10, 32]
    assert o.n_states_total() == 40
    single = Oracle(G.ARITHMETIC)
    rc1, st1 = single.advance(single.initial_stack(), b"(a+a")
    rc2, st2 = o.advance(o.initial_stack(1), b"(a+a")
    assert rc1 == rc2 == 0 and [s + 10 for s in st1] == st2
    assert o.allowed(st2, b")*(") and not o.allowed(st2, b"))")
    assert not o.allowed(o.initial_stack(0), b"(")          # grammar 0 has no parentheses
