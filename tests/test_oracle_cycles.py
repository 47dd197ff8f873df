"""Pins of the oracle's cycle-aware stacks (Sec. 3.2.3; Alg. 1 step 1) and, on the same inputs, the
library's host tables.

What must hold, and what it is checked against:
  * which cycles are registered: hand-derived for two textbook grammars; none for nesting,
    and left recursion (dropping a traversal there would forget a depth);
  * soundness: a compacted stack accepts exactly the continuations of the text that produced
    it -- checked against the LR-free brute-force recogniser (every string up to a length
    bound, every split into text + continuation), on curated grammars and seeded random ones;
  * the right-recursive JSON grammar with compaction yields, byte for byte, the masks of the
    left-recursive JSON grammar (the same language), and its stacks stay bounded where the
    plain stacks grow with the input;
  * compacting after every token equals compacting the plain stack once (the normal form does
    not depend on when it is taken).
"""
import itertools
import json
import random

import numpy as np
import pytest

from cfg_brute import languages
from oracle import GrammarError, Oracle
from paper_2506_03887_amd.binding import Pre3, Pre3Error
from workloads import grammars as G
from workloads.vocab import Vocab

ALPHABET = "abc"

# right recursion in several shapes: through terminals and nonterminals, with a nullable tail,
# with unit and empty productions around it, two cycles that share their first state, a cycle
# of three states, and right recursion next to nesting
CURATED = {
    "list": 'S ::= "a" | "a" "b" S',
    "nullable_tail": 'S ::= A "c"\nA ::= "" | "a" A',
    "through_nonterminal": 'S ::= A "c"\nA ::= B A | B\nB ::= "a" | "b" "b"',
    "shared_head": 'S ::= A "c"\nA ::= "a" B A | "a" C A | "c"\nB ::= "b"\nC ::= "a"',
    "three_states": 'S ::= "a" "b" "c" S | "b"',
    "beside_nesting": 'S ::= "a" S "b" | A\nA ::= "c" A | "c"',
    "two_levels": 'S ::= A S | A\nA ::= "a" A | "b"',
    "unit_chain": 'S ::= A\nA ::= B\nB ::= "a" B | "c" | ""',
    "sibling_item": 'S ::= A "b"\nA ::= "a" A | "a" "c"',
}

# A -> a A | a a c : the loop state after two a's also holds  A -> a a . c , whose reduction pops
# THREE entries: a traversal under it is needed, so nothing may be registered
LOOP_WITH_A_DEEP_ITEM = 'S ::= A "b"\nA ::= "a" A | "a" "a" "c"'



def _byte_vocab():
    toks = [bytes([c]) for c in range(256)] + [b""]
    return Vocab(toks, 256)


def test_hand_derived_cycles():
    # L -> x | x , L : state 1 = after x, state 2 = L at the top level, state 3 = after the comma,
    # from which x leads back to 1; the traversal (1, 3) is one list element
    assert Oracle([G.RIGHT_LIST]).cycles() == [[1, 3]]
    # S -> C C, C -> c C | d : numbering I0 -c-> 1, -d-> 2, -S-> 3, -C-> 4; 1 -c-> 1, -C-> 5;
    # 4 -c-> 6, -d-> 7, -C-> 8; 6 -c-> 6.  The two c-loops (lookaheads {c,d} and {$}) are the cycles
    assert Oracle([G.DRAGON_CC]).cycles() == [[1], [6]]
    o = Oracle([G.RIGHT_LIST])
    rc, st = o.advance(o.initial_stack(), b"x,x,x,x")
    assert rc == 0 and st == [0, 1, 3, 1, 3, 1, 3, 1] and o.compact(st) == [0, 1]
    rc, st = o.advance(o.initial_stack(), b"x,x,x,")
    assert o.compact(st) == [0, 1, 3]
    assert o.compact([0]) == [0] and o.compact([0, 1]) == [0, 1]


@pytest.mark.parametrize("text", [G.ANBN, G.DYCK, G.ARITHMETIC, G.JSON, G.THOUGHT_THEN_JSON, LOOP_WITH_A_DEEP_ITEM])
def test_no_cycle_where_a_traversal_carries_information(text):
    assert Oracle([text]).cycles() == []


def _check_sound(text, n, v=None):
    """Every split of every string up to length n into text + continuation: the compacted stack of
    the text takes the continuation iff the brute-force recogniser says the whole is viable, and
    then ends a sentence iff the whole is one.  Returns how many stacks the compaction shortened."""
    o = Oracle([text])
    sentences, viable = languages(text, n)
    shortened = 0
    stacks = {}
    for p in sorted(viable, key=len):
        rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p.encode())
        assert rc == 0, (text, p)
        c = o.compact(st)
        assert c[-1] == st[-1] and c[0] == st[0] and len(c) <= len(st)
        assert o.compact(c) == c
        shortened += len(c) < len(st)
        stacks[p] = c
        if p:                                       # taken after every byte == taken once
            rc, inc = o.advance(stacks[p[:-1]], p[-1:].encode())
            assert rc == 0 and o.compact(inc) == c, (text, p)
    for k in range(1, n + 1):
        for tup in itertools.product(ALPHABET, repeat=k):
            w = "".join(tup)
            for cut in range(k):
                p, q = w[:cut], w[cut:]
                if p not in viable or (len(q) > 1 and w[:-1] not in viable):
                    continue                        # only the first byte that leaves the language matters
                rc, st = o.advance(stacks[p], q.encode())
                assert (rc == 0) == (w in viable), (text, p, q)
                if rc == 0:
                    assert o.eos_allowed(st) == (w in sentences), (text, p, q)
    return shortened


@pytest.mark.parametrize("name", sorted(CURATED))
def test_compacted_stacks_accept_what_brute_force_accepts(name):
    text = CURATED[name]
    o = Oracle([text])
    assert len(o.cycles()) >= 1, name
    assert _check_sound(text, 8) > 0, name


def test_shared_head_and_three_state_cycles_are_found():
    o = Oracle([CURATED["shared_head"]])
    heads = [c[0] for c in o.cycles()]
    assert len(heads) == 2 and heads[0] == heads[1] and [len(c) for c in o.cycles()] == [2, 2]
    assert [len(c) for c in Oracle([CURATED["three_states"]]).cycles()] == [3]
    # A -> a A | a c : the loop state also holds  A -> a . c  with the dot after ONE symbol: fine
    assert [len(c) for c in Oracle([CURATED["sibling_item"]]).cycles()] == [1]


def _random_right_recursive_grammar(rnd):
    nts = ["S", "A", "B"][: rnd.randint(2, 3)]
    lines = []
    for nt in nts:
        alts = []
        for _ in range(rnd.randint(1, 3)):
            syms = []
            for _ in range(rnd.randint(0, 3)):
                syms.append('"%s"' % rnd.choice(ALPHABET) if rnd.random() < 0.6 else rnd.choice(nts))
            if rnd.random() < 0.45 and syms:
                syms.append(nt)                     # right recursion
            alts.append(" ".join(syms) if syms else '""')
        lines.append("%s ::= %s" % (nt, " | ".join(alts)))
    return "\n".join(lines)


def test_random_grammars_compaction_is_sound_and_tables_agree():
    """Seeded random grammars with many right-recursive alternatives: soundness against brute force,
    and the library's registered cycles and host evaluation of its cycle tables against the oracle."""
    rnd = random.Random(2506_03887 + 3)
    v = _byte_vocab()
    with_cycles = shortened = tried = 0
    while with_cycles < 25 and tried < 6000:
        tried += 1
        text = _random_right_recursive_grammar(rnd)
        try:
            o = Oracle([text])
        except GrammarError:
            continue
        if not o.cycles() or len(languages(text, 6)[1]) < 5:
            continue
        with_cycles += 1
        shortened += _check_sound(text, 6) > 0
        lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=1, stack_cap=64, host_only=True)
        assert lib.reduction_cycles() == o.cycles(), text
        for p in sorted(languages(text, 6)[1]):
            rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p.encode())
            assert lib.debug_compact(st) == o.compact(st), (text, p)
    assert with_cycles >= 25 and shortened >= 15, (with_cycles, shortened, tried)


def test_library_registers_the_same_cycles_and_normal_forms():
    v = _byte_vocab()
    texts = [G.RIGHT_LIST, G.DRAGON_CC, G.EPSILON_MIX, G.RIGHT_LINEAR, G.JSON_RIGHT_RECURSIVE, G.JSON] + list(CURATED.values())
    for text in texts:
        o = Oracle([text])
        lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=1, host_only=True)
        assert lib.reduction_cycles() == o.cycles(), text
    # several grammars: global state ids
    o = Oracle([G.JSON, G.RIGHT_LIST, G.DRAGON_CC])
    lib = Pre3([G.JSON, G.RIGHT_LIST, G.DRAGON_CC], v.bytes, v.offsets, v.eos_id, max_token_len=1, host_only=True)
    want = o.cycles(0) + o.cycles(1) + o.cycles(2)
    assert lib.reduction_cycles() == want and len(want) == 3 and want[0][0] == o.initial_state(1) + 1
    rc, st = o.advance(o.initial_stack(1), b"x,x,x")
    assert lib.debug_compact(st) == o.compact(st) == st[:2]
    with pytest.raises(Pre3Error):
        Pre3([G.RIGHT_LIST], v.bytes, v.offsets, v.eos_id, max_token_len=1, stack_cap=8192, host_only=True,
             compact_cycles=True)


def _small_json_vocab():
    rnd = random.Random(5)
    toks = [bytes([c]) for c in range(256)]
    pieces = ['{"', '":', '",', '"}', '[[', ']]', '],', '},', 'true', 'false', 'null', 'ab', '12', '0.5', 'e+', ' ', '  ', '\n ',
              '\\"', '\\u00', 'a"', '",\n "', '[1,', '1,2', ', ', '": "', 'xyz', '}]', '":{"', '[]', '{}', '-1', '1e5', '"a"', ':[']
    toks += [p.encode() for p in pieces]
    toks += [bytes(rnd.choice(b'ab1 ,"[]{}:') for _ in range(rnd.randint(2, 4))) for _ in range(200)]
    toks.append(b"")
    return Vocab(toks, len(toks) - 1)


def test_right_recursive_json_with_compaction_equals_left_recursive_json():
    """Two grammars of one language: the masks must agree at every byte although the stacks have
    nothing in common; with compaction the right-recursive stacks stay bounded."""
    left, right = Oracle([G.JSON]), Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    plain = Oracle([G.JSON_RIGHT_RECURSIVE])
    assert len(right.cycles()) >= 10
    v = _small_json_vocab()
    rnd = random.Random(9)
    doc = {"name": "x" * 300, "list": list(range(120)), "deep": [[[{"k": [1.5e3, -2, "s\\\"\n"]}]]],
           "nested": {"a": {"b": {"c": ["y" * 50] * 20}}}, "ws": None}
    data = json.dumps(doc, indent=1).encode()
    sl, sr, sp = left.initial_stack(), right.initial_stack(), plain.initial_stack()
    longest_r = longest_p = 0
    for i in range(len(data)):
        if i % 7 == 0 or i > len(data) - 40:
            ml, mr = left.mask_row(sl, v), right.mask_row(sr, v)
            assert (ml == mr).all(), (i, data[max(0, i - 20): i])
            assert (plain.mask_row(sp, v) == mr).all()
        step = data[i: i + 1]
        rc1, sl = left.advance(sl, step)
        rc2, sr = right.advance(sr, step)
        rc3, sp = plain.advance(sp, step)
        assert rc1 == rc2 == rc3 == 0
        assert plain.compact(sp) == sr                          # incremental == all at once
        longest_r, longest_p = max(longest_r, len(sr)), max(longest_p, len(sp))
    assert left.eos_allowed(sl) and right.eos_allowed(sr)
    assert longest_p > 330 and longest_r < 80, (longest_p, longest_r)
    # whole tokens, random walk, jump-forward
    for _ in range(30):
        sl, sr = left.initial_stack(), right.initial_stack()
        for _ in range(40):
            ml = left.mask_row(sl, v)
            assert (ml == right.mask_row(sr, v)).all()
            ids = np.flatnonzero(((ml[np.arange(v.n_tokens) >> 5] >> (np.arange(v.n_tokens) & 31).astype(np.uint32)) & 1))
            ids = ids[ids != v.eos_id]
            t = int(ids[rnd.randrange(len(ids))])
            rc1, sl = left.advance(sl, v.tokens[t])
            rc2, sr = right.advance(sr, v.tokens[t])
            assert rc1 == rc2 == 0
            assert left.jump_forward(sl, 8)[0] == right.jump_forward(sr, 8)[0]


def test_a_list_of_any_length_keeps_a_bounded_stack():
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    plain = Oracle([G.JSON_RIGHT_RECURSIVE])
    st = o.initial_stack()
    rc, st = o.advance(st, b'["')
    for _ in range(500):
        rc, st = o.advance(st, b"abcdefgh", cap=64)
        assert rc == 0 and len(st) < 16
    rc, st = o.advance(st, b'"', cap=64)
    for _ in range(500):
        rc, st = o.advance(st, b", 12345678", cap=64)
        assert rc == 0 and len(st) < 16
    rc, st = o.advance(st, b"]", cap=64)
    assert rc == 0 and o.eos_allowed(st)
    rc, _ = plain.advance(plain.initial_stack(), b'["' + b"abcdefgh" * 20, cap=64)
    assert rc == 2                                              # the plain stack overflows


def _row_after_traversal_only_reduces(o, cycle):
    """For a registered cycle v1..vn of A -> X1..Xn A: the state r = GOTO(vn, A) must do nothing but
    reduce by that production (its kernel holds the finished item only), on at least one lookahead."""
    from oracle import A_ERROR, A_REDUCE
    n, vn = len(cycle), cycle[-1]
    found = 0
    for A in range(o.n_nonterminals()):
        r = o.goto(vn, A)
        if r < 0:
            continue
        acts = [o.action(r, a) for a in range(257)]
        live = {x for x in acts if x[0] != A_ERROR}
        if len(live) == 1:
            (kind, p), = live
            if kind == A_REDUCE and o.production(p) == (o.production(p)[0], n + 1) and o.nonterminal_index(o.production(p)[0]) == A:
                found += 1
    return found == 1


def test_after_a_traversal_and_its_nonterminal_the_parser_can_only_reduce_the_cycles_production():
    """The cycles are registered on a condition on v1 alone; that the state after vn and A then holds only
    the finished production (which the soundness argument uses) follows for conflict-free canonical LR(1)
    tables.  Checked here on the ACTION tables of the curated grammars, the right-recursive JSON grammar
    and 150 seeded random grammars with cycles."""
    texts = [G.RIGHT_LIST, G.DRAGON_CC, G.JSON_RIGHT_RECURSIVE] + list(CURATED.values())
    rnd = random.Random(2506_03887 + 11)
    tried = 0
    while len(texts) < 165 and tried < 40000:
        tried += 1
        text = _random_right_recursive_grammar(rnd)
        try:
            if Oracle([text]).cycles():
                texts.append(text)
        except GrammarError:
            pass
    assert len(texts) >= 165
    n_cycles = 0
    for text in texts:
        o = Oracle([text])
        for cyc in o.cycles():
            assert _row_after_traversal_only_reduces(o, cyc), (text, cyc)
            n_cycles += 1
    assert n_cycles >= 200, n_cycles
