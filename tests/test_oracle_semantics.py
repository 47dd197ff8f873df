"""Pins of what the oracle decides: 'token allowed' == 'text stays a prefix of a sentence',
'EOS allowed' == 'text is a sentence' (paper Sec. 1 mask semantics; App. A.2 parse loop)."""
import itertools
import json
import random
import re

import numpy as np
import pytest

from cfg_brute import languages
from oracle import Oracle, apply_mask, masked_argmax, masked_topk
from workloads import grammars as G
from workloads.vocab import BASE_SEED, arithmetic_vocab, bf16_logits, bpe_like_vocab

N = 8


def _stack_after(o, text):
    rc, st = o.advance(o.initial_stack(), text.encode()) if text else (0, o.initial_stack())
    return rc, st


@pytest.mark.parametrize("name,alphabet,max_tok", [
    ("ARITHMETIC", "a+*()b", 3), ("DYCK", "()x", 3), ("ANBN", "abx", 3),
    ("RIGHT_LIST", "x,y", 3), ("EPSILON_MIX", "abcx", 3), ("RIGHT_LINEAR", "abcd", 3),
    ("DRAGON_CC", "cdx", 3),
])
def test_brute_force_all_strings_up_to_8(name, alphabet, max_tok):
    """Every string of length <= 8 over the grammar's alphabet plus one foreign byte: the set of
    sentences and the set of viable prefixes come from an LR-free set-of-strings fixpoint on
    the raw productions.  For every viable prefix p and every token t with |p.t| <= 8 the
    oracle must allow t exactly when p.t is again a viable prefix, and must allow EOS exactly
    when p is a sentence."""
    text = getattr(G, name)
    o = Oracle(text)
    sentences, viable = languages(text, N)
    assert len(sentences) > 3
    tokens = ["".join(t) for k in range(1, max_tok + 1) for t in itertools.product(alphabet, repeat=k)]
    n_checked = 0
    for p in sorted(viable):
        rc, st = _stack_after(o, p)
        assert rc == 0, p
        assert o.eos_allowed(st) == (p in sentences), p
        for t in tokens:
            if len(p) + len(t) > N:
                continue
            assert o.allowed(st, t.encode()) == ((p + t) in viable), (p, t)
            n_checked += 1
    assert n_checked > 200
    # strings that are not viable cannot be advanced by at all
    for k in range(1, 5):
        for w in itertools.product(alphabet, repeat=k):
            w = "".join(w)
            assert (_stack_after(o, w)[0] == 0) == (w in viable), w


def test_dyck_equals_counter():
    o = Oracle(G.DYCK)
    rnd = random.Random(1)
    for _ in range(3000):
        n = rnd.randint(0, 40)
        w = "".join(rnd.choice("()") if rnd.random() < 0.97 else "x" for _ in range(n))
        depth, viable = 0, True
        for ch in w:
            depth += {"(": 1, ")": -1}.get(ch, -10 ** 6)
            if depth < 0:
                viable = False
                break
        rc, st = _stack_after(o, w)
        assert (rc == 0) == viable, w
        if viable:
            assert o.eos_allowed(st) == (depth == 0), w
            # S -> eps | S ( S ): every open level holds the two states of "S (" above s0; a
            # text ending in ')' still carries the unreduced "S ( S )" of the last group
            # (reductions wait for the next lookahead)
            expect = 1 if not w else (1 + 2 * depth if w[-1] == "(" else 5 + 2 * depth)
            assert len(st) == expect, w


def test_right_linear_equals_regex():
    o = Oracle(G.RIGHT_LINEAR)
    full, pre = re.compile(r"(ab|c)*d"), re.compile(r"(ab|c)*(a|d|ab|)")
    for k in range(0, 9):
        for w in itertools.product("abcd", repeat=k):
            w = "".join(w)
            rc, st = _stack_after(o, w)
            is_prefix = bool(re.fullmatch(r"(ab|c)*(a|d)?", w))
            assert (rc == 0) == is_prefix, w
            if rc == 0:
                assert o.eos_allowed(st) == bool(full.fullmatch(w)), w


# ---------------------------------------------------------------- JSON vs the json module

def _random_json(rnd, depth=0):
    r = rnd.random()
    if depth > 3 or r < 0.35:
        k = rnd.randrange(7)
        if k == 0:
            return rnd.randint(-10 ** 6, 10 ** 6)
        if k == 1:
            return rnd.choice([0.5, -1.25e-7, 3e20, 1.0, -0.0, 12345.678])
        if k == 2:
            return rnd.choice([True, False, None])
        return "".join(rnd.choice('ab z"\\/\b\f\n\r\t{}[]:,0eé中\x7f') for _ in range(rnd.randint(0, 8)))
    if r < 0.7:
        return [_random_json(rnd, depth + 1) for _ in range(rnd.randint(0, 4))]
    return {"k%d" % i + rnd.choice(["", '"', "\\"]): _random_json(rnd, depth + 1) for i in range(rnd.randint(0, 4))}


def _json_ok(data: bytes) -> bool:
    def refuse(_):
        raise ValueError("non-standard constant")
    try:
        json.loads(data.decode("ascii"), parse_constant=refuse)
        return True
    except (ValueError, RecursionError):
        return False


def test_json_grammar_equals_json_module(json_oracle):
    """Membership in the byte-level JSON grammar == json.loads succeeds, on documents written
    by json.dumps in several layouts and on random one-byte corruptions of them (ASCII only,
    non-standard constants refused)."""
    o, rnd = json_oracle, random.Random(7)
    n_bad = n_good = 0
    for i in range(400):
        doc = _random_json(rnd)
        style = i % 4
        text = json.dumps(doc, ensure_ascii=True,
                          indent=[None, 1, None, "\t"][style],
                          separators=[(",", ":"), (", ", ": "), (" , ", " : "), None][style])
        data = text.encode("ascii")
        if i % 5 == 0:
            data = b" \n" + data + b"\r\n\t "
        assert _json_ok(data)
        assert o.accepts(data), data
        for _ in range(12):
            pos = rnd.randrange(len(data))
            kind = rnd.randrange(3)
            if kind == 0:
                mut = data[:pos] + bytes([rnd.choice(b'"\\{}[]:,0123456789.eE+-tfn u\n\x01\x7fax')]) + data[pos + 1:]
            elif kind == 1:
                mut = data[:pos] + data[pos + 1:]
            else:
                mut = data[:pos] + bytes([rnd.choice(b'"\\{}[]:,01.e-t ')]) + data[pos:]
            expect = _json_ok(mut)
            assert o.accepts(mut) == expect, mut
            n_good += expect
            n_bad += not expect
    assert n_good > 300 and n_bad > 1500


def _thought_then_json_ok(data: bytes) -> bool:
    """The free-text-then-JSON documents, recognised without a grammar: a fixed opening, one to
    three lines (a space, one or more bytes from 0x20 up, a line feed), a fixed label, then a
    JSON value that starts right after the label (the json module decides that part)."""
    if not data.startswith(b"Thought:"):
        return False
    rest, n_lines = data[len(b"Thought:"):], 0
    while rest.startswith(b" "):
        end = rest.find(b"\n")
        if end < 2 or min(rest[:end]) < 0x20:
            return False
        rest, n_lines = rest[end + 1:], n_lines + 1
    if not 1 <= n_lines <= 3 or not rest.startswith(b"Answer: "):
        return False
    rest = rest[len(b"Answer: "):]
    return len(rest) > 0 and rest[0] not in b" \t\r\n" and _json_ok(rest)


def test_thought_then_json_grammar_equals_a_direct_recogniser():
    o, rnd = Oracle([G.THOUGHT_THEN_JSON]), random.Random(11)
    n_good = n_bad = 0
    for i in range(150):
        lines = [" " + "".join(rnd.choice('ab {}[]":,\\A\x7f') for _ in range(rnd.randint(1, 9))) + "\n"
                 for _ in range(rnd.randint(1, 3))]
        doc = json.dumps(_random_json(rnd), ensure_ascii=True, indent=[None, 1][i % 2])
        data = ("Thought:" + "".join(lines) + "Answer: " + doc).encode("ascii") + [b"", b" \n"][i % 3 == 0]
        assert _thought_then_json_ok(data) and o.accepts(data), data
        for _ in range(16):
            pos = rnd.randrange(len(data))
            kind = rnd.randrange(4)
            if kind == 0:
                mut = data[:pos] + bytes([rnd.choice(b' \nA"{}[]:,0a\x01\x1f\x20\x7f')]) + data[pos + 1:]
            elif kind == 1:
                mut = data[:pos] + data[pos + 1:]
            elif kind == 2:
                mut = data[:pos] + bytes([rnd.choice(b' \nA"{[:,0a')]) + data[pos:]
            else:                                   # one more or one fewer line
                mut = data.replace(b"\nAnswer", rnd.choice([b"\n x\nAnswer", b"\n \nAnswer", b"Answer"]), 1)
            expect = _thought_then_json_ok(mut)
            assert o.accepts(mut) == expect, mut
            n_good += expect
            n_bad += not expect
    assert n_good > 300 and n_bad > 600
    for text, ok in [(b"Thought: a\nAnswer: 1", True), (b"Thought:\nAnswer: 1", False), (b"Thought: \nAnswer: 1", False),
                     (b"Thought: a\n b\n c\nAnswer: []", True), (b"Thought: a\n b\n c\n d\nAnswer: []", False),
                     (b"Thought: a\nAnswer:  1", False), (b"Thought: a\nAnswer: ", False),
                     (b"Thought: a\n Answer: 1\nAnswer: 2 ", True), (b"Thought: \xff\x20\nAnswer: null", True)]:
        assert _thought_then_json_ok(text) == ok and o.accepts(text) == ok, text


@pytest.mark.parametrize("text,ok", [
    (b"0", True), (b"-0", True), (b"01", False), (b"-", False), (b"1.", False), (b".5", False),
    (b"1e5", True), (b"1E+5", True), (b"1e", False), (b"1.5e-3", True), (b"--1", False),
    (b'"\\u12aF"', True), (b'"\\u12G4"', False), (b'"\\x"', False), (b'"\t"', False),
    (b'"\x7f\x80\xff"', True), (b"[]", True), (b"[,]", False), (b"[1,]", False), (b"{}", True),
    (b'{"a"}', False), (b'{"a":1,}', False), (b'{1:2}', False), (b"tru", False), (b"true", True),
    (b"nullx", False), (b"", False), (b"  ", False), (b"1 2", False), (b"[1 2]", False),
    (b'{"a":{"b":[{},[[]],""]}}', True), (b"[" * 40 + b"]" * 40, True), (b"[" * 5 + b"]" * 4, False),
])
def test_json_special_cases(json_oracle, text, ok):
    assert json_oracle.accepts(text) == ok


# ------------------------------------------------------------------------ invariants

@pytest.fixture(scope="module")
def json_vocab():
    return bpe_like_vocab(4000, 12, BASE_SEED + 99)


def _bits(row, n):
    return ((row[np.arange(n) >> 5] >> (np.arange(n) & 31)) & 1).astype(bool)


def test_invariants_on_json_walks(json_oracle, json_vocab):
    """I1 prefix closure, I2 concatenation, I3 EOS == sentence, I4 liveness, I5 token advance ==
    byte-by-byte advance, I6 stack shape - along seeded random walks."""
    o, v, rnd = json_oracle, json_vocab, random.Random(3)
    by_text = {}
    for t, tok in enumerate(v.tokens):
        by_text.setdefault(tok, []).append(t)
    for walk in range(12):
        st, text = o.initial_stack(), b""
        for step in range(40):
            row = o.mask_row(st, v)
            bits = _bits(row, v.n_tokens)
            assert not (row[-1] >> (v.n_tokens & 31 or 32)) if v.n_tokens & 31 else True   # padding is 0
            assert bits[v.eos_id] == o.eos_allowed(st) == o.accepts(text)               # I3
            assert bits[:256].any()                                                     # I4
            allowed = np.flatnonzero(bits)
            allowed = allowed[allowed != v.eos_id]
            # equal strings get equal bits; I1: every prefix that is itself a token is allowed
            for t in rnd.sample(list(allowed), min(25, len(allowed))):
                tok = v.tokens[t]
                assert all(bits[u] for u in by_text[tok])
                for k in range(1, len(tok)):
                    for u in by_text.get(tok[:k], []):
                        assert bits[u], (tok, tok[:k])
            t = int(rnd.choice(list(allowed)))
            tok = v.tokens[t]
            rc, new = o.advance(st, tok)
            assert rc == 0
            step_st = st                                                                # I5
            for c in tok:
                rc1, step_st = o.advance(step_st, bytes([c]))
                assert rc1 == 0
            assert step_st == new
            assert new[0] == o.initial_state() and all(0 <= s < o.n_states() for s in new)  # I6
            # I2: after advancing by u, v is allowed iff u.v was viable from the old stack
            new_bits = _bits(o.mask_row(new, v), v.n_tokens)
            for u in rnd.sample(range(v.n_tokens - 1), 60):
                assert new_bits[u] == o.allowed(st, tok + v.tokens[u]), (tok, v.tokens[u])
            st, text = new, text + tok
            if len(st) > 60:
                break
    # a token that is not allowed cannot be advanced by, and leaves the stack unchanged
    st = o.initial_stack()
    rc, same = o.advance(st, b"}")
    assert rc == 1 and same == st
    # empty byte strings are never allowed
    assert not o.allowed(st, b"")


def test_advance_overflow_leaves_stack_unchanged(json_oracle):
    o = json_oracle
    st = o.initial_stack()
    rc, deep = o.advance(st, b"[[[[")
    assert rc == 0
    rc2, same = o.advance(deep, b"[[[[[[[[", cap=len(deep) + 3)
    assert rc2 == 2 and same == deep
    assert o.allowed(deep, b"[[[[[[[[")          # 'allowed' itself has no capacity


def test_batched_calls_match_single_calls(json_oracle, json_vocab):
    o, v = json_oracle, json_vocab
    prefixes = [b"", b'{"a', b"[1", b'{"k": [tr', b"[[[[", b'"x\\', b"12.5e", b" 7 "]
    B, cap = len(prefixes) + 1, 64
    data = np.zeros((B, cap), dtype=np.int32)
    length = np.ones(B, dtype=np.int32)
    states = np.zeros(B, dtype=np.int32)
    for b, p in enumerate(prefixes):
        rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p)
        assert rc == 0
        data[b, : len(st)] = st
        length[b] = len(st)
        states[b] = st[-1]
    data[B - 1, 0] = o.initial_state()
    states[B - 1] = -1                                             # a finished sequence
    m = o.fill_mask(states, data, length, v)
    for b in range(B - 1):
        assert (m[b] == o.mask_row(data[b, : length[b]], v)).all()
    only_eos = np.zeros(v.words, dtype=np.uint32)
    only_eos[v.eos_id >> 5] = 1 << (v.eos_id & 31)
    assert (m[B - 1] == only_eos).all()
    # advance_batch: ok, skip, disallowed, EOS where allowed / not allowed, finished, overflow
    tok_of = {tok: t for t, tok in enumerate(v.tokens) if t != v.eos_id}
    tokens = np.array([tok_of[b"{"], -1, tok_of[b"}"], v.eos_id, tok_of[b"["], tok_of[b"n"],
                       tok_of[b"1"], v.eos_id, tok_of[b"1"]], dtype=np.int32)
    s2, d2, l2 = states.copy(), data.copy(), length.copy()
    d2[4, :] = data[4, :]
    err = o.advance_batch(s2, d2, l2, tokens, v)
    assert err.tolist() == [0, 0, 1, 1, 0, 0, 0, 0, 1]
    assert s2[7] == -1 and (d2[7] == data[7]).all() and l2[7] == length[7]       # EOS: stack untouched
    assert (d2[2] == data[2]).all() and l2[2] == length[2] and s2[2] == states[2]
    assert l2[1] == length[1] and s2[1] == states[1]
    rc, st0 = o.advance(o.initial_stack(), b"{")
    assert d2[0, : l2[0]].tolist() == st0 and s2[0] == st0[-1]
    # overflow: the row has no room for the push; the sequence is left unchanged
    n4 = int(length[4])
    tight = np.ascontiguousarray(data[4:5, :n4])
    s3, l3 = states[4:5].copy(), length[4:5].copy()
    before = tight.copy()
    err3 = o.advance_batch(s3, tight, l3, np.array([tok_of[b"["]], dtype=np.int32), v)
    assert err3.tolist() == [2] and (tight == before).all() and l3[0] == n4 and s3[0] == states[4]


def test_apply_mask_is_a_bf16_select():
    rng = np.random.default_rng(5)
    B, V = 5, 1000 + 17
    logits = bf16_logits(rng, B, V)
    logits[0, :6] = [0x7FC0, 0xFFC1, 0x7F80, 0xFF80, 0x0000, 0x8000]      # NaNs, infs, zeros
    W = (V + 31) // 32
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[1] = 0
    mask[2] = 0xFFFFFFFF
    bits = ((mask[:, np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1).astype(bool)
    expect = np.where(bits, logits, np.uint16(0xFF80))
    got = logits.copy()
    apply_mask(got, mask, V)
    assert (got == expect).all()
    # strided rows: only the first V entries of each row are touched
    wide = np.full((B, V + 9), 0x1234, dtype=np.uint16)
    wide[:, :V] = logits
    apply_mask(wide, mask, V)
    assert (wide[:, :V] == expect).all() and (wide[:, V:] == 0x1234).all()


def _bits_of(mask, V):
    return ((mask[:, np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1).astype(bool)


def test_masked_argmax_is_numpy_argmax_over_the_candidates():
    # pinned to a library routine: numpy's argmax (first occurrence of the maximum) over the
    # float32 values of the allowed, non-NaN entries
    rng = np.random.default_rng(11)
    B, V = 9, 2000 + 13
    logits = bf16_logits(rng, B, V)
    # coarse values in some rows so that equal maxima occur
    logits[3] = (np.round(rng.normal(size=V) * 2).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    logits[4] = logits[3]
    logits[5, ::7] = 0x7FC0                                   # NaNs sprinkled in
    logits[5, 3::11] = 0xFFC0
    logits[6, 100] = 0x7F80                                   # +inf wins when allowed
    W = (V + 31) // 32
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[7] = 0                                               # nothing allowed
    mask[8] = 0
    mask[8, 5] = 1 << 9                                       # exactly one token allowed
    bits = _bits_of(mask, V)
    values = (logits.astype(np.uint32) << 16).view(np.float32)
    expect = np.full(B, -1, dtype=np.int32)
    for b in range(B):
        cand = np.flatnonzero(bits[b] & ~np.isnan(values[b]))
        if len(cand):
            expect[b] = cand[np.argmax(values[b, cand])]
    got = masked_argmax(logits, mask, V)
    assert got.tolist() == expect.tolist()
    assert expect[7] == -1 and expect[8] == 5 * 32 + 9
    # the choice is what a sampler would see after apply_mask: the masked logits' own maximum
    masked = logits.copy()
    apply_mask(masked, mask, V)
    mv = (masked.astype(np.uint32) << 16).view(np.float32)
    for b in range(B):
        if expect[b] >= 0:
            assert mv[b, expect[b]] == np.nanmax(mv[b])


def test_masked_argmax_hand_cases():
    V = 40
    W = 2
    def run(values_u16, allowed):
        logits = np.full((1, V), 0xC000, dtype=np.uint16)     # -2.0 everywhere
        for t, x in values_u16.items():
            logits[0, t] = x
        mask = np.zeros((1, W), dtype=np.uint32)
        for t in allowed:
            mask[0, t >> 5] |= np.uint32(1 << (t & 31))
        return int(masked_argmax(logits, mask, V)[0])
    one, two, neg0, pos0, nan, ninf, pinf = 0x3F80, 0x4000, 0x8000, 0x0000, 0x7FC1, 0xFF80, 0x7F80
    assert run({3: two, 9: one}, [3, 9, 12]) == 3
    assert run({3: two, 9: two}, [9, 3]) == 3                 # equal values: smallest id
    assert run({3: two, 9: one}, [9, 12]) == 9                # the larger one is masked
    assert run({35: two}, [35, 1]) == 35                      # second mask word
    assert run({4: neg0, 7: pos0}, [4, 7]) == 4               # -0 == +0: first wins
    assert run({4: pos0, 7: neg0}, [4, 7]) == 4
    assert run({2: nan, 5: one}, [2, 5]) == 5                 # NaN is never chosen
    assert run({2: nan}, [2]) == -1
    assert run({2: ninf, 6: ninf}, [6, 2]) == 2               # -inf is a value like any other
    assert run({2: ninf, 6: nan}, [6, 2]) == 2
    assert run({2: pinf, 6: two}, [6, 2]) == 2
    assert run({}, []) == -1


def test_masked_topk_is_a_stable_numpy_sort_of_the_candidates():
    # pinned to a library routine: numpy's stable argsort of the negated float32 values over the
    # allowed, non-NaN entries in id order (stable = equal values keep ascending ids)
    rng = np.random.default_rng(12)
    B, V = 10, 3000 + 7
    logits = bf16_logits(rng, B, V)
    logits[3] = (np.round(rng.normal(size=V) * 2).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    logits[4, ::3] = 0x0000                                   # zeros of both signs among the largest values
    logits[4, 1::3] = 0x8000
    logits[4, 2::3] = 0xBF80
    logits[5, ::7] = 0x7FC0
    logits[5, 3::11] = 0xFFC0
    logits[6, 100] = 0x7F80
    logits[6, 200:230] = 0xFF80
    W = (V + 31) // 32
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[7] = 0
    mask[8] = 0
    mask[8, 5] = (1 << 9) | (1 << 30)                         # two tokens allowed
    mask[9] &= rng.integers(0, 2 ** 32, size=W, dtype=np.uint64).astype(np.uint32) & 0x11111111   # sparse
    bits = _bits_of(mask, V)
    values = (logits.astype(np.uint32) << 16).view(np.float32)
    for k in (1, 5, 64):
        ids, vals = masked_topk(logits, mask, V, k)
        assert ids.shape == (B, k) and vals.shape == (B, k)
        for b in range(B):
            cand = np.flatnonzero(bits[b] & ~np.isnan(values[b]))
            order = cand[np.argsort(-values[b, cand], kind="stable")][:k]
            want = np.full(k, -1, dtype=np.int64)
            want[: len(order)] = order
            assert ids[b].tolist() == want.tolist(), (k, b)
            assert vals[b, : len(order)].tolist() == logits[b, order].tolist()
            assert (vals[b, len(order):] == 0xFF80).all()
        assert (ids[:, 0] == masked_argmax(logits, mask, V)).all()      # the head of the list is the greedy choice
    ids, _ = masked_topk(logits, mask, V, 64)
    assert (ids[7] == -1).all() and ids[8, :2].tolist() == sorted([5 * 32 + 9, 5 * 32 + 30], key=lambda t: (-values[8, t], t))
    assert (ids[8, 2:] == -1).all()


def test_masked_topk_hand_cases():
    V, W = 40, 2
    def run(values_u16, allowed, k):
        logits = np.full((1, V), 0xC000, dtype=np.uint16)     # -2.0 everywhere
        for t, x in values_u16.items():
            logits[0, t] = x
        mask = np.zeros((1, W), dtype=np.uint32)
        for t in allowed:
            mask[0, t >> 5] |= np.uint32(1 << (t & 31))
        ids, vals = masked_topk(logits, mask, V, k)
        return ids[0].tolist(), vals[0].tolist()
    one, two, neg0, pos0, nan, ninf, pinf = 0x3F80, 0x4000, 0x8000, 0x0000, 0x7FC1, 0xFF80, 0x7F80
    assert run({3: one, 9: two, 12: one}, [3, 9, 12, 20], 3) == ([9, 3, 12], [two, one, one])
    assert run({3: one, 9: two}, [3, 9], 4) == ([9, 3, -1, -1], [two, one, ninf, ninf])
    assert run({4: neg0, 7: pos0, 9: neg0}, [9, 7, 4], 2) == ([4, 7], [neg0, pos0])     # zeros tie, patterns kept
    assert run({2: nan, 5: one, 6: ninf}, [2, 5, 6], 3) == ([5, 6, -1], [one, ninf, ninf])
    assert run({2: pinf, 35: two}, [2, 35, 36], 3) == ([2, 35, 36], [pinf, two, 0xC000])
    assert run({}, [], 2) == ([-1, -1], [ninf, ninf])


def test_arithmetic_workload_vocab_has_the_terminals():
    v = arithmetic_vocab(BASE_SEED + 1)
    assert v.n_tokens == 513 and v.eos_id == 512
    assert all(bytes([c]) in v.tokens for c in b"a+*()")


@pytest.mark.parametrize("name,alphabet", [
    ("ARITHMETIC", "a+*()b"), ("DYCK", "()x"), ("ANBN", "abx"), ("RIGHT_LIST", "x,y"),
    ("EPSILON_MIX", "abcx"), ("RIGHT_LINEAR", "abcd"), ("DRAGON_CC", "cdx"),
])
def test_jump_forward_equals_brute_force(name, alphabet):
    """Forced bytes from the LR-free sets of sentences and viable prefixes: while the text is not
    a sentence and exactly one byte keeps it viable, that byte is forced."""
    text = getattr(G, name)
    o = Oracle(text)
    sentences, viable = languages(text, N)
    n_forced = 0
    for p in sorted(viable):
        if len(p) > 4:
            continue
        horizon = N - 1 - len(p)                 # every p.w.c looked up below has length <= N
        w = ""
        while len(w) < horizon and (p + w) not in sentences:
            nxt = [c for c in alphabet if (p + w + c) in viable]
            if len(nxt) != 1:
                break
            w += nxt[0]
        rc, st = _stack_after(o, p)
        got, new_stack = o.jump_forward(st, max_bytes=horizon)
        assert got == w.encode(), (p, w, got)
        assert new_stack == _stack_after(o, p + w)[1]
        n_forced += len(w)
    if name == "ANBN":                           # a^n b^k: the remaining b's are forced
        assert n_forced >= 4


def test_jump_forward_hand_cases_and_batch():
    o = Oracle('S ::= "hello" | "help" A\nA ::= "!" | A "?"')
    s0 = o.initial_stack()
    assert o.jump_forward(s0)[0] == b"hel"
    assert o.jump_forward(o.advance(s0, b"hell")[1])[0] == b"o"
    assert o.jump_forward(o.advance(s0, b"help")[1])[0] == b"!"
    assert o.jump_forward(o.advance(s0, b"help!")[1])[0] == b""          # a sentence: EOS is allowed, nothing is forced
    assert o.jump_forward(s0, max_bytes=2)[0] == b"he"
    j = Oracle(G.JSON)
    j0 = j.initial_stack()
    for prefix, forced in [(b"t", b"rue"), (b"[tru", b"e"), (b"n", b"ull"), (b"fa", b"lse"), (b'"', b""), (b"[", b""),
                           (b'{"a"', b""), (b"[1,", b""), (b'"\\u12', b"")]:
        assert j.jump_forward(j.advance(j0, prefix)[1])[0] == forced, prefix
    # a schema grammar forces its key text
    sch = G.schema_grammar(11, 6, 2, 4)
    so = Oracle(sch.text)
    forced, st = so.jump_forward(so.advance(so.initial_stack(), b'{"')[1])
    assert len(forced) >= 4 and b'"' in forced                       # the first key's text and its closing quote
    assert so.advance(so.initial_stack(), b'{"' + forced)[1] == st
    # batch form: same bytes, finished rows untouched, a tight cap stops before the overflowing byte
    cap = 16
    prefixes = [b"t", b"[tru", b'"', b"n"]
    data = np.zeros((5, cap), dtype=np.int32)
    length = np.ones(5, dtype=np.int32)
    for b, p in enumerate(prefixes):
        st = j.advance(j0, p)[1]
        data[b, : len(st)], length[b] = st, len(st)
    data[4, 0] = j0[0]
    states = data[np.arange(5), length - 1].copy()
    states[4] = -1
    out, cnt = j.jump_forward_batch(states, data, length, 8)
    assert [out[b, : cnt[b]].tobytes() for b in range(5)] == [b"rue", b"e", b"", b"ull", b""]
    assert states[4] == -1 and length[4] == 1
    for b, (p, f) in enumerate(zip(prefixes, [b"rue", b"e", b"", b"ull"])):
        st = j.advance(j0, p + f)[1]
        assert data[b, : length[b]].tolist() == st and states[b] == st[-1]
    deep = j.advance(j0, b"[" * 10 + b"t")[1]
    tight = np.zeros((1, len(deep) + 1), dtype=np.int32)
    tight[0, : len(deep)] = deep
    l1, s1 = np.array([len(deep)], dtype=np.int32), np.array([deep[-1]], dtype=np.int32)
    out, cnt = j.jump_forward_batch(s1, tight, l1, 8)
    full = j.jump_forward(deep, 8)[0]
    assert full == b"rue" and out[0, : cnt[0]].tobytes() == full[: cnt[0]] and l1[0] <= tight.shape[1]
