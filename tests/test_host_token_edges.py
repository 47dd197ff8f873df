"""The token-level prefix-conditioned edges, checked on the CPU: for stacks met along seeded
decoding trajectories the host evaluation of the compiled condition tree (the same tables the
GPU descends) must give the oracle's mask row, except for the tokens the tree explicitly leaves
to a byte-by-byte walk.  Covers deep and shallow condition limits, several grammars in one
handle, and the stack-independence of a row given the entries the tree tested."""
import numpy as np
import pytest

from oracle import Oracle
from paper_2506_03887_amd.binding import Pre3
from workloads import grammars as G
from workloads import trajectory
from workloads.vocab import BASE_SEED, arithmetic_vocab, bpe_like_vocab


def _row_bits(row, V):
    return ((row[np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1).astype(bool)


def _check_along_trajectory(texts, vocab, steps, batch, seed, nest_cap, grammar_idx=None, compact=False, **lib_options):
    o = Oracle(texts, compact_cycles=compact)
    lib_options = dict(lib_options, compact_cycles=compact)
    lib = Pre3(texts, vocab.bytes, vocab.offsets, vocab.eos_id, max_token_len=max(1, vocab.max_len), host_only=True,
               **lib_options)
    assert lib.token_edge_stats()["built"] == 1
    drv = trajectory.Driver(o, vocab, batch, 256, seed, grammar_idx, nest_cap, None, True)
    V = vocab.n_tokens
    resolved = undecided = unresolved = 0
    deepest = 0
    for _ in range(steps):
        for b in range(batch):
            if drv.states[b] < 0:
                continue
            stack = drv.data[b, : drv.len[b]]
            ok, row, walk = lib.debug_resolve_row(stack)
            if not ok:                                   # the kernel walks the whole vocabulary for such a stack
                unresolved += 1
                continue
            want = _row_bits(o.mask_row(stack, vocab), V)
            got = _row_bits(row, V)
            left = np.zeros(V, dtype=bool)
            left[walk] = True
            assert not (got & left).any(), "a token left to the walk must not be set by the tree"
            assert (got[~left] == want[~left]).all(), (stack.tolist(), np.flatnonzero(got != want)[:5].tolist())
            resolved += 1
            undecided += int(left.sum())
            deepest = max(deepest, lib.last_resolve_info["deepest_entry"])
        drv.step(last_step=False)
    return resolved, undecided, unresolved, deepest


def test_arithmetic_rows_equal_oracle_rows():
    v = arithmetic_vocab(BASE_SEED + 1)
    resolved, undecided, unresolved, deepest = _check_along_trajectory([G.ARITHMETIC], v, 40, 4, 3, 8)
    assert resolved > 100 and unresolved == 0 and undecided == 0 and deepest >= 2


@pytest.mark.parametrize("depth_limit", [48, 4, 1])
def test_json_rows_equal_oracle_rows(depth_limit):
    v = bpe_like_vocab(3000, 12, BASE_SEED + 61)
    resolved, undecided, unresolved, deepest = _check_along_trajectory(
        [G.JSON], v, 30, 6, 5, 6, max_condition_depth=depth_limit)
    assert resolved + unresolved > 120 and resolved > 0
    if depth_limit == 48:
        assert unresolved == 0 and undecided == 0        # every token became a single edge
    else:
        assert undecided > 0 or unresolved > 0           # shallow limits leave work to the byte-by-byte walk


def test_right_recursive_json_rows_on_cycle_aware_stacks():
    """With cycle-aware stacks the trees leave out conditions that a compacted stack cannot meet:
    compacted stacks still get exact rows from shallow descents, and a stack that was never
    compacted gets no answer from the tree (so the kernel walks) rather than a wrong one."""
    v = bpe_like_vocab(3000, 12, BASE_SEED + 61)
    resolved, undecided, unresolved, deepest = _check_along_trajectory(
        [G.JSON_RIGHT_RECURSIVE], v, 40, 6, 5, 6, compact=True)
    assert resolved > 200 and unresolved == 0 and undecided < resolved     # next to nothing is left to the walk
    plain = Oracle([G.JSON_RIGHT_RECURSIVE])
    lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, host_only=True,
               compact_cycles=True)
    rc, st = plain.advance(plain.initial_stack(), b'["abcdefgh')
    assert rc == 0 and len(plain.compact(st)) < len(st)
    ok, row, walk = lib.debug_resolve_row(np.array(st, dtype=np.int32))
    want = _row_bits(plain.mask_row(st, v), v.n_tokens)
    if ok:                                               # whatever the tree does decide must be right
        left = np.zeros(v.n_tokens, dtype=bool)
        left[walk] = True
        assert (_row_bits(row, v.n_tokens)[~left] == want[~left]).all()
    ok, row, walk = lib.debug_resolve_row(np.array(plain.compact(st), dtype=np.int32))
    assert ok and len(walk) == 0 and (_row_bits(row, v.n_tokens) == want).all()


@pytest.mark.parametrize("threshold", [1, 16, 3000])
def test_json_rows_with_id_lists(threshold):
    v = bpe_like_vocab(3000, 12, BASE_SEED + 61)
    resolved, undecided, unresolved, _ = _check_along_trajectory([G.JSON], v, 20, 6, 9, 6, row_threshold=threshold)
    assert resolved > 80 and unresolved == 0 and undecided == 0


def test_rows_of_several_grammars_in_one_handle():
    texts = [G.schema_grammar(21, 5, 2, 3).text, G.JSON, G.DYCK]
    v = bpe_like_vocab(2500, 12, BASE_SEED + 62)
    gi = np.array([0, 1, 2, 0, 1, 2], dtype=np.int32)
    resolved, _, _, _ = _check_along_trajectory(texts, v, 25, 6, 7, 5, grammar_idx=gi)
    assert resolved > 60


def test_row_depends_only_on_the_entries_the_tree_tested():
    """A row found after testing k stack entries must be the oracle's row for EVERY stack with
    the same top k entries: replace what lies below by another valid context and compare."""
    o = Oracle([G.JSON])
    v = bpe_like_vocab(2000, 12, BASE_SEED + 63)
    lib = Pre3([G.JSON], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, host_only=True)
    V = v.n_tokens
    contexts = [b"[", b"[[", b'{"a":', b'[{"k":[', b'{"a":1,"b":[2,']
    tails = [b"1", b'"x', b"tru", b"-0.", b'{"q":', b"[3,"]
    checked = 0
    for tail in tails:
        rows = []
        for ctx in contexts:
            rc, stack = o.advance(o.initial_stack(0), ctx + tail)
            assert rc == 0
            ok, row, walk = lib.debug_resolve_row(np.array(stack, dtype=np.int32))
            assert ok and len(walk) == 0
            assert (_row_bits(row, V) == _row_bits(o.mask_row(stack, v), V)).all()
            rows.append((lib.last_resolve_info["deepest_entry"], list(stack), row.copy()))
            checked += 1
        # two stacks that agree on the tested suffix get the same row
        for k1, s1, r1 in rows:
            for k2, s2, r2 in rows:
                k = max(k1, k2)
                if s1[-k:] == s2[-k:] and len(s1) >= k and len(s2) >= k:
                    assert (r1 == r2).all()
    assert checked == len(contexts) * len(tails)
