"""Cycle-aware stacks (PRE3_FLAG_COMPACT_CYCLES) through the C ABI against the CPU oracle: a library
compiled with the option must leave, after every call that changes the bound stacks, exactly the
stacks the oracle leaves when it compacts after every advance -- states, len, live entries, err --
and the masks of those stacks; lists of any length must keep bounded stacks where the same calls
without the option run out of capacity."""
import numpy as np
import pytest

from oracle import Oracle
from replay import replay, replay_advance_fill
from workloads import grammars as G
from workloads import trajectory
from workloads.vocab import BASE_SEED, bpe_like_vocab

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch, torch.device("cuda:0")


def test_right_recursive_json_full_size():
    """B=256, V=128256 on the right-recursive JSON grammar (20 registered cycles)."""
    r = replay(7, steps=128, full_mask_steps=[0, 1, 40, 127])
    assert r["full_masks"] == 4
    r = replay_advance_fill(7, steps=96, full_mask_steps=[0, 50, 95])
    assert r["full_masks"] == 3


@pytest.mark.parametrize("options", [dict(token_edges=False), dict(merged_reductions=False), dict(max_condition_depth=3)])
def test_cycle_aware_stacks_under_every_merging_level(options):
    """Compaction does not depend on how masks and walks are computed: byte-by-byte masks, one
    reduction per step, and shallow condition trees (leftover walks) give the same stacks and masks."""
    r = replay(7, steps=20, full_mask_steps=[0, 7, 19], check_apply=False, **options)
    assert r["full_masks"] == 3
    r = replay_advance_fill(7, steps=16, full_mask_steps=[0, 15], **options)
    assert r["full_masks"] == 2


def _bound(lib, B, cap, s0):
    torch, dev = _torch()
    data = torch.zeros((B, cap), dtype=torch.int32, device=dev)
    data[:, 0] = s0
    length = torch.ones(B, dtype=torch.int32, device=dev)
    states = torch.full((B,), s0, dtype=torch.int32, device=dev)
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states, data, length, err)
    return states, data, length, err


def test_long_lists_keep_bounded_stacks_and_plain_stacks_overflow():
    """Eight sequences write lists of different kinds (string characters, digits, array elements,
    members, white space, nested arrays) far longer than the capacity of 48 entries."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    v = bpe_like_vocab(2000, 8, BASE_SEED + 81)
    ids = {tok: t for t, tok in reversed(list(enumerate(v.tokens)))}      # first id of each byte string
    cap, n_rounds = 48, 400
    scripts = [                                        # (opening, repeated unit, closing)
        (b'["', b"abcd", b'"]'), (b"[1", b"2345", b"]"), (b"[", b"7,", b"8]"), (b'{"k":1', b',"k":2', b"}"),
        (b"[", b" \n\t ", b"]"), (b"[[", b'"x",', b"0]]"), (b'"', b"\\n\\u00e9", b'"'), (b"[", b"[],", b"[]]"),
    ]
    B = len(scripts)
    streams = []
    for head, unit, tail in scripts:
        streams.append(list(head) + list(unit) * n_rounds + list(tail))
    steps = max(len(s) for s in streams)
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap,
               compact_cycles=True)
    plain = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    s0 = lib.initial_state(0)
    states_d, data_d, len_d, err_d = _bound(lib, B, cap, s0)
    p_states, p_data, p_len, p_err = _bound(plain, B, cap, s0)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = np.full(B, s0, dtype=np.int32)
    overflowed = np.zeros(B, dtype=bool)
    longest = 0
    for s in range(steps):
        tok = np.array([ids[bytes([st[s]])] if s < len(st) else -1 for st in streams], dtype=np.int32)
        tok_d = torch.from_numpy(tok).to(dev)
        lib.advance(tok_d)
        err_h = o.advance_batch(states_h, data_h, len_h, tok, v)
        assert not err_h.any(), (s, err_h)
        plain.advance(tok_d)
        overflowed |= p_err.cpu().numpy() == 2
        if s % 16 == 0 or s >= steps - 8:
            assert (err_d.cpu().numpy() == 0).all(), s
            assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), s
            live = np.arange(cap)[None, :] < len_h[:, None]
            assert (data_d.cpu().numpy()[live] == data_h[live]).all(), s
        longest = max(longest, int(len_h.max()))
    assert longest <= 24, longest
    assert overflowed.all(), overflowed
    for b in range(B):                                  # every document ended as a sentence
        assert o.eos_allowed(data_h[b, : len_h[b]])
    mask_d = torch.empty((B, v.words), dtype=torch.int32, device=dev)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    assert (mask_d.cpu().numpy().view(np.uint32) == o.fill_mask(states_h, data_h, len_h, v)).all()


def test_capacity_beyond_the_fused_staging_uses_the_compaction_kernel():
    """With stack_cap = 4000 four staged stacks no longer fit advance_kernel's LDS, so pre3_advance
    compacts with the kernel of its own; the stacks must be the same."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    v = bpe_like_vocab(2000, 8, BASE_SEED + 83)
    ids = {tok: t for t, tok in reversed(list(enumerate(v.tokens)))}
    cap = 4000
    streams = [list(b'[[1,2,[3,4,5],"ab\\ncd",{"k":[1,2,3],"l":{}}],7,8,9,10]'), list(b'{"a":"xyzw","b":[[],[],[[]]],"c":12345}'),
               list(b'[' + b'[' * 40 + b'1' + b']' * 40 + b',2,3]')]
    B = len(streams)
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap,
               compact_cycles=True)
    s0 = lib.initial_state(0)
    states_d, data_d, len_d, err_d = _bound(lib, B, cap, s0)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = np.full(B, s0, dtype=np.int32)
    for s in range(max(len(st) for st in streams)):
        tok = np.array([ids[bytes([st[s]])] if s < len(st) else -1 for st in streams], dtype=np.int32)
        lib.advance(torch.from_numpy(tok).to(dev))
        assert not o.advance_batch(states_h, data_h, len_h, tok, v).any(), s
        assert (err_d.cpu().numpy() == 0).all(), s
        assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), s
        live = np.arange(cap)[None, :] < len_h[:, None]
        assert (data_d.cpu().numpy()[live] == data_h[live]).all(), s
        if s % 9 == 4:                                  # jump-forward takes the same fallback at this capacity
            out = torch.zeros((B, 8), dtype=torch.uint8, device=dev)
            cnt = torch.zeros(B, dtype=torch.int32, device=dev)
            lib.jump_forward(out, cnt)
            want_bytes, want_cnt = o.jump_forward_batch(states_h, data_h, len_h, 8)
            assert cnt.cpu().numpy().tolist() == want_cnt.tolist() == [0] * B, s      # white space is always allowed
            assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), s
    for b in range(B):
        assert o.eos_allowed(data_h[b, : len_h[b]])


def test_jump_forward_and_whole_tokens_on_lists_of_fixed_keys():
    """A grammar with forced runs inside a right-recursive list: jump-forward crosses whole list
    elements, and the stacks it leaves are compacted like those of an advance."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    text = r'''
doc   ::= "[" items "]"
items ::= item | item "," items
item  ::= "{\"id\":" digits "}"
digits ::= digit | digit digits
digit ::= [0-9]
'''
    v = bpe_like_vocab(3000, 10, BASE_SEED + 82)
    o = Oracle([text], compact_cycles=True)
    assert len(o.cycles()) >= 2
    B, cap = 16, 64
    lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap, compact_cycles=True)
    assert lib.reduction_cycles() == o.cycles()
    drv = trajectory.Driver(o, v, B, cap, 23, None, 100, None, False)
    states_d, data_d, len_d = (torch.from_numpy(x.copy()).to(dev) for x in (drv.states, drv.data, drv.len))
    err_d = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    out = torch.zeros((B, 16), dtype=torch.uint8, device=dev)
    cnt = torch.zeros(B, dtype=torch.int32, device=dev)
    forced = 0
    for s in range(120):
        want_bytes, want_cnt = o.jump_forward_batch(drv.states, drv.data, drv.len, 16)
        lib.jump_forward(out, cnt)
        got_cnt, got = cnt.cpu().numpy(), out.cpu().numpy()
        assert got_cnt.tolist() == want_cnt.tolist(), s
        for b in range(B):
            assert got[b, : got_cnt[b]].tobytes() == want_bytes[b, : want_cnt[b]].tobytes(), (s, b)
        forced += int(want_cnt.sum())
        tokens, reset = drv.step(last_step=False)        # the driver advances (and compacts) the host side
        lib.advance(torch.from_numpy(tokens).to(dev))
        assert (err_d.cpu().numpy() == 0).all()
        live_rows = drv.states >= 0
        assert (states_d.cpu().numpy() == drv.states).all() and (len_d.cpu().numpy()[live_rows] == drv.len[live_rows]).all()
        live = (np.arange(cap)[None, :] < drv.len[:, None]) & live_rows[:, None]
        assert (data_d.cpu().numpy()[live] == drv.data[live]).all(), s
        assert int(drv.len.max()) <= 16
        fin = np.flatnonzero(drv.states < 0)
        if len(fin):                                     # restart finished sequences on both sides
            for b in fin:
                drv._reset(int(b))
            idx = torch.from_numpy(fin).to(dev)
            data_d[idx, 0] = int(drv.data[fin[0], 0])
            len_d[idx] = 1
            states_d[idx] = int(drv.data[fin[0], 0])
    assert forced > 300, forced


def test_row_plus_staged_stack_beyond_the_lds_takes_three_launches():
    """400,000 tokens (a mask row of 50,000 bytes) and a capacity of 3,000 entries (12,000 bytes): together
    with the kernel's own LDS they pass 64 KB, so pre3_advance_fill_mask must fall back to advance,
    compaction and mask as separate launches -- and leave the same stacks and masks."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    v = bpe_like_vocab(400000, 12, BASE_SEED + 84)
    ids = {tok: t for t, tok in reversed(list(enumerate(v.tokens)))}
    cap = 3000
    streams = [list(b'[[1,2,[3,4,5],"ab\\ncd",{"k":[1,2,3]}],7,8]'), list(b'{"a":"xyzw","b":[[],[],[[]]],"c":12345}'),
               list(b'[1,2,3,4,5,6,7,8,9,10,11,12,13]')]
    B = len(streams)
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap,
               compact_cycles=True)
    assert lib.token_edge_stats()["built"] == 1 and v.words * 4 + cap * 4 > 65536 - 8192
    s0 = lib.initial_state(0)
    states_d, data_d, len_d, err_d = _bound(lib, B, cap, s0)
    mask_d = torch.zeros((B, v.words), dtype=torch.int32, device=dev)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = np.full(B, s0, dtype=np.int32)
    for s in range(max(len(st) for st in streams)):
        tok = np.array([ids[bytes([st[s]])] if s < len(st) else -1 for st in streams], dtype=np.int32)
        lib.advance_fill_mask(torch.from_numpy(tok).to(dev), mask_d)
        assert not o.advance_batch(states_h, data_h, len_h, tok, v).any(), s
        assert (err_d.cpu().numpy() == 0).all(), s
        assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), s
        live = np.arange(cap)[None, :] < len_h[:, None]
        assert (data_d.cpu().numpy()[live] == data_h[live]).all(), s
        if s % 6 == 0:
            assert (mask_d.cpu().numpy().view(np.uint32) == o.fill_mask(states_h, data_h, len_h, v)).all(), s


@pytest.mark.parametrize("call", ["advance", "advance_fill_mask", "jump_forward"])
def test_stacks_that_were_never_compacted_are_compacted_whole(call):
    """The caller binds stacks that a parser without the option has built: hundreds of entries that
    hold long runs of traversals (several 64-entry chunks each, runs that cross chunk borders, runs
    of different cycles one after the other).  The next call that changes them must leave what the
    oracle leaves when it advances and then compacts the whole stack."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    v = bpe_like_vocab(2000, 8, BASE_SEED + 85)
    ids = {tok: t for t, tok in reversed(list(enumerate(v.tokens)))}
    cap = 1024
    prefixes = [                                        # (document so far, the byte that comes next)
        (b'["' + b"abcd" * 70, b"e"), (b"[1" + b"2345" * 60, b"6"), (b"[" + b"7," * 150, b"8"),
        (b'{"k":1' + b',"k":2' * 60, b","), (b"[" + b" \n\t " * 60, b"1"), (b"[[" + b'"x",' * 90, b"0"),
        (b"[" + b"[]," * 100, b"["), (b"[" + b"1," * 31 + b'"' + b"ab" * 40, b'"'),
        (b"[" + b"1," * 40 + b"[" + b"2," * 50 + b'{"a":3' + b',"a":4' * 30, b"}"),
        (b'["' + b"\\n" * 50 + b'",' + b"9," * 45 + b"10", b"]"), (b"[1,2,3", b","), (b"[", b"]"),
        (b"[1]" + b" \n" * 50, None), (b'{"k":[]}' + b"\t" * 90, None),      # a sentence, then white space: ends here (None = the end-of-sequence token)
    ]
    B = len(prefixes)
    plain = Oracle([G.JSON_RIGHT_RECURSIVE])
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap,
               compact_cycles=True)
    data_h = np.zeros((B, cap), dtype=np.int32)
    len_h = np.zeros(B, dtype=np.int32)
    for b, (text, _) in enumerate(prefixes):
        rc, st = plain.advance(plain.initial_stack(0), text)
        assert rc == 0 and len(st) <= cap - 8
        data_h[b, : len(st)], len_h[b] = st, len(st)
    assert (len_h > 192).sum() >= 5 and int(len_h.max()) > 300          # several chunks of 64 entries
    folded = [len(o.compact(list(data_h[b, : len_h[b]]))) for b in range(B)]
    assert max(folded) <= 24, folded
    states_h = data_h[np.arange(B), len_h - 1].copy()
    states_d, data_d, len_d = (torch.from_numpy(a.copy()).to(dev) for a in (states_h, data_h, len_h))
    err_d = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    tok = np.array([v.eos_id if nxt is None else ids[nxt] for _, nxt in prefixes], dtype=np.int32)
    if call == "jump_forward":
        out = torch.zeros((B, 8), dtype=torch.uint8, device=dev)
        cnt = torch.zeros(B, dtype=torch.int32, device=dev)
        lib.jump_forward(out, cnt)
        want_bytes, want_cnt = o.jump_forward_batch(states_h, data_h, len_h, 8)
        assert cnt.cpu().numpy().tolist() == want_cnt.tolist()
        assert (out.cpu().numpy() == want_bytes).all()
    else:
        if call == "advance":
            lib.advance(torch.from_numpy(tok).to(dev))
        else:
            mask_d = torch.zeros((B, v.words), dtype=torch.int32, device=dev)
            lib.advance_fill_mask(torch.from_numpy(tok).to(dev), mask_d)
        assert not o.advance_batch(states_h, data_h, len_h, tok, v).any()
        assert (err_d.cpu().numpy() == 0).all()
        if call == "advance_fill_mask":
            assert (mask_d.cpu().numpy().view(np.uint32) == o.fill_mask(states_h, data_h, len_h, v)).all()
    assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), (len_d.cpu().numpy(), len_h)
    live = np.arange(cap)[None, :] < len_h[:, None]
    assert (data_d.cpu().numpy()[live] == data_h[live]).all()
    assert lib.fault_count() == 0
