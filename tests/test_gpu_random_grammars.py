"""Seeded random tiny grammars on the GPU: for every viable prefix (up to length 6) of each
grammar both LR(1) builders accept, the device's mask row, advance (allowed and disallowed
tokens) and advance+mask must equal the oracle's, with each level of edge merging on and off."""
import random

import numpy as np
import pytest

from cfg_brute import languages
from oracle import GrammarError, Oracle
from test_random_grammars import N, _vocab, random_grammar

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("options", [dict(), dict(token_edges=False), dict(merged_reductions=False),
                                     dict(max_condition_depth=1)])
def test_random_grammars_on_the_device(options):
    import torch
    from paper_2506_03887_amd import Pre3
    dev = torch.device("cuda:0")
    rnd = random.Random(77)
    v = _vocab()
    V, W, cap = v.n_tokens, v.words, 32
    done = 0
    while done < 12:
        text = random_grammar(rnd)
        try:
            o = Oracle(text)
        except GrammarError:
            continue
        _, viable = languages(text, N)
        if len(viable) < 4:
            continue
        done += 1
        prefixes = sorted(viable)
        B = len(prefixes)
        data = np.zeros((B, cap), dtype=np.int32)
        length = np.ones(B, dtype=np.int32)
        for b, p in enumerate(prefixes):
            rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p.encode())
            assert rc == 0
            data[b, : len(st)], length[b] = st, len(st)
        states = data[np.arange(B), length - 1].copy()
        lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=3, stack_cap=cap, **options)
        st_d, da_d, ln_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
        err_d = torch.zeros(B, dtype=torch.int32, device=dev)
        m_d = torch.zeros((B, W), dtype=torch.int32, device=dev)
        lib.fill_mask(st_d, da_d, ln_d, m_d)
        want = o.fill_mask(states, data, length, v)
        assert (m_d.cpu().numpy().view(np.uint32) == want).all(), text
        # one token per row, allowed or not (EOS included), through advance + next mask
        toks = np.array([rnd.randrange(V) for _ in range(B)], dtype=np.int32)
        e_h = o.advance_batch(states, data, length, toks, v)
        lib.bind_state(st_d, da_d, ln_d, err_d)
        lib.advance_fill_mask(torch.from_numpy(toks).to(dev), m_d)
        assert (err_d.cpu().numpy() == e_h).all(), text
        assert (st_d.cpu().numpy() == states).all() and (ln_d.cpu().numpy() == length).all(), text
        live = np.arange(cap)[None, :] < length[:, None]
        assert (da_d.cpu().numpy()[live] == data[live]).all(), text
        assert (m_d.cpu().numpy().view(np.uint32) == o.fill_mask(states, data, length, v)).all(), text


@pytest.mark.parametrize("options", [dict(), dict(token_edges=False), dict(max_condition_depth=2)])
def test_random_right_recursive_grammars_with_cycle_aware_stacks(options):
    """Seeded random grammars with right-recursive alternatives, compiled with cycle-aware stacks:
    starting from the compacted stack of every viable prefix, streams of random tokens (allowed or
    not) through pre3_advance, pre3_advance_fill_mask and pre3_jump_forward must leave the oracle's
    compacted stacks, error codes and masks -- several cycles per grammar, shared first states,
    uncompacted stacks handed to pre3_fill_mask."""
    import torch
    from paper_2506_03887_amd import Pre3
    from test_oracle_cycles import _random_right_recursive_grammar
    dev = torch.device("cuda:0")
    rnd = random.Random(99)
    v = _vocab()
    V, W, cap = v.n_tokens, v.words, 48
    done = shortened = 0
    while done < 10:
        text = _random_right_recursive_grammar(rnd)
        try:
            o = Oracle(text, compact_cycles=True)
        except GrammarError:
            continue
        _, viable = languages(text, N)
        if not o.cycles() or len(viable) < 5:
            continue
        done += 1
        plain = Oracle(text)
        prefixes = sorted(viable)
        B = len(prefixes)
        data = np.zeros((B, cap), dtype=np.int32)
        length = np.ones(B, dtype=np.int32)
        raw = np.zeros((B, cap), dtype=np.int32)
        raw_len = np.ones(B, dtype=np.int32)
        for b, p in enumerate(prefixes):
            rc, st = (0, plain.initial_stack()) if not p else plain.advance(plain.initial_stack(), p.encode())
            assert rc == 0
            raw[b, : len(st)], raw_len[b] = st, len(st)
            st = o.compact(st)
            data[b, : len(st)], length[b] = st, len(st)
        shortened += int((length < raw_len).sum())
        states = data[np.arange(B), length - 1].copy()
        lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=3, stack_cap=cap, compact_cycles=True, **options)
        assert lib.reduction_cycles() == o.cycles(), text
        m_d = torch.zeros((B, W), dtype=torch.int32, device=dev)
        # a stack that was never compacted still gets its exact mask
        r_st = torch.from_numpy(raw[np.arange(B), raw_len - 1].copy()).to(dev)
        lib.fill_mask(r_st, torch.from_numpy(raw).to(dev), torch.from_numpy(raw_len).to(dev), m_d)
        want = o.fill_mask(states, data, length, v)
        assert (m_d.cpu().numpy().view(np.uint32) == want).all(), text
        st_d, da_d, ln_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
        err_d = torch.zeros(B, dtype=torch.int32, device=dev)
        lib.bind_state(st_d, da_d, ln_d, err_d)
        out = torch.zeros((B, 4), dtype=torch.uint8, device=dev)
        cnt = torch.zeros(B, dtype=torch.int32, device=dev)
        for step in range(9):
            toks = np.array([rnd.randrange(V) if rnd.random() < 0.3 else -2 for _ in range(B)], dtype=np.int32)
            for b in range(B):                           # mostly allowed tokens, so that the stacks move
                if toks[b] == -2:
                    row = o.mask_row(data[b, : length[b]], v, done=states[b] < 0)
                    ids = np.flatnonzero((row[np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1)
                    ids = ids[ids != v.eos_id]
                    toks[b] = int(ids[rnd.randrange(len(ids))]) if len(ids) else -1
            e_h = o.advance_batch(states, data, length, toks, v)
            if step % 3 == 0:
                lib.advance(torch.from_numpy(toks).to(dev))
            else:
                lib.advance_fill_mask(torch.from_numpy(toks).to(dev), m_d)
                assert (m_d.cpu().numpy().view(np.uint32) == o.fill_mask(states, data, length, v)).all(), (text, step)
            if step % 3 == 2:
                want_bytes, want_cnt = o.jump_forward_batch(states, data, length, 4)
                lib.jump_forward(out, cnt)
                assert cnt.cpu().numpy().tolist() == want_cnt.tolist(), (text, step)
            assert (err_d.cpu().numpy() == e_h).all(), (text, step)
            assert (st_d.cpu().numpy() == states).all() and (ln_d.cpu().numpy() == length).all(), (text, step)
            live = np.arange(cap)[None, :] < length[:, None]
            assert (da_d.cpu().numpy()[live] == data[live]).all(), (text, step)
    assert shortened > 20, shortened
