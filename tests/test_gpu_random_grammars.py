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
