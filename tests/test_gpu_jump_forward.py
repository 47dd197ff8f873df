"""pre3_jump_forward through the C ABI against the CPU oracle: forced bytes, their counts and the
advanced stacks along seeded trajectories (JSON, schema grammars with fixed keys, several grammars
in one handle), hand cases, a tight stack capacity, and a decode loop that uses it."""
import json

import numpy as np
import pytest

from oracle import Oracle, masked_argmax as oracle_masked_argmax
from workloads import trajectory
from workloads import grammars as G
from workloads.vocab import BASE_SEED, bf16_logits, bpe_like_vocab

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch, torch.device("cuda:0")


def _jump(lib, states, data, length, max_bytes):
    """Runs the device call on copies of the given host state; returns host arrays."""
    torch, dev = _torch()
    B = len(states)
    st, da, ln = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    err = torch.full((B,), 7, dtype=torch.int32, device=dev)
    lib.bind_state(st, da, ln, err)
    out = torch.full((B, max(1, max_bytes)), 0xEE, dtype=torch.uint8, device=dev)[:, :max_bytes].contiguous()
    cnt = torch.full((B,), -5, dtype=torch.int32, device=dev)
    lib.jump_forward(out, cnt)
    assert (err.cpu().numpy() == 7).all(), "err is not touched"
    return out.cpu().numpy(), cnt.cpu().numpy(), st.cpu().numpy(), da.cpu().numpy(), ln.cpu().numpy()


def _compare(o, lib, states, data, length, max_bytes):
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    want_bytes, want_cnt = o.jump_forward_batch(s_h, d_h, l_h, max_bytes)
    got_bytes, got_cnt, s_g, d_g, l_g = _jump(lib, states, data, length, max_bytes)
    assert got_cnt.tolist() == want_cnt.tolist()
    for b in range(len(states)):
        assert got_bytes[b, : got_cnt[b]].tobytes() == want_bytes[b, : want_cnt[b]].tobytes(), b
    assert (s_g == s_h).all() and (l_g == l_h).all()
    live = np.arange(data.shape[1])[None, :] < l_h[:, None]
    assert (d_g[live] == d_h[live]).all()
    return int(want_cnt.sum())


@pytest.mark.parametrize("which,steps,max_bytes", [("json", 40, 8), ("schema", 60, 64), ("schema", 30, 3), ("mixed", 40, 16)])
def test_forced_bytes_along_trajectories(which, steps, max_bytes):
    from paper_2506_03887_amd import Pre3
    v = bpe_like_vocab(4000, 12, BASE_SEED + 71)
    if which == "json":
        texts, gi = [G.JSON], None
    elif which == "schema":
        texts, gi = [G.schema_grammar(11, 6, 2, 4).text], None
    else:
        texts, gi = [G.schema_grammar(12, 5, 2, 3).text, G.JSON, G.schema_grammar(13, 8, 1, 5).text], np.arange(24) % 3
    o = Oracle(texts)
    B, cap = 24, 256
    lib = Pre3(texts, v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    drv = trajectory.Driver(o, v, B, cap, 17, gi, 5, None, True)
    forced = 0
    for _ in range(steps):
        forced += _compare(o, lib, drv.states, drv.data, drv.len, max_bytes)
        drv.step(last_step=False)
    assert forced > (50 if which != "json" else 3), forced


def test_hand_cases_and_tight_capacity():
    from paper_2506_03887_amd import Pre3
    v = bpe_like_vocab(1000, 8, BASE_SEED + 72)
    o = Oracle([G.JSON])
    cap = 40
    lib = Pre3([G.JSON], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    prefixes = [b"t", b"[tru", b"n", b"fa", b'"', b"[", b'{"a"', b"[1,", b"1", b"", b"[" * 10 + b"nul", b"[[f"]
    B = len(prefixes) + 1
    data = np.zeros((B, cap), dtype=np.int32)
    length = np.ones(B, dtype=np.int32)
    for b, p in enumerate(prefixes):
        st = o.initial_stack() if not p else o.advance(o.initial_stack(), p)[1]
        data[b, : len(st)], length[b] = st, len(st)
    data[B - 1, 0] = o.initial_state(0)
    states = data[np.arange(B), length - 1].copy()
    states[B - 1] = -1                                        # a finished sequence
    got_bytes, got_cnt, s_g, _, l_g = _jump(lib, states, data, length, 8)
    texts = [got_bytes[b, : got_cnt[b]].tobytes() for b in range(B)]
    assert texts == [b"rue", b"e", b"ull", b"lse", b"", b"", b"", b"", b"", b"", b"l", b"alse", b""]
    assert s_g[B - 1] == -1 and l_g[B - 1] == 1
    _compare(o, lib, states, data, length, 8)
    _compare(o, lib, states, data, length, 0)
    _compare(o, lib, states, data, length, 1)
    # capacity reached in the middle of a forced run: stop before the byte that does not fit
    deep = o.advance(o.initial_stack(), b"[" * 10 + b"t")[1]
    for room in (0, 1, 2):
        c = len(deep) + room
        lib2 = Pre3([G.JSON], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=c)
        d2 = np.zeros((1, c), dtype=np.int32)
        d2[0, : len(deep)] = deep
        _compare(o, lib2, np.array([deep[-1]], dtype=np.int32), d2, np.array([len(deep)], dtype=np.int32), 8)


def test_decode_loop_with_jump_forward_emits_valid_documents():
    """Greedy decoding of a schema grammar where, after every sampled token, the forced bytes are
    appended without a model call; both sides in lockstep, and finished texts parse as JSON."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    v = bpe_like_vocab(6000, 12, BASE_SEED + 73)
    text = G.schema_grammar(14, 6, 2, 4).text
    o = Oracle([text])
    B, V, W, cap = 32, v.n_tokens, v.words, 512
    lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    s0 = o.initial_state(0)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h, states_h = np.ones(B, dtype=np.int32), np.full(B, s0, dtype=np.int32)
    st, da, ln = (torch.from_numpy(x.copy()).to(dev) for x in (states_h, data_h, len_h))
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(st, da, ln, err)
    mask = torch.empty((B, W), dtype=torch.int32, device=dev)
    tok = torch.empty(B, dtype=torch.int32, device=dev)
    jb = torch.empty((B, 48), dtype=torch.uint8, device=dev)
    jn = torch.empty(B, dtype=torch.int32, device=dev)
    rng = np.random.default_rng(5)
    texts = [bytearray() for _ in range(B)]
    finished = [None] * B
    forced_total = 0
    lib.jump_forward(jb, jn)                                   # the document's opening may be forced too
    o.jump_forward_batch(states_h, data_h, len_h, 48)
    for s in range(200):
        lib.fill_mask(st, da, ln, mask)
        logits = bf16_logits(rng, B, V)
        eos_boost = logits[:, v.eos_id].astype(np.uint32) << 16
        logits[:, v.eos_id] = ((eos_boost.view(np.float32) + 3.0).view(np.uint32) >> 16).astype(np.uint16)
        mask_h = o.fill_mask(states_h, data_h, len_h, v)
        assert (mask.cpu().numpy().view(np.uint32) == mask_h).all()
        want = oracle_masked_argmax(logits, mask_h, V)
        want[states_h < 0] = -1
        lib.apply_mask_argmax(torch.from_numpy(logits.view(np.int16)).to(dev).view(torch.bfloat16), mask, tok)
        tk = torch.where(st >= 0, tok, torch.full_like(tok, -1))
        assert tk.cpu().numpy().tolist() == want.tolist()
        lib.advance(tk)
        e_h = o.advance_batch(states_h, data_h, len_h, want, v)
        assert (err.cpu().numpy() == e_h).all()
        lib.jump_forward(jb, jn)
        wb, wn = o.jump_forward_batch(states_h, data_h, len_h, 48)
        gb, gn = jb.cpu().numpy(), jn.cpu().numpy()
        assert gn.tolist() == wn.tolist()
        for b in range(B):
            if want[b] < 0 or e_h[b] != 0:
                continue
            if want[b] == v.eos_id:
                finished[b] = bytes(texts[b])
                continue
            assert gb[b, : gn[b]].tobytes() == wb[b, : wn[b]].tobytes()
            texts[b] += v.tokens[want[b]] + gb[b, : gn[b]].tobytes()
            forced_total += int(gn[b])
        assert (st.cpu().numpy() == states_h).all() and (ln.cpu().numpy() == len_h).all()
    done = [t for t in finished if t is not None]
    assert len(done) >= 4 and forced_total > 200, (len(done), forced_total)
    for t in done:
        json.loads(t.decode("latin-1"))


def test_runs_of_forced_bytes_longer_than_a_wave():
    """A literal of 100 bytes, a choice, a literal of 70 bytes: the forced runs are cut at max_bytes, at the
    64 bytes one step can take, at the choice, at the end of the sentence and at the stack capacity, always where
    the oracle's byte-by-byte search stops."""
    from paper_2506_03887_amd import Pre3
    v = bpe_like_vocab(500, 6, BASE_SEED + 73)
    lit1 = bytes(97 + (7 * i) % 26 for i in range(100))
    lit2 = bytes(48 + (3 * i) % 10 for i in range(70))
    text = 'S ::= "%s" T "%s"\nT ::= "x" | "y"' % (lit1.decode(), lit2.decode())
    o = Oracle([text])
    cap = 256
    lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    prefixes = [b"", lit1[:1], lit1[:36], lit1[:99], lit1, lit1 + b"x", lit1 + b"y" + lit2[:69], lit1 + b"x" + lit2]
    B = len(prefixes)
    data = np.zeros((B, cap), dtype=np.int32)
    length = np.ones(B, dtype=np.int32)
    for b, p in enumerate(prefixes):
        st = o.initial_stack() if not p else o.advance(o.initial_stack(), p)[1]
        data[b, : len(st)], length[b] = st, len(st)
    states = data[np.arange(B), length - 1].copy()
    for max_bytes in (1, 31, 63, 64, 65, 100, 101, 128, 200):
        forced = _compare(o, lib, states, data, length, max_bytes)
        assert forced > 0
    got_bytes, got_cnt, _, _, _ = _jump(lib, states, data, length, 200)
    assert got_bytes[0, : got_cnt[0]].tobytes() == lit1 and got_bytes[5, : got_cnt[5]].tobytes() == lit2 and got_cnt[7] == 0
    # the capacity ends a run in its middle: 1 .. 70 entries of room above the stack after the first literal and "x"
    deep = o.advance(o.initial_stack(), lit1 + b"x")[1]
    for room in (0, 1, 5, 63, 64, 65, 69, 70, 71):
        c = len(deep) + room
        lib2 = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=c)
        d2 = np.zeros((1, c), dtype=np.int32)
        d2[0, : len(deep)] = deep
        _compare(o, lib2, np.array([deep[-1]], dtype=np.int32), d2, np.array([len(deep)], dtype=np.int32), 200)
