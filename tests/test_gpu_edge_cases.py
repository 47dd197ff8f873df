"""GPU edge cases through the C ABI, each checked against the CPU oracle: empty batch, ragged
vocabulary sizes, strided / unaligned logits, every per-sequence error of advance, finished
rows, tokens deep enough to spill the private stack, snapshots, HIP-graph replay."""
import numpy as np
import pytest

from oracle import Oracle, apply_mask as oracle_apply_mask, masked_argmax as oracle_masked_argmax
from workloads import grammars as G
from workloads.vocab import BASE_SEED, Vocab, bf16_logits, bpe_like_vocab

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch, torch.device("cuda:0")


def _lib(grammars, vocab, **kw):
    from paper_2506_03887_amd import Pre3
    return Pre3(grammars, vocab.bytes, vocab.offsets, vocab.eos_id, max_token_len=max(1, vocab.max_len), **kw)


def _stacks(o, prefixes, cap, grammar=0):
    B = len(prefixes)
    data = np.zeros((B, cap), dtype=np.int32)
    length = np.ones(B, dtype=np.int32)
    for b, p in enumerate(prefixes):
        rc, st = (0, o.initial_stack(grammar)) if not p else o.advance(o.initial_stack(grammar), p)
        assert rc == 0, p
        data[b, : len(st)] = st
        length[b] = len(st)
    states = data[np.arange(B), length - 1].copy()
    return states, data, length


def _gpu_mask(lib, states, data, length, words):
    torch, dev = _torch()
    m = torch.full((len(states), words), 0x77777777, dtype=torch.int32, device=dev)
    lib.fill_mask(torch.from_numpy(states).to(dev), torch.from_numpy(data).to(dev), torch.from_numpy(length).to(dev), m)
    return m.cpu().numpy().view(np.uint32)


@pytest.fixture(scope="module")
def deep_vocab():
    """JSON vocabulary with tokens that nest up to 32 levels in one token (private stacks of the
    walk spill from LDS to global memory), empty tokens, duplicates and a ragged size."""
    base = bpe_like_vocab(3000, 16, BASE_SEED + 77).tokens[:-1]
    extra = [b"[" * 32, b"[" * 17 + b"1", b"[[[[[[[[[[[[[[[[[[[[{\"a\":[[", b"{\"k\":" * 6, b"[" * 9 + b"]" * 9,
             b"", b"", b"[" * 32, b"]" * 20, b"\"" + b"x" * 30 + b"\"", b"[1," * 10, b"]]]]]]]],"]
    toks = base + extra + [b""]                  # EOS last
    assert len(toks) % 32 != 0 and len(toks) % 8 != 0
    return Vocab(toks, len(toks) - 1)


@pytest.mark.parametrize("token_edges", [True, False])
def test_deep_tokens_spill_the_private_stack(deep_vocab, token_edges):
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v, token_edges=token_edges, max_condition_depth=3 if token_edges else 0)
    assert lib.walk_depth_bound > 16
    prefixes = [b"", b"[", b"[[[[[[[[[", b'{"a":', b'{"a":[[[[[[[[[[[[[[[[[[[[', b'"abc', b"[1", b"[[[[[[[[[1" + b"]" * 3, b"12"]
    states, data, length = _stacks(o, prefixes, 256)
    got = _gpu_mask(lib, states, data, length, v.words)
    want = o.fill_mask(states, data, length, v)
    assert (got == want).all()
    # the deep tokens really are allowed somewhere, and equal strings get equal bits
    t_deep = [t for t, tok in enumerate(v.tokens) if tok == b"[" * 32]
    assert len(t_deep) == 2
    for b in range(len(prefixes)):
        bits = [(want[b, t >> 5] >> (t & 31)) & 1 for t in t_deep]
        assert bits[0] == bits[1]
    assert (want[0, t_deep[0] >> 5] >> (t_deep[0] & 31)) & 1
    # advance by the deep tokens, token by token, against the oracle
    torch, dev = _torch()
    toks = np.array([t_deep[0], t_deep[1], v.tokens.index(b"]]]]]]]],"), v.tokens.index(b"[" * 17 + b"1"),
                     v.tokens.index(b"]" * 20), -1, v.tokens.index(b"[1," * 10), v.tokens.index(b"]]]]]]]],"),
                     v.eos_id], dtype=np.int32)
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    e_d = torch.full((len(toks),), -5, dtype=torch.int32, device=dev)
    lib.bind_state(s_d, d_d, l_d, e_d)
    lib.advance(torch.from_numpy(toks).to(dev))
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    err = o.advance_batch(s_h, d_h, l_h, toks, v)
    assert (e_d.cpu().numpy() == err).all() and set(err.tolist()) >= {0, 1}
    assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all()
    live = np.arange(256)[None, :] < l_h[:, None]
    assert (d_d.cpu().numpy()[live] == d_h[live]).all()
    assert l_h.max() > 60                                        # a 32-bracket token was committed


@pytest.mark.parametrize("grammar,compact,token_edges", [("JSON", False, True), ("JSON", False, False),
                                                         ("JSON_RIGHT_RECURSIVE", True, True), ("JSON_RIGHT_RECURSIVE", False, True)])
def test_tokens_of_the_maximum_length(grammar, compact, token_edges):
    """Tokens of 254 bytes, the longest the library accepts (and of 65..253): strings, digits, white
    space, escapes, 254 opening brackets, lists -- beyond the bytes a walk stages per token and beyond
    the length of a run; masks on several stacks and an advance by each of them against the oracle."""
    torch, dev = _torch()
    text = getattr(G, grammar)
    base = bpe_like_vocab(400, 8, BASE_SEED + 79).tokens[:-1]
    long_tokens = [b'"' + b"x" * 252 + b'"', b"[" * 254, b"1" * 254, b'"' + b"ab" * 100, b"[1," * 84, b" " * 254,
                   b'"' + b"\\n" * 120 + b'"', b"7" * 65, b'"' + b"y" * 63, b'"' + b"y" * 64 + b'"', b"[" * 100 + b"]" * 100,
                   b"[[],[[]],{}," * 21, b'{"k":' * 50, b'"' + b"z" * 253 + b'"x']
    assert max(len(t) for t in long_tokens) == 256 and sum(len(t) == 254 for t in long_tokens) >= 4
    long_tokens[-1] = long_tokens[-1][:254]              # 254 bytes that end inside the string
    toks = base + long_tokens + [b""]
    v = Vocab(toks, len(toks) - 1)
    assert v.max_len == 254
    cap = 1024
    o = Oracle([text], compact_cycles=compact)
    from paper_2506_03887_amd import Pre3
    lib = Pre3([text], v.bytes, v.offsets, v.eos_id, max_token_len=254, stack_cap=cap, token_edges=token_edges,
               compact_cycles=compact)
    prefixes = [b"", b"[", b'{"a":', b'"abc', b"[1", b"[[[[", b'{"a":[1,', b"12", b'["q",', b"[ ", b'"\\', b"[[[[[[[[[[", b"-", b'{"k":{"k":']
    states, data, length = _stacks(o, prefixes, cap)
    if compact:
        o.compact_batch(data, length)
    B = len(prefixes)
    got = _gpu_mask(lib, states, data, length, v.words)
    want = o.fill_mask(states, data, length, v)
    assert (got == want).all()
    first_long = len(base)
    allowed_long = sum(int((want[b, t >> 5] >> (t & 31)) & 1) for b in range(B) for t in range(first_long, first_long + len(long_tokens)))
    assert allowed_long >= 25, allowed_long
    for k in range(len(long_tokens)):                    # every sequence takes long token k (allowed or not)
        s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
        s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
        e_d = torch.full((B,), -5, dtype=torch.int32, device=dev)
        m_d = torch.zeros((B, v.words), dtype=torch.int32, device=dev)
        lib.bind_state(s_d, d_d, l_d, e_d)
        tok = np.full(B, first_long + k, dtype=np.int32)
        if k % 2:
            lib.advance(torch.from_numpy(tok).to(dev))
        else:
            lib.advance_fill_mask(torch.from_numpy(tok).to(dev), m_d)
        err = o.advance_batch(s_h, d_h, l_h, tok, v)
        assert (e_d.cpu().numpy() == err).all(), (k, long_tokens[k][:12])
        assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all(), k
        live = np.arange(cap)[None, :] < l_h[:, None]
        assert (d_d.cpu().numpy()[live] == d_h[live]).all(), k
        if k % 2 == 0:
            assert (m_d.cpu().numpy().view(np.uint32) == o.fill_mask(s_h, d_h, l_h, v)).all(), k


def test_very_deep_stacks(deep_vocab):
    """Stacks of tens of thousands of entries (capacity 65,536): 9,000 to 32,750 open brackets, then
    masks, advances that close many levels at once, and an advance that would pass the capacity."""
    torch, dev = _torch()
    o = Oracle(G.JSON)
    v = deep_vocab
    cap = 65536
    lib = _lib(G.JSON, v, stack_cap=cap)
    prefixes = [b"[" * 9000, b"[" * 30000 + b"1", b'{"a":' * 3000 + b"[", b"[" * 32750, b"[" * 32740 + b'"s"']
    states, data, length = _stacks(o, prefixes, cap)
    assert length.max() > 65000 and length.min() > 15000
    got = _gpu_mask(lib, states, data, length, v.words)
    assert (got == o.fill_mask(states, data, length, v)).all()
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    e_d = torch.full((len(prefixes),), -5, dtype=torch.int32, device=dev)
    m_d = torch.zeros((len(prefixes), v.words), dtype=torch.int32, device=dev)
    lib.bind_state(s_d, d_d, l_d, e_d)
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    seq = [[v.tokens.index(b"[" * 32), v.tokens.index(b"]]]]]]]],"), v.tokens.index(b"[1," * 10), v.tokens.index(b"[" * 32),
            v.tokens.index(b"]" * 20)],
           [v.tokens.index(b"]" * 20)] * 5]
    for step in range(5):
        tok = np.array([seq[0][step], seq[1][step], seq[0][step], seq[0][step], seq[1][step]], dtype=np.int32)
        if step % 2:
            lib.advance(torch.from_numpy(tok).to(dev))
        else:
            lib.advance_fill_mask(torch.from_numpy(tok).to(dev), m_d)
        err = o.advance_batch(s_h, d_h, l_h, tok, v)
        assert (e_d.cpu().numpy() == err).all(), step
        assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all(), step
        live = np.arange(cap)[None, :] < l_h[:, None]
        assert (d_d.cpu().numpy()[live] == d_h[live]).all(), step
        if step % 2 == 0:
            assert (m_d.cpu().numpy().view(np.uint32) == o.fill_mask(s_h, d_h, l_h, v)).all(), step
        if step == 0:
            assert err[3] == 2 and err[0] == 0               # 32 more brackets do not fit under the capacity


@pytest.mark.parametrize("token_edges", [True, False])
def test_vocabulary_of_arbitrary_bytes(token_edges):
    """Tokens drawn from all 256 byte values (NUL, control bytes, 0x80..0xFF, quotes and backslashes in
    any position), duplicates and empty tokens included; masks on stacks inside and outside strings,
    then every sequence advances by a random token of the vocabulary, allowed or not."""
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + 83)
    toks = [bytes(rng.integers(0, 256, size=int(rng.integers(1, 7)), dtype=np.uint8).tolist()) for _ in range(5000)]
    toks += [bytes([c]) for c in range(256)] + [b"", b"", toks[3], toks[3], b"\x00", b"\xff\xfe", b'"\x80"', b"\\\xff"]
    toks.append(b"")
    v = Vocab(toks, len(toks) - 1)
    o = Oracle(G.JSON)
    lib = _lib(G.JSON, v, token_edges=token_edges)
    prefixes = [b"", b'"', b'"\x80\xffa', b'"\\', b'["\x7f', b'{"k\xc3\xa9":"', b"[1", b'{"a":', b'"\\u00', b"[[[", b'{"a":"b",', b"tru"]
    states, data, length = _stacks(o, prefixes, 64)
    got = _gpu_mask(lib, states, data, length, v.words)
    want = o.fill_mask(states, data, length, v)
    assert (got == want).all()
    assert want[1].view(np.uint8).sum() > want[0].view(np.uint8).sum()     # inside a string far more tokens are allowed
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    e_d = torch.full((len(prefixes),), -5, dtype=torch.int32, device=dev)
    lib.bind_state(s_d, d_d, l_d, e_d)
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    n_ok = 0
    for step in range(40):
        tok = rng.integers(0, v.n_tokens, size=len(prefixes)).astype(np.int32)
        if step % 2:                                          # every other step: a token that is allowed, if any
            for b in range(len(prefixes)):
                row = o.mask_row(d_h[b, : l_h[b]], v, done=s_h[b] < 0)
                ids = np.flatnonzero((row[np.arange(v.n_tokens) >> 5] >> (np.arange(v.n_tokens) & 31).astype(np.uint32)) & 1)
                ids = ids[ids != v.eos_id]
                if len(ids):
                    tok[b] = ids[rng.integers(len(ids))]
        lib.advance(torch.from_numpy(tok).to(dev))
        err = o.advance_batch(s_h, d_h, l_h, tok, v)
        n_ok += int((err == 0).sum())
        assert (e_d.cpu().numpy() == err).all(), step
        assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all(), step
        live = np.arange(64)[None, :] < l_h[:, None]
        assert (d_d.cpu().numpy()[live] == d_h[live]).all(), step
    assert n_ok > 150
    assert (_gpu_mask(lib, s_h, d_h, l_h, v.words) == o.fill_mask(s_h, d_h, l_h, v)).all()


def test_advance_error_codes_and_overflow(deep_vocab):
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v)
    torch, dev = _torch()
    cap = 24
    prefixes = [b"[[[[[[[[[[", b"[[[[[[[[[[", b"[1", b"[1", b"12", b"12", b"[1", b"{"]
    states, data, length = _stacks(o, prefixes, cap)
    states[5] = -1                                               # a finished sequence
    tok = {t: i for i, t in reversed(list(enumerate(v.tokens))) if i != v.eos_id}
    toks = np.array([tok[b"[" * 9 + b"]" * 9],                    # transient overflow of cap -> 2
                     tok[b"]"],                                    # fine
                     tok[b"}"],                                    # not allowed -> 1
                     v.eos_id,                                     # EOS where the text is no sentence -> 1
                     v.eos_id,                                     # EOS allowed -> DONE
                     tok[b"1"],                                    # any token on a finished sequence -> 1
                     v.n_tokens + 5,                               # id out of range -> 1
                     [t for t, s in enumerate(v.tokens) if s == b"" and t != v.eos_id][0]],   # empty token -> 1
                    dtype=np.int32)
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    e_d = torch.full((len(toks),), -5, dtype=torch.int32, device=dev)
    lib.bind_state(s_d, d_d, l_d, e_d)
    lib.advance(torch.from_numpy(toks).to(dev))
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    err = o.advance_batch(s_h, d_h, l_h, toks, v)
    assert err.tolist() == [2, 0, 1, 1, 0, 1, 1, 1]
    assert (e_d.cpu().numpy() == err).all()
    assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all() and s_h[4] == -1
    live = np.arange(cap)[None, :] < l_h[:, None]
    assert (d_d.cpu().numpy()[live] == d_h[live]).all()
    # failing sequences are untouched, including the part of the row above len
    for b in (0, 2, 3, 5, 6, 7):
        assert (d_d.cpu().numpy()[b] == data[b]).all() and l_h[b] == length[b]
    # a finished row gets only the EOS bit; fill_mask reads snapshots that need not be the bound buffers
    got = _gpu_mask(lib, s_h, d_h, l_h, v.words)
    assert (got == o.fill_mask(s_h, d_h, l_h, v)).all()
    only_eos = np.zeros(v.words, dtype=np.uint32)
    only_eos[v.eos_id >> 5] = 1 << (v.eos_id & 31)
    assert (got[4] == only_eos).all() and (got[5] == only_eos).all()


def test_empty_batch_and_single_row(deep_vocab):
    torch, dev = _torch()
    from paper_2506_03887_amd import apply_mask
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v)
    z32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
    lib.fill_mask(z32(0), z32(0, 8), z32(0), z32(0, v.words))
    lib.fill_apply_mask(z32(0), z32(0, 8), z32(0), z32(0, v.words), torch.zeros((0, v.n_tokens), dtype=torch.bfloat16, device=dev))
    apply_mask(torch.zeros((0, v.n_tokens), dtype=torch.bfloat16, device=dev), z32(0, v.words), v.n_tokens)
    lib.bind_state(z32(0), z32(0, 8), z32(0), z32(0))
    lib.advance(z32(0))
    torch.cuda.synchronize()
    states, data, length = _stacks(o, [b'{"a": [1, '], 64)
    assert (_gpu_mask(lib, states, data, length, v.words) == o.fill_mask(states, data, length, v)).all()


@pytest.mark.parametrize("V,stride,offset", [(513, 513, 0), (1000, 1000, 0), (1000, 1008, 0), (1003, 1016, 0),
                                             (1000, 1001, 0), (264, 264, 3), (40000, 40008, 8)])
def test_apply_mask_layouts(V, stride, offset):
    """Ragged vocabulary sizes, padded rows, rows that are not 16-byte aligned (scalar path),
    NaN / inf payloads: the result is a pure select on raw bf16 patterns."""
    torch, dev = _torch()
    from paper_2506_03887_amd import apply_mask
    rng = np.random.default_rng(V + stride)
    B, W = 7, (V + 31) // 32
    host = np.full((B, stride), 0x1234, dtype=np.uint16)
    host[:, :V] = bf16_logits(rng, B, V)
    host[0, :6] = [0x7FC1, 0xFFC0, 0x7F80, 0xFF80, 0x0000, 0x8000]
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[1], mask[2] = 0, 0xFFFFFFFF
    mask[3, ::2], mask[4, 1::2] = 0, 0xFFFFFFFF
    flat = torch.zeros(B * stride + offset + 16, dtype=torch.int16, device=dev)
    view = flat[offset: offset + B * stride].view(B, stride)
    view.copy_(torch.from_numpy(host.view(np.int16)).to(dev))
    apply_mask(view[:, :V] if stride == V else view, torch.from_numpy(mask.view(np.int32)).to(dev), V)
    want = host.copy()
    oracle_apply_mask(want, mask, V)
    assert (view.cpu().numpy().view(np.uint16) == want).all()
    assert int(flat[:offset].abs().sum()) == 0 and int(flat[offset + B * stride:].abs().sum()) == 0


@pytest.mark.parametrize("B", [1003, 1100])
def test_apply_mask_on_both_sides_of_the_grid_switch(B):
    """pre3_apply_mask orders its blocks by the XCD that wrote a row's mask while the mask fits the L2s
    (16 MB) and falls back to the (span, row) grid beyond: at V = 128,256 the switch lies between 1,046 and
    1,047 rows.  Batches that are no multiple of 8 on both sides, every logit compared."""
    torch, dev = _torch()
    from paper_2506_03887_amd import apply_mask
    V = 128256
    W = (V + 31) // 32
    assert (B * W * 4 <= 16 << 20) == (B == 1003)
    rng = np.random.default_rng(B)
    host = bf16_logits(rng, B, V)
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[1::5] &= rng.integers(0, 2 ** 32, size=mask[1::5].shape, dtype=np.uint64).astype(np.uint32)
    mask[2::7] = 0
    mask[3::11] = 0xFFFFFFFF
    mask[B - 1, ::3] = 0
    logits = torch.from_numpy(host.view(np.int16)).to(dev)
    apply_mask(logits.view(torch.bfloat16), torch.from_numpy(mask.view(np.int32)).to(dev), V)
    want = host.copy()
    oracle_apply_mask(want, mask, V)
    got = logits.cpu().numpy().view(np.uint16)
    assert (got == want).all(), np.argwhere(got != want)[:4].tolist()


def test_batches_beyond_the_grid_limit_of_one_dimension():
    """More rows than a grid dimension holds (65,535): pre3_apply_mask switches to its flat kernel,
    the arg max and the top-k put the rows on the x dimension.  Small vocabulary, every row checked."""
    torch, dev = _torch()
    from oracle import masked_argmax as oracle_masked_argmax, masked_topk as oracle_masked_topk
    from paper_2506_03887_amd import Pre3, apply_mask
    from workloads.vocab import Vocab
    V, B, cap = 72, 70001, 4
    W = (V + 31) // 32
    rng = np.random.default_rng(V + B)
    logits = bf16_logits(rng, B, V)
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[:, W - 1] &= np.uint32((1 << (V % 32)) - 1)
    mask[5], mask[B - 1] = 0, 0
    mask[B - 1, 1] = 1 << 7
    toks = [bytes([97 + i % 5]) for i in range(V - 1)] + [b""]
    v = Vocab(toks, V - 1)
    lib = Pre3(G.ARITHMETIC, v.bytes, v.offsets, v.eos_id, max_token_len=1, stack_cap=cap)
    s0 = lib.initial_state(0)
    keep = (torch.full((B,), s0, dtype=torch.int32, device=dev), torch.full((B, cap), s0, dtype=torch.int32, device=dev),
            torch.ones(B, dtype=torch.int32, device=dev), torch.zeros(B, dtype=torch.int32, device=dev))
    lib.bind_state(*keep)
    l_d = torch.from_numpy(logits.view(np.int16)).to(dev)
    m_d = torch.from_numpy(mask.view(np.int32)).to(dev)
    tok = torch.full((B,), -7, dtype=torch.int32, device=dev)
    lib.apply_mask_argmax(l_d.view(torch.bfloat16), m_d, tok)
    assert (tok.cpu().numpy() == oracle_masked_argmax(logits, mask, V)).all()
    ids = torch.full((B, 5), -7, dtype=torch.int32, device=dev)
    vals = torch.zeros((B, 5), dtype=torch.int16, device=dev)
    lib.apply_mask_topk(l_d.view(torch.bfloat16), m_d, ids, vals)
    want_ids, want_vals = oracle_masked_topk(logits, mask, V, 5)
    assert (ids.cpu().numpy() == want_ids).all() and (vals.cpu().numpy().view(np.uint16) == want_vals).all()
    assert want_ids[B - 1].tolist() == [39, -1, -1, -1, -1] and (want_ids[5] == -1).all()
    apply_mask(l_d, m_d, V)
    want = logits.copy()
    oracle_apply_mask(want, mask, V)
    assert (l_d.cpu().numpy().view(np.uint16) == want).all()
    # a stack advance over the same batch: every sequence takes the token "a" (id 0 spells "a")
    tokens = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.advance(tokens)
    o = Oracle([G.ARITHMETIC])
    rc, st = o.advance(o.initial_stack(), b"a")
    assert rc == 0 and (keep[3].cpu().numpy() == 0).all() and (keep[2].cpu().numpy() == len(st)).all()
    assert (keep[1].cpu().numpy()[:, : len(st)] == np.array(st, dtype=np.int32)).all()


@pytest.mark.parametrize("stride_pad,offset", [(0, 0), (8, 0), (3, 0), (0, 4)])
def test_fused_call_equals_two_calls_on_any_layout(deep_vocab, stride_pad, offset):
    torch, dev = _torch()
    from paper_2506_03887_amd import apply_mask
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v)
    prefixes = [b"", b'{"a', b"[1", b'{"k": [tr', b"[[[[", b'"x\\', b"12.5e", b" 7 ", b'{"a":{"b":[{},[[]],"']
    states, data, length = _stacks(o, prefixes, 64)
    states[7] = -1
    B, V, stride = len(prefixes), v.n_tokens, v.n_tokens + stride_pad
    host = np.full((B, stride), 0x4321, dtype=np.uint16)
    host[:, :V] = bf16_logits(np.random.default_rng(5), B, V)
    flat = torch.zeros(B * stride + offset + 8, dtype=torch.int16, device=dev)
    view = flat[offset: offset + B * stride].view(B, stride)
    view.copy_(torch.from_numpy(host.view(np.int16)).to(dev))
    s_d, d_d, l_d = (torch.from_numpy(x).to(dev) for x in (states, data, length))
    m = torch.full((B, v.words), 0x11111111, dtype=torch.int32, device=dev)
    lib.fill_apply_mask(s_d, d_d, l_d, m, view)
    want_mask = o.fill_mask(states, data, length, v)
    want = host.copy()
    oracle_apply_mask(want, want_mask, V)
    assert (m.cpu().numpy().view(np.uint32) == want_mask).all()
    assert (view.cpu().numpy().view(np.uint16) == want).all()


@pytest.mark.parametrize("stride_pad,offset,one_kernel", [(0, 0, True), (8, 0, True), (3, 0, True), (0, 4, True), (16, 8, True),
                                                          (0, 0, False)])
def test_whole_step_call_error_codes_overflow_and_layouts(deep_vocab, stride_pad, offset, one_kernel):
    """pre3_advance_fill_apply_mask on the token mix of the advance test (overflow of the capacity, tokens that
    are not allowed, EOS allowed and not, a finished sequence, an id out of range, the empty token) and on
    padded, offset and misaligned rows of logits (where the rows are not 16-byte aligned the call takes
    its two-call form): err, states, stacks, the mask of the resulting stacks and every logit pattern,
    padding included, are the oracle's; the buffers around the logits stay untouched."""
    torch, dev = _torch()
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v)
    cap = 24
    prefixes = [b"[[[[[[[[[[", b"[[[[[[[[[[", b"[1", b"[1", b"12", b"12", b"[1", b"{", b'{"a": [tr']
    states, data, length = _stacks(o, prefixes, cap)
    states[5] = -1
    tok = {t: i for i, t in reversed(list(enumerate(v.tokens))) if i != v.eos_id}
    toks = np.array([tok[b"[" * 9 + b"]" * 9], tok[b"]"], tok[b"}"], v.eos_id, v.eos_id, tok[b"1"], v.n_tokens + 5,
                     [t for t, s in enumerate(v.tokens) if s == b"" and t != v.eos_id][0], -1], dtype=np.int32)
    B, V, stride = len(prefixes), v.n_tokens, v.n_tokens + stride_pad
    host = np.full((B, stride), 0x4321, dtype=np.uint16)
    host[:, :V] = bf16_logits(np.random.default_rng(11), B, V)
    host[0, :6] = [0x7FC1, 0xFFC0, 0x7F80, 0xFF80, 0x0000, 0x8000]
    flat = torch.zeros(B * stride + offset + 8, dtype=torch.int16, device=dev)
    view = flat[offset: offset + B * stride].view(B, stride)
    view.copy_(torch.from_numpy(host.view(np.int16)).to(dev))
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    e_d = torch.full((B,), -5, dtype=torch.int32, device=dev)
    m = torch.full((B, v.words), 0x11111111, dtype=torch.int32, device=dev)
    lib.bind_state(s_d, d_d, l_d, e_d)
    lib.advance_fill_apply_mask(torch.from_numpy(toks).to(dev), m, view, one_kernel=one_kernel)
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    err = o.advance_batch(s_h, d_h, l_h, toks, v)
    assert err.tolist() == [2, 0, 1, 1, 0, 1, 1, 1, 0]
    assert (e_d.cpu().numpy() == err).all()
    assert (s_d.cpu().numpy() == s_h).all() and (l_d.cpu().numpy() == l_h).all() and s_h[4] == -1
    live = np.arange(cap)[None, :] < l_h[:, None]
    assert (d_d.cpu().numpy()[live] == d_h[live]).all()
    for b in (0, 2, 3, 5, 6, 7, 8):                              # failing and skipped sequences are untouched
        assert (d_d.cpu().numpy()[b] == data[b]).all() and l_h[b] == length[b]
    want_mask = o.fill_mask(s_h, d_h, l_h, v)
    assert (m.cpu().numpy().view(np.uint32) == want_mask).all()
    want = host.copy()
    oracle_apply_mask(want, want_mask, V)
    assert (view.cpu().numpy().view(np.uint16) == want).all()
    assert int(flat[:offset].abs().sum()) == 0 and int(flat[offset + B * stride:].abs().sum()) == 0


def test_whole_step_call_rejects_bad_arguments_and_takes_an_empty_batch(deep_vocab):
    torch, dev = _torch()
    from paper_2506_03887_amd.binding import Pre3Error
    o = Oracle(G.JSON)
    v = deep_vocab
    lib = _lib(G.JSON, v)
    z32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
    B, V = 3, v.n_tokens
    logits = torch.zeros((B, V), dtype=torch.int16, device=dev)
    with pytest.raises(Pre3Error):                                # nothing bound yet
        lib.advance_fill_apply_mask(z32(B), z32(B, v.words), logits)
    states, data, length = _stacks(o, [b"[1", b"{", b""], 32)
    s_d, d_d, l_d = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    lib.bind_state(s_d, d_d, l_d, z32(B))
    h, raw = lib._h, lib._lib
    ptr = lambda t: t.data_ptr()
    m, tk = z32(B, v.words), torch.full((B,), -1, dtype=torch.int32, device=dev)
    call = lambda tokens, mask, lg, stride, flags: raw.pre3_advance_fill_apply_mask(h, tokens, mask, lg, stride, flags, None)
    assert call(None, ptr(m), ptr(logits), V, 0) == -1
    assert call(ptr(tk), None, ptr(logits), V, 0) == -1
    assert call(ptr(tk), ptr(m), None, V, 0) == -1
    assert call(ptr(tk), ptr(m), ptr(logits), V - 1, 0) == -1          # rows shorter than the vocabulary
    assert call(ptr(tk), ptr(m), ptr(logits), V, 4) == -1              # unknown flag
    assert call(ptr(tk), ptr(m), ptr(logits) + 1, V + 1, 0) == -1      # logits not 2-byte aligned
    assert call(ptr(tk), ptr(m), ptr(logits), V, 3) == 0               # both flags; tokens of -1 leave the stacks alone
    torch.cuda.synchronize()
    assert (s_d.cpu().numpy() == states).all() and (l_d.cpu().numpy() == length).all()
    assert (m.cpu().numpy().view(np.uint32) == o.fill_mask(states, data, length, v)).all()
    lib.bind_state(z32(0), z32(0, 8), z32(0), z32(0))             # an empty batch: the call does nothing
    lib.advance_fill_apply_mask(z32(0), z32(0, v.words), torch.zeros((0, V), dtype=torch.int16, device=dev), one_kernel=True)
    torch.cuda.synchronize()


def test_hip_graph_replays_match_eager():
    """A captured step (fill -> apply -> advance, kernels only) is replayed several times with
    eager work between the replays (token upload, fresh logits, slot-reuse resets); every
    replay must leave what the eager calls leave."""
    torch, dev = _torch()
    from paper_2506_03887_amd import apply_mask
    from workloads import configs, trajectory
    cfg = configs.get(2)
    v = cfg.vocab
    o = Oracle(cfg.grammars)
    steps = 8
    traj = trajectory.generate(o, v, cfg.batch, steps, cfg.cap, cfg.seed + 3, None, cfg.nest_cap, None, True, None)
    lib = _lib(cfg.grammars, v)
    B, V = cfg.batch, v.n_tokens
    init_data, init_len = torch.from_numpy(traj.init_data).to(dev), torch.from_numpy(traj.init_len).to(dev)
    data, length = init_data.clone(), init_len.clone()
    states = data[:, 0].clone()
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states, data, length, err)
    mask = torch.zeros((B, v.words), dtype=torch.int32, device=dev)
    logits0 = torch.from_numpy(bf16_logits(np.random.default_rng(1), B, V).view(np.int16)).to(dev)
    logits = logits0.clone()
    tok = torch.zeros(B, dtype=torch.int32, device=dev)
    toks = torch.from_numpy(traj.tokens).to(dev)
    reset = torch.from_numpy(traj.reset).to(dev)
    s0 = o.initial_state()

    def start():
        data.copy_(init_data); length.copy_(init_len); states.copy_(init_data[:, 0])

    def eager_inputs(s):
        tok.copy_(toks[s]); logits.copy_(logits0)
        length.masked_fill_(reset[s], 1); states.masked_fill_(reset[s], s0)

    def one_step():
        lib.fill_mask(states, data, length, mask)
        apply_mask(logits, mask, V)
        lib.advance(tok)

    start(); eager_inputs(0); one_step()             # warm up outside capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    start()
    with torch.cuda.graph(g):
        one_step()
    ref = []
    start()
    for s in range(steps):
        eager_inputs(s)
        one_step()
        torch.cuda.synchronize()
        ref.append((mask.clone(), logits.clone(), states.clone(), length.clone(), data.clone()))
    assert traj.reset.any()                           # the run includes slot reuse
    start()
    for s in range(steps):
        eager_inputs(s)                               # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((mask, logits, states, length, data), ref[s]):
            assert torch.equal(got, want), f"replay {s} differs from the eager step"
    assert int(err.abs().sum()) == 0


def test_hip_graph_of_the_greedy_loop_replays_like_eager():
    """argmax -> advance+mask -> jump-forward -> mask, captured as one step and replayed: each
    replay (with fresh logits uploaded eagerly in between) must leave what eager calls leave."""
    torch, dev = _torch()
    from workloads import configs
    cfg = configs.get(2)
    v = cfg.vocab
    sch = G.schema_grammar(11, 6, 2, 4).text                  # forced key text gives jump-forward work
    lib = _lib([sch], v, stack_cap=256)
    B, V, W, cap, steps = 32, v.n_tokens, v.words, 256, 10
    s0 = lib.initial_state(0)
    data = torch.zeros((B, cap), dtype=torch.int32, device=dev)
    length = torch.ones(B, dtype=torch.int32, device=dev)
    states = torch.full((B,), s0, dtype=torch.int32, device=dev)
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states, data, length, err)
    mask = torch.zeros((B, W), dtype=torch.int32, device=dev)
    tok = torch.zeros(B, dtype=torch.int32, device=dev)
    jb = torch.zeros((B, 16), dtype=torch.uint8, device=dev)
    jn = torch.zeros(B, dtype=torch.int32, device=dev)
    rng = np.random.default_rng(8)
    all_logits = [torch.from_numpy(bf16_logits(rng, B, V).view(np.int16)).to(dev) for _ in range(steps)]
    logits = all_logits[0].clone()

    def start():
        data.zero_(); data[:, 0] = s0; length.fill_(1); states.fill_(s0)
        lib.fill_mask(states, data, length, mask)

    def one_step():
        lib.apply_mask_argmax(logits.view(torch.bfloat16), mask, tok)
        lib.advance_fill_mask(tok, mask)
        lib.jump_forward(jb, jn)
        lib.fill_mask(states, data, length, mask)

    start(); one_step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    start()
    with torch.cuda.graph(g):
        one_step()
    ref = []
    start()
    for s in range(steps):
        logits.copy_(all_logits[s])
        one_step()
        torch.cuda.synchronize()
        ref.append(tuple(x.clone() for x in (tok, mask, states, length, data, jn, err)))
    assert sum(int(r[5].sum()) for r in ref) > 0              # bytes were forced along the way
    start()
    for s in range(steps):
        logits.copy_(all_logits[s])                           # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((tok, mask, states, length, data, jn, err), ref[s]):
            assert torch.equal(got, want), f"replay {s} differs from the eager step"


@pytest.mark.parametrize("greedy", [False, True])
def test_hip_graph_of_the_one_kernel_step_replays_like_eager(greedy):
    """The one-kernel step (pre3_advance_fill_apply_mask; greedy: pre3_advance_fill_argmax with the token buffer
    updated in place) captured once and replayed: each replay, with fresh logits and -- for the masking form -- fresh
    tokens uploaded eagerly in between, must leave what the eager call leaves."""
    torch, dev = _torch()
    from workloads import configs
    cfg = configs.get(2)
    v = cfg.vocab
    lib = _lib(cfg.grammars, v, stack_cap=256)
    B, V, W, cap, steps = 32, v.n_tokens, v.words, 256, 8
    s0 = lib.initial_state(0)
    data = torch.zeros((B, cap), dtype=torch.int32, device=dev)
    length = torch.ones(B, dtype=torch.int32, device=dev)
    states = torch.full((B,), s0, dtype=torch.int32, device=dev)
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states, data, length, err)
    mask = torch.zeros((B, W), dtype=torch.int32, device=dev)
    tok = torch.zeros(B, dtype=torch.int32, device=dev)
    rng = np.random.default_rng(9)
    all_logits = [torch.from_numpy(bf16_logits(rng, B, V).view(np.int16)).to(dev) for _ in range(steps + 1)]
    logits = all_logits[0].clone()

    def start():
        data.zero_(); data[:, 0] = s0; length.fill_(1); states.fill_(s0)
        lib.fill_mask(states, data, length, mask)
        lib.apply_mask_argmax(all_logits[steps].view(torch.bfloat16), mask, tok)     # a first token that is allowed

    def one_step():
        if greedy:
            lib.advance_fill_argmax(tok, mask, logits, tok, restart_on_eos=True, one_kernel=True)
        else:
            lib.advance_fill_apply_mask(tok, mask, logits, restart_on_eos=True, one_kernel=True)

    def next_token():                                         # the masking form: the caller samples; here the arg max
        if not greedy:
            lib.apply_mask_argmax(logits.view(torch.bfloat16), mask, tok)

    assert lib.step_is_one_kernel(logits, one_kernel=True)
    start(); one_step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    start()
    with torch.cuda.graph(g):
        one_step()
    ref = []
    start()
    for s in range(steps):
        logits.copy_(all_logits[s])
        one_step()
        torch.cuda.synchronize()
        ref.append(tuple(x.clone() for x in (tok, mask, states, length, data, err, logits)))
        next_token()
    assert len({int(r[2][0]) for r in ref}) > 2              # the sequences did move
    start()
    for s in range(steps):
        logits.copy_(all_logits[s])                           # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((tok, mask, states, length, data, err, logits), ref[s]):
            assert torch.equal(got, want), f"replay {s} differs from the eager step"
        next_token()


def test_which_form_the_step_call_takes(deep_vocab):
    """pre3_step_is_one_kernel: the one kernel for batches between a quarter of the compute units and all of them
    (64..256 on the 256 units of an MI355X), at any batch size when asked for (beyond one sequence per unit in
    several launches), and never for logits whose rows are not 16-byte aligned or shorter than the vocabulary."""
    torch, dev = _torch()
    v = deep_vocab
    lib = _lib(G.JSON, v)
    units = torch.cuda.get_device_properties(0).multi_processor_count
    V = v.n_tokens
    stride = (V + 7) // 8 * 8
    z32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
    for B in (4, units // 4 - 1, units // 4, units, units + 1, 4 * units, 4 * units + 1):
        states = torch.full((B,), lib.initial_state(0), dtype=torch.int32, device=dev)
        data = torch.zeros((B, 32), dtype=torch.int32, device=dev)
        data[:, 0] = states
        lib.bind_state(states, data, torch.ones(B, dtype=torch.int32, device=dev), z32(B))
        flat = torch.zeros(B * stride + 16, dtype=torch.int16, device=dev)
        aligned = flat[: B * stride].view(B, stride)
        assert lib.step_is_one_kernel(aligned) == (units // 4 <= B <= units), B
        assert lib.step_kernel_launches(aligned, one_kernel=True) == (B + units - 1) // units, B
        assert not lib.step_is_one_kernel(flat[4: 4 + B * stride].view(B, stride), one_kernel=True)          # rows at 8 bytes
        if B > 1:
            assert not lib.step_is_one_kernel(torch.zeros((B, stride + 4), dtype=torch.int16, device=dev), one_kernel=True)
    torch.cuda.synchronize()


def _short_token_vocab(rng, V):
    """V - 1 tokens of one to four bytes over the arithmetic grammar's alphabet, then the end-of-sequence token."""
    alphabet = np.frombuffer(b"a+*()b- ", dtype=np.uint8)
    lens = rng.integers(1, 5, size=V - 1)
    flat = alphabet[rng.integers(0, len(alphabet), size=int(lens.sum()))].tobytes()
    offs = np.concatenate([[0], np.cumsum(lens)])
    return Vocab([flat[offs[i]: offs[i + 1]] for i in range(V - 1)] + [b""], V - 1)


def _allowed(row, V):
    return np.flatnonzero((row[np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1)


@pytest.mark.parametrize("V", [200_003, 207_360, 207_368])
def test_whole_step_as_one_call_on_a_vocabulary_of_two_hundred_thousand(V):
    """The one-kernel step keeps up to 27 groups of eight logits per lane (207,360 tokens) when it masks and
    20 (153,600) when it takes the arg max: a vocabulary of about 200,000 tokens takes the one kernel for the
    masking call and two launches for the greedy call, one of 207,368 takes two launches for both, and every
    form gives the oracle's stacks, mask rows, masked logits and picks."""
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + 93 + V)
    v = _short_token_vocab(rng, V)
    o = Oracle(G.ARITHMETIC)
    lib = _lib(G.ARITHMETIC, v, stack_cap=64)
    assert lib.token_edge_stats()["built"] > 0
    kinds = [b"", b"(a+", b"a*(a", b"((a)", b"a", b"(", b"a+", b"((a*a)+"]
    reps = 8                                                       # 64 rows: the mask + masking call takes the step kernel too
    s1, d1, l1 = _stacks(o, kinds, 64)
    states, data, length = np.tile(s1, reps), np.tile(d1, (reps, 1)), np.tile(l1, reps)
    B, W = len(states), v.words
    stride = (V + 7) // 8 * 8 + 8
    st, da, ln = torch.from_numpy(states).to(dev), torch.from_numpy(data).to(dev), torch.from_numpy(length).to(dev)
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(st, da, ln, err)
    lg = torch.zeros((B, stride), dtype=torch.int16, device=dev)
    assert lib.step_is_one_kernel(lg, one_kernel=True) == (V <= 207_360)

    def masked(logits, rows):
        expect = logits.copy()
        oracle_apply_mask(expect, rows, V)
        return expect

    # mask rows of the stacks as they are, applied in the same call
    want = np.tile(o.fill_mask(s1, d1, l1, v), (reps, 1))
    logits = bf16_logits(rng, B, V)
    lg[:, :V] = torch.from_numpy(logits.view(np.int16)).to(dev)
    m = torch.full((B, W), 0x55555555, dtype=torch.int32, device=dev)
    lib.fill_apply_mask(st, da, ln, m, lg.view(torch.bfloat16)[:, :V])
    assert (m.cpu().numpy().view(np.uint32) == want).all()
    assert (lg[:, :V].cpu().numpy().view(np.uint16) == masked(logits, want)).all()
    assert int(lg[:, V:].abs().sum().item()) == 0                  # nothing written past a row's end

    # three whole steps in one call each, then a greedy one
    for step in range(4):
        picks1 = np.array([_allowed(want[b], V)[(5 + 3 * step + b) % 11] for b in range(len(kinds))], dtype=np.int32)
        picks = np.tile(picks1, reps)
        e1 = o.advance_batch(s1, d1, l1, picks1, v)
        assert (e1 == 0).all()
        want = np.tile(o.fill_mask(s1, d1, l1, v), (reps, 1))
        logits = bf16_logits(rng, B, V)
        lg[:, :V] = torch.from_numpy(logits.view(np.int16)).to(dev)
        m.fill_(0x55555555)
        toks = torch.from_numpy(picks).to(dev)
        if step < 3:
            lib.advance_fill_apply_mask(toks, m, lg.view(torch.bfloat16)[:, :V], one_kernel=True)
            assert (lg[:, :V].cpu().numpy().view(np.uint16) == masked(logits, want)).all(), step
        else:
            out = torch.full((B,), -7, dtype=torch.int32, device=dev)
            lib.advance_fill_argmax(toks, m, lg.view(torch.bfloat16)[:, :V], out, one_kernel=True)
            assert (lg[:, :V].cpu().numpy().view(np.uint16) == logits).all()
            assert (out.cpu().numpy() == oracle_masked_argmax(logits, want, V)).all()
        assert (err.cpu().numpy() == 0).all() and (st.cpu().numpy() == np.tile(s1, reps)).all()
        assert (ln.cpu().numpy() == np.tile(l1, reps)).all()
        assert (m.cpu().numpy().view(np.uint32) == want).all(), step
        assert int(lg[:, V:].abs().sum().item()) == 0


def test_vocabulary_larger_than_the_lds_bitmap_takes_the_walk_path():
    """A mask row of more than 56 KiB does not fit the token-edge kernels' LDS bitmap: every call
    must then give the same results through the byte-by-byte kernel."""
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + 91)
    V = 14336 * 32 + 2000 + 5                                  # beyond the bitmap, ragged tail
    alphabet = np.frombuffer(b"a+*()b- ", dtype=np.uint8)
    lens = rng.integers(1, 5, size=V - 1)
    flat = alphabet[rng.integers(0, len(alphabet), size=int(lens.sum()))].tobytes()
    offs = np.concatenate([[0], np.cumsum(lens)])
    toks = [flat[offs[i]: offs[i + 1]] for i in range(V - 1)] + [b""]
    v = Vocab(toks, V - 1)
    o = Oracle(G.ARITHMETIC)
    lib = _lib(G.ARITHMETIC, v, stack_cap=64)
    assert lib.token_edge_stats()["built"] == 0               # no token-level edges for such a vocabulary
    prefixes = [b"", b"(a+", b"a*(a", b"((a)"]
    states, data, length = _stacks(o, prefixes, 64)
    B, W = len(prefixes), v.words
    want = o.fill_mask(states, data, length, v)
    assert (_gpu_mask(lib, states, data, length, W) == want).all()
    # fused mask + apply, then advance + next mask, all through the fallback
    logits = bf16_logits(rng, B, V)
    lg = torch.from_numpy(logits.view(np.int16)).to(dev)
    st, da, ln = torch.from_numpy(states).to(dev), torch.from_numpy(data).to(dev), torch.from_numpy(length).to(dev)
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    m = torch.zeros((B, W), dtype=torch.int32, device=dev)
    lib.fill_apply_mask(st, da, ln, m, lg.view(torch.bfloat16))
    expect = logits.copy()
    oracle_apply_mask(expect, want, V)
    assert (m.cpu().numpy().view(np.uint32) == want).all()
    assert (lg.cpu().numpy().view(np.uint16) == expect).all()
    lib.bind_state(st, da, ln, err)
    picks = np.array([int(np.flatnonzero(((want[b][np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1))[7])
                      for b in range(B)], dtype=np.int32)
    e_h = o.advance_batch(states, data, length, picks, v)
    lib.advance_fill_mask(torch.from_numpy(picks).to(dev), m)
    assert (err.cpu().numpy() == e_h).all() and (st.cpu().numpy() == states).all() and (ln.cpu().numpy() == length).all()
    assert (m.cpu().numpy().view(np.uint32) == o.fill_mask(states, data, length, v)).all()


def test_rebinding_other_batch_sizes_does_not_accumulate_device_memory():
    """A server that resizes its batch rebinds again and again: the per-batch workspaces are reused or
    replaced, never abandoned (free device memory stays level), and every binding advances correctly."""
    torch, dev = _torch()
    o = Oracle(G.JSON)
    v = bpe_like_vocab(3000, 16, BASE_SEED + 90)
    lib = _lib(G.JSON, v, stack_cap=64)
    s0 = lib.initial_state(0)
    tok = v.tokens.index(b"[")
    rc, want = o.advance([s0], b"[")
    assert rc == 0

    def bind_and_advance(B):
        data = torch.zeros((B, 64), dtype=torch.int32, device=dev)
        data[:, 0] = s0
        length = torch.ones(B, dtype=torch.int32, device=dev)
        states = torch.full((B,), s0, dtype=torch.int32, device=dev)
        err = torch.full((B,), -3, dtype=torch.int32, device=dev)
        lib.bind_state(states, data, length, err)
        lib.advance(torch.full((B,), tok, dtype=torch.int32, device=dev))
        out = torch.empty(B, dtype=torch.int32, device=dev)
        mask = torch.empty((B, v.words), dtype=torch.int32, device=dev)
        lib.fill_mask(states, data, length, mask)
        lib.apply_mask_argmax(torch.zeros((B, v.n_tokens), dtype=torch.bfloat16, device=dev), mask, out)
        torch.cuda.synchronize()
        assert int(err.abs().sum().item()) == 0 and int((length != len(want)).sum().item()) == 0
        assert (data[:, : len(want)].cpu().numpy() == np.array(want, dtype=np.int32)[None, :]).all()

    sizes = [8, 4096, 64, 20000, 1, 512]
    for B in sizes:                       # every size once: the workspaces reach their largest extent
        bind_and_advance(B)
    torch.cuda.empty_cache()
    free_before = torch.cuda.mem_get_info()[0]
    for _ in range(6):
        for B in sizes:
            bind_and_advance(B)
    torch.cuda.empty_cache()
    free_after = torch.cuda.mem_get_info()[0]
    assert free_before - free_after < (8 << 20), (free_before, free_after)
