"""pre3_advance_static (the entry point that allocates nothing: the walks' spill area is an array
inside the library's device code) against pre3_advance, through the C ABI: same states, len, live
stack entries and err, bit for bit, on two calls in a row of which the second has a smaller batch;
deep tokens that really spill; cycle-aware stacks; the size limit."""
import numpy as np
import pytest

from oracle import Oracle
from workloads import configs, grammars as G, trajectory
from workloads.vocab import BASE_SEED, Vocab, bpe_like_vocab

pytestmark = pytest.mark.gpu


def _both(lib, tokens, states, data, length, label):
    """Runs pre3_advance (bound copies) and pre3_advance_static (other copies) on the same inputs
    and compares every output.  Returns the outputs as numpy arrays."""
    import torch
    dev = torch.device("cuda:0")
    B, cap = data.shape
    print(f"[no-alloc] {label}: batch {B} cap {cap}", flush=True)
    t_d = torch.from_numpy(tokens).to(dev)
    ref = [torch.from_numpy(x.copy()).to(dev) for x in (states, data, length)]
    e_ref = torch.full((B,), -9, dtype=torch.int32, device=dev)
    lib.bind_state(ref[0], ref[1], ref[2], e_ref)
    lib.advance(t_d)
    new = [torch.from_numpy(x.copy()).to(dev) for x in (states, data, length)]
    e_new = torch.full((B,), -9, dtype=torch.int32, device=dev)
    lib.advance_static(t_d, new[0], new[1], new[2], e_new)
    torch.cuda.synchronize()
    s_r, d_r, l_r = (x.cpu().numpy() for x in ref)
    s_n, d_n, l_n = (x.cpu().numpy() for x in new)
    assert (e_new.cpu().numpy() == e_ref.cpu().numpy()).all(), label
    assert (s_n == s_r).all() and (l_n == l_r).all(), label
    live = np.arange(cap)[None, :] < l_r[:, None]
    assert (d_n[live] == d_r[live]).all(), label
    return s_r, d_r, l_r, e_ref.cpu().numpy()


def _stacks(o, prefixes, cap):
    B = len(prefixes)
    data = np.zeros((B, cap), dtype=np.int32)
    length = np.ones(B, dtype=np.int32)
    for b, p in enumerate(prefixes):
        rc, st = (0, o.initial_stack(0)) if not p else o.advance(o.initial_stack(0), p)
        assert rc == 0, p
        data[b, : len(st)] = st
        length[b] = len(st)
    return data[np.arange(B), length - 1].copy(), data, length


def _deep_vocab():
    base = bpe_like_vocab(3000, 16, BASE_SEED + 77).tokens[:-1]
    extra = [b"[" * 32, b"[" * 17 + b"1", b"[[[[[[[[[[[[[[[[[[[[{\"a\":[[", b"{\"k\":" * 6, b"]" * 20, b"[1," * 10, b"]]]]]]]],"]
    toks = base + extra + [b""]
    return Vocab(toks, len(toks) - 1)


def test_two_calls_in_a_row_the_second_smaller_with_spilled_private_stacks():
    from paper_2506_03887_amd import Pre3
    o = Oracle(G.JSON)
    v = _deep_vocab()
    cap = 256
    lib = Pre3(G.JSON, v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    assert lib.walk_depth_bound > 16                      # walks deeper than the LDS part use the spill area
    prefixes = [b"", b"[", b"[[[[[[[[[", b'{"a":', b'{"a":[[[[[[[[[[[[[[[[[[[[', b'"abc', b"[1", b"[[[[[[[[[1" + b"]" * 3, b"12"]
    states, data, length = _stacks(o, prefixes, cap)
    idx = lambda t: v.tokens.index(t)
    toks = np.array([idx(b"[" * 32), idx(b"[" * 32), idx(b"]]]]]]]],"), idx(b"[" * 17 + b"1"), idx(b"]" * 20), -1,
                     idx(b"[1," * 10), idx(b"]]]]]]]],"), v.eos_id], dtype=np.int32)
    s1, d1, l1, e1 = _both(lib, toks, states, data, length, "first call, 9 sequences")
    # the oracle agrees with both (so the comparison above did not compare two wrong answers)
    s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
    err = o.advance_batch(s_h, d_h, l_h, toks, v)
    assert (e1 == err).all() and (s1 == s_h).all() and (l1 == l_h).all() and l_h.max() > 60
    # second call: fewer sequences (the first four, as the first call left them), other tokens
    toks2 = np.array([idx(b"[[[[[[[[[[[[[[[[[[[[{\"a\":[["), idx(b"]" * 20), idx(b"[" * 32), idx(b"[1," * 10)], dtype=np.int32)
    s2, d2, l2, e2 = _both(lib, toks2, s1[:4].copy(), d1[:4].copy(), l1[:4].copy(), "second call, 4 sequences")
    s_h, d_h, l_h = s1[:4].copy(), d1[:4].copy(), l1[:4].copy()
    err = o.advance_batch(s_h, d_h, l_h, toks2, v)
    assert (e2 == err).all() and (s2 == s_h).all() and (l2 == l_h).all()
    assert set(e1.tolist()) | set(e2.tolist()) >= {0, 1}


def test_trajectory_steps_then_a_smaller_batch():
    """Steps of the JSON workload (64 sequences, then 17 of them), nothing bound for the static call."""
    from paper_2506_03887_amd import Pre3
    cfg = configs.get(2)
    v = cfg.vocab
    o = Oracle(cfg.grammars)
    traj = trajectory.generate(o, v, cfg.batch, 12, cfg.cap, cfg.seed, None, cfg.nest_cap)
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cfg.cap)
    data, length = traj.init_data.copy(), traj.init_len.copy()
    states = data[np.arange(cfg.batch), length - 1].copy()
    for s in range(8):
        rs = np.flatnonzero(traj.reset[s])
        data[rs, 0] = o.initial_state(0)
        length[rs] = 1
        states[rs] = data[rs, 0]
        states, data, length, err = _both(lib, traj.tokens[s], states, data, length, f"step {s}")
        assert not err.any()
    sub = np.arange(0, 64, 4)[:16].tolist() + [63]
    for s in range(8, 12):
        tok = traj.tokens[s][sub].copy()
        tok[::5] = v.n_tokens - 2                          # some tokens that are not allowed
        st, da, ln = states[sub].copy(), data[sub].copy(), length[sub].copy()
        fin = st < 0
        st[fin], ln[fin] = da[fin, 0], 1
        _both(lib, tok, st, da, ln, f"step {s}, 17 sequences")


def test_cycle_aware_stacks():
    from paper_2506_03887_amd import Pre3
    v = bpe_like_vocab(4000, 16, BASE_SEED + 78)
    o = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    for cap in (96, 4000):                                # compaction inside the advance kernel / by a kernel of its own
        lib = Pre3([G.JSON_RIGHT_RECURSIVE], v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap,
                   compact_cycles=True)
        traj = trajectory.generate(o, v, 24, 10, cap, BASE_SEED + 5, None, 6, len_cap=min(cap, 90))
        data, length = traj.init_data.copy(), traj.init_len.copy()
        states = data[np.arange(24), length - 1].copy()
        for s in range(10):
            rs = np.flatnonzero(traj.reset[s])
            data[rs, 0] = o.initial_state(0)
            length[rs] = 1
            states[rs] = data[rs, 0]
            n = 24 if s < 6 else 7
            st, da, ln, err = _both(lib, traj.tokens[s][:n].copy(), states[:n].copy(), data[:n].copy(), length[:n].copy(),
                                    f"cap {cap} step {s}")
            s_h, d_h, l_h = states.copy(), data.copy(), length.copy()
            e_h = o.advance_batch(s_h, d_h, l_h, traj.tokens[s], v)
            assert not e_h.any() and (st == s_h[:n]).all() and (ln == l_h[:n]).all()
            states, data, length = s_h, d_h, l_h


def test_sizes_beyond_the_static_scratch_are_refused():
    import torch
    from paper_2506_03887_amd import Pre3, binding
    dev = torch.device("cuda:0")
    v = _deep_vocab()
    lib = Pre3(G.JSON, v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=8)
    deep = lib.walk_depth_bound - 16
    assert deep > 0
    B = (1 << 20) // deep + 1                              # one sequence too many
    s0 = lib.initial_state(0)
    data = torch.zeros((B, 8), dtype=torch.int32, device=dev)
    data[:, 0] = s0
    length = torch.ones(B, dtype=torch.int32, device=dev)
    states = torch.full((B,), s0, dtype=torch.int32, device=dev)
    err = torch.full((B,), -9, dtype=torch.int32, device=dev)
    tokens = torch.full((B,), v.tokens.index(b"["), dtype=torch.int32, device=dev)
    with pytest.raises(binding.Pre3Error) as e:
        lib.advance_static(tokens, states, data, length, err)
    assert e.value.status == binding.E_LIMIT and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert int((err != -9).sum().item()) == 0 and int((length != 1).sum().item()) == 0      # nothing ran
    B -= 1                                                 # the largest batch that fits
    lib.advance_static(tokens[:B], states[:B], data[:B], length[:B], err[:B])
    torch.cuda.synchronize()
    rc, want = Oracle(G.JSON).advance([s0], b"[")
    assert rc == 0 and len(want) <= 8
    assert int(err[:B].abs().sum().item()) == 0 and int((length[:B] != len(want)).sum().item()) == 0
    assert (data[:B, : len(want)].cpu().numpy() == np.array(want, dtype=np.int32)[None, :]).all()
    with pytest.raises(binding.Pre3Error):
        lib.advance_static(tokens[:4], states[:4], data.new_zeros((4, 16)), length[:4], err[:4])   # cap > stack_cap
