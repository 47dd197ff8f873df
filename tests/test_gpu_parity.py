"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the five
seeded workload configurations.  Integer/bit work: everything must be bit-exact."""
import numpy as np
import pytest

from replay import replay, replay_advance_fill

pytestmark = pytest.mark.gpu


def test_cfg1_arithmetic_all_steps():
    r = replay(1)
    assert r["full_masks"] == 32


def test_cfg2_json_all_steps():
    r = replay(2)
    assert r["full_masks"] == 128


def test_cfg1_byte_by_byte_path():
    """Same workload with the token-level edges switched off: every pair is walked."""
    assert replay(1, token_edges=False)["full_masks"] == 32


def test_cfg2_byte_by_byte_path():
    assert replay(2, steps=24, token_edges=False)["full_masks"] == 24


def test_cfg2_one_reduction_step_at_a_time():
    """Merged reduction edges switched off: walks and advance follow single reduction steps."""
    assert replay(2, steps=24, token_edges=False, merged_reductions=False)["full_masks"] == 24
    assert replay(1, merged_reductions=False)["full_masks"] == 32


@pytest.mark.parametrize("depth", [1, 2, 4])
def test_cfg2_shallow_conditions_leave_tokens_to_the_walk(depth):
    """Conditions limited to a few stack entries: the tree leaves walk lists (and, at depth 1,
    whole rows) to the byte-by-byte walk inside the edge kernel."""
    assert replay(2, steps=16, max_condition_depth=depth)["full_masks"] == 16


@pytest.mark.parametrize("threshold", [64, 4008])
def test_cfg2_rows_assembled_from_id_lists(threshold):
    """A larger row threshold leaves token ids in per-node lists that the kernels OR into the row."""
    r = replay(2, steps=40, row_threshold=threshold)
    assert r["full_masks"] == 40
    assert replay_advance_fill(2, steps=40, row_threshold=threshold)["steps"] == 40


def test_cfg3_json_full_size():
    """B=256, V=128256, 256 steps: states/stacks and the whole bitmask (all B*W words) on every
    step, the masked logits (both entry points) on 6 steps spread over the run."""
    r = replay(3, apply_steps=[0, 1, 50, 100, 200, 255])
    assert r["full_masks"] == 256 and r["applied"] == 6


def test_cfg4_schema_full_size():
    """B=512, V=152064, 256 steps: states/stacks on every step, the whole bitmask on every fourth
    step (and the last), two full rows on every other step, the masked logits on 4 steps."""
    r = replay(4, full_mask_steps=list(range(0, 256, 4)) + [255], apply_steps=[0, 40, 128, 255])
    assert r["full_masks"] == 65 and r["applied"] == 4 and r["sampled_rows"] == 2 * (256 - 65)


def test_cfg5_mixed_grammars_deep_stacks():
    """B=256, V=128256, 512 steps, 8 grammars, seeded deep stacks: states/stacks and the whole
    bitmask on every step, the masked logits on 5 steps."""
    r = replay(5, apply_steps=[0, 1, 64, 256, 511])
    assert r["full_masks"] == 512 and r["applied"] == 5
    assert max(r["depth_hist"]) >= 60 and len(r["depth_hist"]) > 40


def test_cfg6_free_text_then_json_full_size():
    """The second workload: documents that open with unconstrained text (dense masks) and end in
    a JSON answer, B=256, V=128256."""
    r = replay(6, steps=160, apply_steps=[0, 1, 30, 80, 159])
    assert r["full_masks"] == 160 and r["applied"] == 5


def test_advance_fill_mask_all_configs():
    """pre3_advance_fill_mask (advance + next mask in one launch, slot reuse on EOS) on every
    configuration; config 2 also with shallow conditions (leftover walks inside the fused kernel)
    and without token-level edges (two-launch fallback)."""
    assert replay_advance_fill(1)["full_masks"] == 32
    assert replay_advance_fill(2, steps=64)["full_masks"] == 64
    assert replay_advance_fill(2, steps=12, max_condition_depth=2)["full_masks"] == 12
    # the stack operations of the token-level edges: off (every token walked), and for every token of 2+ bytes
    assert replay_advance_fill(2, steps=64, token_effects=False)["full_masks"] == 64
    assert replay_advance_fill(2, steps=64, effect_min_len=2)["full_masks"] == 64
    assert replay_advance_fill(3, steps=24, effect_min_len=12, full_mask_steps=[0, 23])["full_masks"] == 2
    assert replay_advance_fill(2, steps=12, token_edges=False)["full_masks"] == 12
    assert replay_advance_fill(3, steps=96)["full_masks"] == 96
    assert replay_advance_fill(4, steps=64, full_mask_steps=range(0, 64, 4))["full_masks"] == 16
    assert replay_advance_fill(5, steps=96)["full_masks"] == 96
    assert replay_advance_fill(6, steps=96, full_mask_steps=range(0, 96, 2))["full_masks"] == 48


def test_whole_step_as_one_call_all_configs():
    """pre3_advance_fill_apply_mask (advance, next mask and masked logits in one call) against the oracle's
    advance, fill and apply: states, stacks, err, the whole bitmask and every logit pattern, padding included.
    Config 1 has a ragged vocabulary (513 tokens, 17 mask words): with 7 elements of padding per row the one
    kernel runs with its partial last group and word-wise mask stores, without padding the rows are not
    16-byte aligned and the call takes its two-call form.  Config 2 also with leftover walks inside the kernel
    (shallow conditions), rows put together from id lists, every token walked, and without token-level edges
    (two-call form); configs 3-6 at full size, 7 with cycle-aware stacks.  All of these ask for the one-kernel
    form whatever the batch size; the last three leave the choice to the library."""
    assert replay_advance_fill(1, step_call_every=1, logits_pad=7)["step_calls"] == 32
    assert replay_advance_fill(1, step_call_every=1)["step_calls"] == 32
    assert replay_advance_fill(2, steps=64, step_call_every=1)["step_calls"] == 64
    assert replay_advance_fill(2, steps=64, step_call_every=2, logits_pad=24)["step_calls"] == 32
    assert replay_advance_fill(2, steps=12, step_call_every=1, max_condition_depth=2)["step_calls"] == 12
    assert replay_advance_fill(2, steps=40, step_call_every=1, row_threshold=64)["step_calls"] == 40
    assert replay_advance_fill(2, steps=40, step_call_every=1, token_effects=False)["step_calls"] == 40
    assert replay_advance_fill(2, steps=12, step_call_every=1, token_edges=False)["step_calls"] == 12
    assert replay_advance_fill(3, steps=64, step_call_every=4)["step_calls"] == 16
    assert replay_advance_fill(4, steps=32, step_call_every=8, full_mask_steps=[])["step_calls"] == 4
    assert replay_advance_fill(5, steps=64, step_call_every=8)["step_calls"] == 8
    assert replay_advance_fill(6, steps=48, step_call_every=8, full_mask_steps=[])["step_calls"] == 6
    assert replay_advance_fill(7, steps=64, step_call_every=4)["step_calls"] == 16
    # the form the library chooses by itself: one kernel at 256 sequences, the two calls at 4 and at 512
    assert replay_advance_fill(3, steps=16, step_call_every=4, one_kernel=False)["step_calls"] == 4
    assert replay_advance_fill(1, step_call_every=1, logits_pad=7, one_kernel=False)["step_calls"] == 32
    assert replay_advance_fill(4, steps=8, step_call_every=4, full_mask_steps=[], one_kernel=False)["step_calls"] == 2


def test_whole_step_on_batches_larger_than_the_chip():
    """A batch of more sequences than compute units goes through the one kernel in several launches of equal shares
    (333 sequences on 256 units: 167 + 166; 1,031: four launches of 207 and one of 203): every sequence
    must be advanced, masked and applied exactly once, whatever launch it falls in -- config 2 at 333 and 1,031
    sequences, config 7 (cycle-aware stacks) and config 3 at 300."""
    assert replay_advance_fill(2, steps=24, step_call_every=1, batch=333, logits_pad=8)["step_calls"] == 24
    assert replay_advance_fill(2, steps=8, step_call_every=1, batch=1031)["step_calls"] == 8
    assert replay_advance_fill(7, steps=16, step_call_every=2, batch=300, full_mask_steps=[])["step_calls"] == 8
    assert replay_advance_fill(3, steps=12, step_call_every=3, batch=300, full_mask_steps=[])["step_calls"] == 4


@pytest.mark.parametrize("fused", [False, True, "step", "step, 12 entries"])
def test_mixed_token_stream_valid_invalid_skipped_and_eos(fused):
    """Sequences of config 2 fed, per step and sequence, one of: an allowed token, an arbitrary
    token (mostly not allowed), EOS (allowed or not), or no token; finished sequences keep
    receiving tokens.  err, states, stacks and the next masks must follow the oracle exactly
    ("step": through the one kernel of pre3_advance_fill_apply_mask, whose masked logits are checked too)."""
    import torch
    from oracle import Oracle
    from paper_2506_03887_amd import Pre3
    from workloads import configs
    dev = torch.device("cuda:0")
    cfg = configs.get(2)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, 20            # a small capacity: overflows do happen
    if fused == "step, 12 entries":                              # below 16 entries the step kernel stages the stack
        fused, cap = "step", 12                                  # window with vector loads
    o = Oracle(cfg.grammars)
    s0 = o.initial_state(0)
    data = np.zeros((B, cap), dtype=np.int32)
    data[:, 0] = s0
    length = np.ones(B, dtype=np.int32)
    states = np.full(B, s0, dtype=np.int32)
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=v.max_len, stack_cap=cap)
    st, da, ln = (torch.from_numpy(x.copy()).to(dev) for x in (states, data, length))
    err = torch.zeros(B, dtype=torch.int32, device=dev)
    mask = torch.empty((B, W), dtype=torch.int32, device=dev)
    lib.bind_state(st, da, ln, err)
    lib.fill_mask(st, da, ln, mask)
    rng = np.random.default_rng(cfg.seed + 31)
    seen = {0: 0, 1: 0, 2: 0}
    opening = [t for t in range(V - 1) if v.tokens[t] and set(v.tokens[t]) <= set(b"[{")]
    for step in range(80):
        m_h = o.fill_mask(states, data, length, v)
        assert (mask.cpu().numpy().view(np.uint32) == m_h).all(), step
        toks = np.full(B, -1, dtype=np.int32)
        kind = rng.random(B)
        for b in range(B):
            if kind[b] < 0.55 and states[b] >= 0:
                allowed = np.flatnonzero((m_h[b][np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1)
                deepen = [t for t in opening if (m_h[b][t >> 5] >> (t & 31)) & 1]
                toks[b] = rng.choice(deepen) if deepen and rng.random() < 0.7 else rng.choice(allowed)
            elif kind[b] < 0.75:
                toks[b] = rng.integers(0, V)
            elif kind[b] < 0.85:
                toks[b] = v.eos_id
            elif kind[b] < 0.88:
                toks[b] = V + int(rng.integers(0, 5))            # an id beyond the vocabulary
        e_h = o.advance_batch(states, data, length, toks, v)
        for code in (0, 1, 2):
            seen[code] += int((e_h == code).sum())
        t_d = torch.from_numpy(toks).to(dev)
        if fused == "step":
            from oracle import apply_mask as oracle_apply_mask
            from workloads.vocab import bf16_logits
            logits = bf16_logits(rng, B, V)
            logits_d = torch.from_numpy(logits.view(np.int16)).to(dev)
            lib.advance_fill_apply_mask(t_d, mask, logits_d, one_kernel=True)
            oracle_apply_mask(logits, o.fill_mask(states, data, length, v), V)
            assert (logits_d.cpu().numpy().view(np.uint16) == logits).all(), step
        elif fused:
            lib.advance_fill_mask(t_d, mask)
        else:
            lib.advance(t_d)
            lib.fill_mask(st, da, ln, mask)
        assert (err.cpu().numpy() == e_h).all(), step
        assert (st.cpu().numpy() == states).all() and (ln.cpu().numpy() == length).all(), step
        live = np.arange(cap)[None, :] < length[:, None]
        assert (da.cpu().numpy()[live] == data[live]).all(), step
        # a few finished sequences start over so that the stream stays lively
        again = (states < 0) & (rng.random(B) < 0.3)
        if again.any():
            states[again], length[again] = s0, 1
            st[torch.from_numpy(again).to(dev)] = s0
            ln[torch.from_numpy(again).to(dev)] = 1
            lib.fill_mask(st, da, ln, mask)
    assert seen[0] > (1000 if cap >= 20 else 300) and seen[1] > 300 and seen[2] > 0, seen
