"""pre3_apply_mask_argmax and pre3_apply_mask_topk through the C ABI against the CPU oracle: value and layout cases of the
greedy choice itself, then a closed decode loop (mask -> choice -> advance) in which the GPU
and the oracle each pick their own tokens from the same logits and must stay in lockstep."""
import numpy as np
import pytest

from oracle import Oracle, masked_argmax as oracle_masked_argmax, masked_topk as oracle_masked_topk
from workloads import configs
from workloads import grammars as G
from workloads.vocab import BASE_SEED, Vocab, bf16_logits

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch, torch.device("cuda:0")


def _bound_lib(vocab, batch, cap=8):
    """A handle over the expression grammar whose vocabulary has the wanted size; the bound
    sequences are only there to give the call its batch."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    lib = Pre3(G.ARITHMETIC, vocab.bytes, vocab.offsets, vocab.eos_id, max_token_len=max(1, vocab.max_len),
               stack_cap=cap)
    s0 = lib.initial_state(0)
    keep = (torch.full((batch,), s0, dtype=torch.int32, device=dev),
            torch.full((batch, cap), s0, dtype=torch.int32, device=dev),
            torch.ones(batch, dtype=torch.int32, device=dev), torch.zeros(batch, dtype=torch.int32, device=dev))
    lib.bind_state(*keep)
    return lib


def _special_logits(rng, B, V):
    logits = bf16_logits(rng, B, V)
    coarse = (np.round(rng.normal(size=(B, V)) * 2).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    logits[1::4] = coarse[1::4]                               # rows with many equal maxima
    logits[2::4, ::5] = 0x7FC0                                # NaNs of both signs
    logits[2::4, 2::7] = 0xFFC3
    logits[3::4, ::3] = 0xFF80                                # -inf entries
    logits[0, : min(V, 6)] = [0x7F80, 0x8000, 0x0000, 0x7F80, 0xFF80, 0x7FC0][: min(V, 6)]
    return logits


def _special_masks(rng, B, V):
    W = (V + 31) // 32
    mask = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    sparse = rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    for _ in range(4):
        sparse &= rng.integers(0, 2 ** 32, size=(B, W), dtype=np.uint64).astype(np.uint32)
    mask[1::3] = sparse[1::3]                                 # about 3 % of the tokens allowed
    if B > 4:
        mask[4] = 0                                           # nothing allowed
    if B > 5:
        mask[5] = 0
        mask[5, W - 1] = 1 << ((V - 1) & 31)                  # only the last token
    if B > 6:
        mask[6] = 0xFFFFFFFF
    if V % 32:
        mask[:, W - 1] &= np.uint32((1 << (V % 32)) - 1)      # padding bits are zero, as fill_mask leaves them
    return mask


@pytest.mark.parametrize("V,B,stride_pad,offset", [(513, 4, 0, 0), (513, 9, 7, 0), (1003, 16, 5, 0), (1003, 16, 13, 3),
                                                   (32000, 64, 0, 0), (32000, 7, 8, 0), (128256, 256, 0, 0),
                                                   (128256, 3, 0, 8), (40, 300, 0, 0)])
def test_masked_argmax_values_and_layouts(V, B, stride_pad, offset):
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + V + B)
    toks = [bytes([97 + i % 5]) for i in range(V - 1)] + [b""]
    lib = _bound_lib(Vocab(toks, V - 1), B)
    logits = _special_logits(rng, B, V)
    mask = _special_masks(rng, B, V)
    if B > 7:                                                 # every allowed logit is -inf or NaN
        mask[7] = _special_masks(rng, 1, V)[0]                # a dense row
        allowed = ((mask[7][np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1).astype(bool)
        logits[7, allowed] = 0xFF80
        logits[7, np.flatnonzero(allowed)[:3]] = 0x7FC0
    if B > 8:                                                 # the largest value is zero, of both signs, -0 first
        logits[8] |= 0x8000
        logits[8, 5::11] = 0x8000
        logits[8, 9::13] = 0x0000
        mask[8] = _special_masks(rng, 1, V)[0]
    if B > 12:                                                # the same with few tokens allowed, and only -0
        logits[12] |= 0x8000
        logits[12, 3::7] = 0x8000
        mask[12, 1:] &= mask[11, 1:]
    want = oracle_masked_argmax(logits, mask, V)
    stride = V + stride_pad
    flat = torch.full((B * stride + offset + 8,), 0x1234, dtype=torch.int16, device=dev)
    view = flat[offset: offset + B * stride].view(B, stride)[:, :V]
    view.copy_(torch.from_numpy(logits.view(np.int16)).to(dev))
    before = flat.clone()
    out = torch.full((B,), -7, dtype=torch.int32, device=dev)
    m_d = torch.from_numpy(mask.view(np.int32)).to(dev)
    for _ in range(2):                                        # the second call finds the workspace clean
        out.fill_(-7)
        lib.apply_mask_argmax(view.view(torch.bfloat16), m_d, out)
        assert out.cpu().numpy().tolist() == want.tolist()
    assert torch.equal(flat, before), "the logits are read-only for this call"
    if B > 7:
        assert want[4] == -1 and want[5] == V - 1 and want[7] >= 0


@pytest.mark.parametrize("V,B,stride_pad,offset,ks", [
    (513, 4, 0, 0, (1, 8, 64)), (513, 9, 7, 0, (5,)), (1003, 16, 13, 3, (3, 64)), (32000, 64, 0, 0, (1, 40)),
    (16384, 5, 0, 0, (64,)), (16385, 5, 0, 0, (64,)), (128256, 256, 0, 0, (50,)), (128256, 3, 0, 8, (64,)), (40, 300, 0, 0, (4, 64))])
def test_masked_topk_values_and_layouts(V, B, stride_pad, offset, ks):
    """Same special rows as the arg max test (equal maxima, NaNs, infinities, zeros of both signs, empty
    and single-token masks); ids and bf16 patterns must equal the oracle's sorted list entry by entry."""
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + 3 * V + B)
    toks = [bytes([97 + i % 5]) for i in range(V - 1)] + [b""]
    lib = _bound_lib(Vocab(toks, V - 1), B)
    logits = _special_logits(rng, B, V)
    if B > 3:
        logits[3, ::2] = 0x0000                               # zeros of both signs tie, ids decide
        logits[3, 1::2] = 0x8000
    mask = _special_masks(rng, B, V)
    if B > 8:                                                 # fewer allowed tokens than k in one row
        mask[8] = 0
        mask[8, 0] = 0b1011
    stride = V + stride_pad
    flat = torch.full((B * stride + offset + 8,), 0x1234, dtype=torch.int16, device=dev)
    view = flat[offset: offset + B * stride].view(B, stride)[:, :V]
    view.copy_(torch.from_numpy(logits.view(np.int16)).to(dev))
    before = flat.clone()
    m_d = torch.from_numpy(mask.view(np.int32)).to(dev)
    for k in ks:
        want_ids, want_vals = oracle_masked_topk(logits, mask, V, k)
        ids = torch.full((B, k), -7, dtype=torch.int32, device=dev)
        vals = torch.full((B, k), 0x1111, dtype=torch.int16, device=dev)
        for _ in range(2):                                    # the second call reuses the workspace
            ids.fill_(-7)
            lib.apply_mask_topk(view.view(torch.bfloat16), m_d, ids, vals)
            got_ids, got_vals = ids.cpu().numpy(), vals.cpu().numpy().view(np.uint16)
            bad = np.argwhere(got_ids != want_ids)
            assert len(bad) == 0, (k, bad[:4].tolist(), got_ids[bad[0][0]][:8].tolist(), want_ids[bad[0][0]][:8].tolist())
            assert (got_vals == want_vals).all(), k
        ids.fill_(-7)
        lib.apply_mask_topk(view.view(torch.bfloat16), m_d, ids)          # without the values
        assert (ids.cpu().numpy() == want_ids).all()
        first = torch.empty(B, dtype=torch.int32, device=dev)
        lib.apply_mask_argmax(view.view(torch.bfloat16), m_d, first)
        assert torch.equal(first, ids[:, 0])
    assert torch.equal(flat, before), "the logits are read-only for this call"


def _bf16(x):
    return (np.asarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


@pytest.mark.parametrize("V,B,stride_pad,ks", [(70001, 300, 7, (50, 64)), (70001, 300, 0, (7,)), (128256, 520, 0, (50,)),
                                               (128256, 200, 0, (50, 3))])
def test_masked_topk_over_segments_of_several_chunks(V, B, stride_pad, ks):
    """Batches large enough that a block takes several chunks of 16,384 tokens in a row (a whole row from
    one row per compute unit on; at B = 200 two chunks, and a second kernel merges the segments): rows of equal
    logits (every chunk overflows the candidate list, ties decided by id), logits rising or falling with
    the id (the list is cut to its k best between chunks), masks that leave the first chunks empty or
    nearly empty, a single chunk with thousands of ties under a few larger values, NaN rows."""
    torch, dev = _torch()
    rng = np.random.default_rng(BASE_SEED + 5 * V + B)
    toks = [bytes([97 + i % 5]) for i in range(V - 1)] + [b""]
    lib = _bound_lib(Vocab(toks, V - 1), B)
    logits = _special_logits(rng, B, V)
    mask = _special_masks(rng, B, V)
    W = mask.shape[1]
    full = np.full(W, 0xFFFFFFFF, dtype=np.uint32)
    if V % 32:
        full[W - 1] = np.uint32((1 << (V % 32)) - 1)
    base = 8
    logits[base + 0] = 0x3F80; mask[base + 0] = full                        # all 1.0, all allowed
    logits[base + 1] = 0xC000                                               # all -2.0, sparse mask
    logits[base + 2] = _bf16(np.linspace(-3, 3, V)); mask[base + 2] = full  # rising with the id
    logits[base + 3] = _bf16(np.linspace(3, -3, V)); mask[base + 3] = full  # falling
    mask[base + 4] = 0; mask[base + 4, (3 * 16384) // 32 + 7:] = full[(3 * 16384) // 32 + 7:]   # the first chunks are empty
    mask[base + 5] = 0; mask[base + 5, 3] = 0x0FFFFFFF; mask[base + 5, 1024: 1536] = 0xFFFFFFFF  # 28 tokens, then a whole chunk
    logits[base + 6] = 0x7FC0; logits[base + 6, ::4099] = _bf16(rng.normal(size=len(range(0, V, 4099)))); mask[base + 6] = full
    logits[base + 7] = _bf16(rng.normal(size=V) - 8); logits[base + 7, 16384 + 100: 16384 + 3300] = 0x4000   # 3,200 ties at 2.0 in one chunk
    logits[base + 7, [5, 20000, 40000, 69000]] = 0x4040; mask[base + 7] = full
    logits[base + 8] = 0x8000; logits[base + 8, ::2] = 0x0000; mask[base + 8] = full               # zeros of both signs
    # 1,280 allowed tokens held by 40 threads of one chunk (fewer holders than k: every one is listed),
    # once followed by a full chunk, once as the last of its segment
    few = np.zeros(V, dtype=bool)
    for g in range(4):
        for t in range(40):
            few[(t + g * 512) * 8: (t + g * 512) * 8 + 8] = True
    for row, chunk, more in ((base + 9, 1, True), (base + 10, 3, False)):
        allowed = np.zeros(V, dtype=bool)
        allowed[chunk * 16384: chunk * 16384 + 16384] = few[: min(16384, V - chunk * 16384)]
        if more:
            allowed[3 * 16384: 4 * 16384] = True
        bits = np.zeros(W * 32, dtype=np.uint8)
        bits[:V] = allowed
        mask[row] = np.packbits(bits.reshape(W, 32), axis=1, bitorder="little").view(np.uint32)[:, 0]
    # a thousand equal logits spread over all chunks and nothing else allowed; the same under a few larger ones
    for row, extra in ((base + 11, False), (base + 12, True)):
        bits = np.zeros(W * 32, dtype=np.uint8)
        bits[np.arange(0, V, 70)] = 1
        logits[row] = 0x3FC0
        if extra:
            bits[[3, 33333, V - 2]] = 1
            logits[row, [3, 33333, V - 2]] = 0x4100
        mask[row] = np.packbits(bits.reshape(W, 32), axis=1, bitorder="little").view(np.uint32)[:, 0]
    stride = V + stride_pad
    flat = torch.full((B * stride + 8,), 0x1234, dtype=torch.int16, device=dev)
    view = flat[: B * stride].view(B, stride)[:, :V]
    view.copy_(torch.from_numpy(logits.view(np.int16)).to(dev))
    m_d = torch.from_numpy(mask.view(np.int32)).to(dev)
    for k in ks:
        want_ids, want_vals = oracle_masked_topk(logits, mask, V, k)
        ids = torch.full((B, k), -7, dtype=torch.int32, device=dev)
        vals = torch.full((B, k), 0x1111, dtype=torch.int16, device=dev)
        lib.apply_mask_topk(view.view(torch.bfloat16), m_d, ids, vals)
        got_ids, got_vals = ids.cpu().numpy(), vals.cpu().numpy().view(np.uint16)
        bad = np.argwhere(got_ids != want_ids)
        assert len(bad) == 0, (k, bad[:4].tolist(), got_ids[bad[0][0]][:8].tolist(), want_ids[bad[0][0]][:8].tolist())
        assert (got_vals == want_vals).all(), k
        assert want_ids[base + 0, :3].tolist() == [0, 1, 2] and want_ids[base + 4, 0] >= 3 * 16384 + 7 * 32


def test_masked_topk_argument_errors():
    from paper_2506_03887_amd.binding import Pre3Error
    torch, dev = _torch()
    V, B = 100, 2
    toks = [bytes([97 + i % 5]) for i in range(V - 1)] + [b""]
    lib = _bound_lib(Vocab(toks, V - 1), B)
    logits = torch.zeros((B, V), dtype=torch.bfloat16, device=dev)
    mask = torch.zeros((B, (V + 31) // 32), dtype=torch.int32, device=dev)
    for k in (0, 65):
        with pytest.raises(Pre3Error):
            lib.apply_mask_topk(logits, mask, torch.zeros((B, k), dtype=torch.int32, device=dev))
    with pytest.raises(Pre3Error):
        lib.apply_mask_topk(torch.zeros((B, 50), dtype=torch.bfloat16, device=dev), mask,
                            torch.zeros((B, 4), dtype=torch.int32, device=dev))     # rows shorter than the vocabulary


@pytest.mark.parametrize("cfg_idx,steps,fused_advance", [(1, 32, False), (2, 48, False), (2, 48, True), (3, 12, True),
                                                         (2, 400, True), (6, 10, True), (7, 10, True)])
def test_greedy_decode_in_lockstep_with_the_oracle(cfg_idx, steps, fused_advance):
    """Both sides decode greedily from the same seeded logits; tokens, states, stacks, err and
    masks must agree at every step (a sequence that ends restarts, as in the benchmark)."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    cfg = configs.get(cfg_idx)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    o = Oracle(cfg.grammars, compact_cycles=cfg.compact)
    gi, _ = configs.sequence_setup(cfg)
    s0 = np.array([o.initial_state(int(g)) for g in gi], dtype=np.int32)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = s0.copy()
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap,
               compact_cycles=cfg.compact)
    data_d, len_d = torch.from_numpy(data_h.copy()).to(dev), torch.from_numpy(len_h.copy()).to(dev)
    states_d, err_d = torch.from_numpy(states_h.copy()).to(dev), torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    tok_d = torch.empty(B, dtype=torch.int32, device=dev)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    rng = np.random.default_rng(cfg.seed + 5)
    for s in range(steps):
        logits = bf16_logits(rng, B, V)
        mask_h = o.fill_mask(states_h, data_h, len_h, v)
        assert (mask_d.cpu().numpy().view(np.uint32) == mask_h).all(), f"mask differs at step {s}"
        want_tok = oracle_masked_argmax(logits, mask_h, V)
        lib.apply_mask_argmax(torch.from_numpy(logits.view(np.int16)).to(dev).view(torch.bfloat16), mask_d, tok_d)
        assert tok_d.cpu().numpy().tolist() == want_tok.tolist(), f"greedy tokens differ at step {s}"
        assert (want_tok >= 0).all()
        err_h = o.advance_batch(states_h, data_h, len_h, want_tok, v)
        fin = states_h < 0                                    # slot reuse
        states_h[fin], len_h[fin] = s0[fin], 1
        if fused_advance:
            lib.advance_fill_mask(tok_d, mask_d, restart_on_eos=True)
        else:
            lib.advance(tok_d)
            done = states_d < 0
            states_d[done] = torch.from_numpy(s0).to(dev)[done]
            len_d[done] = 1
            lib.fill_mask(states_d, data_d, len_d, mask_d)
        assert (err_d.cpu().numpy() == err_h).all()
        assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all()
        live = np.arange(cap)[None, :] < len_h[:, None]
        assert (data_d.cpu().numpy()[live] == data_h[live]).all()


def _special_rows_under_a_mask(rng, B, V, mask_h):
    """Seeded logits whose first rows hold the cases the order keys cannot decide by themselves or must not get
    wrong: zeros of both signs only, NaN patterns only, -inf only, positive NaN patterns around one finite
    value, +inf twice, a negative NaN below everything, and -0 before +0 among the allowed tokens."""
    logits = bf16_logits(rng, B, V)
    allowed = [np.flatnonzero((mask_h[b][np.arange(V) >> 5] >> (np.arange(V) & 31).astype(np.uint32)) & 1) for b in range(B)]
    if B >= 8:
        logits[0] = np.where(rng.random(V) < 0.5, 0x8000, 0x0000)            # -0 / +0 everywhere: the first allowed id wins
        logits[1] = np.where(rng.random(V) < 0.5, 0x7FC1, 0xFFC0)            # NaN everywhere: -1
        logits[2] = 0xFF80                                                   # -inf everywhere: the first allowed id
        logits[3] = 0x7FC1                                                   # positive NaN patterns ...
        if len(allowed[3]) > 2:
            logits[3, allowed[3][len(allowed[3]) // 2]] = 0xC000             # ... and one finite (negative) value
        if len(allowed[4]) > 3:
            logits[4, allowed[4][-1]] = logits[4, allowed[4][1]] = 0x7F80    # +inf twice: the smaller id
        logits[5] = 0xFFC1                                                   # negative NaN patterns and one -inf
        if len(allowed[5]) > 1:
            logits[5, allowed[5][-1]] = 0xFF80
        logits[6] = 0xBF80                                                   # -1 everywhere, then -0 before +0
        if len(allowed[6]) > 2:
            logits[6, allowed[6][0]], logits[6, allowed[6][-1]] = 0x8000, 0x0000
    return logits


@pytest.mark.parametrize("cfg_idx,steps,pad,one_kernel,batch", [
    (1, 32, 7, True, None), (1, 32, 0, True, None), (2, 120, 0, True, None), (2, 40, 16, True, None), (3, 12, 0, False, None),
    (5, 8, 0, True, None), (6, 8, 0, True, None), (7, 10, 0, True, None), (4, 4, 0, True, None), (4, 3, 0, False, None),
    (2, 30, 0, True, 333), (7, 6, 0, True, 300)])
def test_greedy_decode_through_the_one_call_step_in_lockstep_with_the_oracle(cfg_idx, steps, pad, one_kernel, batch):
    """pre3_advance_fill_argmax (advance, next mask and next greedy token in one call, the token buffer updated in
    place) against the oracle's advance, fill and arg max: tokens, states, stacks, err and the whole mask at every
    step, the logits untouched.  The first rows of every step's logits hold the value cases of _special_rows_under_a_mask.
    Config 1 has a ragged vocabulary (partial last group; without padding its rows are misaligned and the call
    takes its two-call form); config 4 at 512 sequences runs the one kernel, in two launches, only because it is asked
    for; config 7 has cycle-aware stacks; 333 and 300 sequences go as launches of 167 + 166 and 150 + 150."""
    import dataclasses
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    cfg = configs.get(cfg_idx)
    if batch is not None:
        cfg = dataclasses.replace(cfg, batch=batch)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    o = Oracle(cfg.grammars, compact_cycles=cfg.compact)
    gi, _ = configs.sequence_setup(cfg)
    s0 = np.array([o.initial_state(int(g)) for g in gi], dtype=np.int32)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = s0.copy()
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap,
               compact_cycles=cfg.compact)
    data_d, len_d = torch.from_numpy(data_h.copy()).to(dev), torch.from_numpy(len_h.copy()).to(dev)
    states_d, err_d = torch.from_numpy(states_h.copy()).to(dev), torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    tok_d = torch.empty(B, dtype=torch.int32, device=dev)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    rng = np.random.default_rng(cfg.seed + 6)
    mask_h = o.fill_mask(states_h, data_h, len_h, v)
    logits = _special_rows_under_a_mask(rng, B, V, mask_h)
    want_tok = oracle_masked_argmax(logits, mask_h, V)
    lib.apply_mask_argmax(torch.from_numpy(logits.view(np.int16)).to(dev).view(torch.bfloat16), mask_d, tok_d)
    assert tok_d.cpu().numpy().tolist() == want_tok.tolist()
    n_none = 0
    for s in range(steps):
        # rows with no choice (all NaN) carry -1: no token, the sequence stays where it is
        n_none += int((want_tok < 0).sum())
        err_h = o.advance_batch(states_h, data_h, len_h, want_tok, v)
        fin = states_h < 0                                    # slot reuse
        states_h[fin], len_h[fin] = s0[fin], 1
        mask_h = o.fill_mask(states_h, data_h, len_h, v)
        logits = _special_rows_under_a_mask(rng, B, V, mask_h)
        host = np.full((B, V + pad), 0x1234, dtype=np.uint16)
        host[:, :V] = logits
        logits_d = torch.from_numpy(host.view(np.int16)).to(dev)
        want_tok = oracle_masked_argmax(logits, mask_h, V)
        mask_d.fill_(0x5A5A5A5A)
        lib.advance_fill_argmax(tok_d, mask_d, logits_d, tok_d, restart_on_eos=True, one_kernel=one_kernel)
        assert (err_d.cpu().numpy() == err_h).all() and not err_h.any(), f"err differs at step {s}"
        assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), f"states differ at step {s}"
        live = np.arange(cap)[None, :] < len_h[:, None]
        assert (data_d.cpu().numpy()[live] == data_h[live]).all(), f"stacks differ at step {s}"
        assert (mask_d.cpu().numpy().view(np.uint32) == mask_h).all(), f"mask differs at step {s}"
        assert tok_d.cpu().numpy().tolist() == want_tok.tolist(), f"greedy tokens differ at step {s}"
        assert (logits_d.cpu().numpy().view(np.uint16) == host).all(), f"logits were written at step {s}"
    assert lib.fault_count() == 0
    if B >= 8:
        assert n_none >= steps                                # the all-NaN row had no choice at every step


@pytest.mark.parametrize("cfg_idx,steps,k", [(2, 60, 8), (3, 8, 50), (4, 6, 8)])
def test_topk_sampling_decode_in_lockstep_with_the_oracle(cfg_idx, steps, k):
    """A top-k sampler on real grammar masks (free-form JSON and a schema whose keys are forced; many
    groups of 8 tokens fully masked): the k candidates and their logits must equal the oracle's at every step;
    both sides then take the same seeded choice among them and advance."""
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    cfg = configs.get(cfg_idx)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    o = Oracle(cfg.grammars)
    s0 = o.initial_state(0)
    data_h = np.zeros((B, cap), dtype=np.int32)
    data_h[:, 0] = s0
    len_h = np.ones(B, dtype=np.int32)
    states_h = np.full(B, s0, dtype=np.int32)
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap)
    data_d, len_d = torch.from_numpy(data_h.copy()).to(dev), torch.from_numpy(len_h.copy()).to(dev)
    states_d, err_d = torch.from_numpy(states_h.copy()).to(dev), torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    ids_d = torch.empty((B, k), dtype=torch.int32, device=dev)
    vals_d = torch.empty((B, k), dtype=torch.int16, device=dev)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    rng = np.random.default_rng(cfg.seed + 11)
    for s in range(steps):
        logits = bf16_logits(rng, B, V)
        mask_h = o.fill_mask(states_h, data_h, len_h, v)
        want_ids, want_vals = oracle_masked_topk(logits, mask_h, V, k)
        lib.apply_mask_topk(torch.from_numpy(logits.view(np.int16)).to(dev).view(torch.bfloat16), mask_d, ids_d, vals_d)
        assert (ids_d.cpu().numpy() == want_ids).all(), f"candidates differ at step {s}"
        assert (vals_d.cpu().numpy().view(np.uint16) == want_vals).all(), f"candidate logits differ at step {s}"
        n_valid = (want_ids >= 0).sum(axis=1)
        assert (n_valid >= 1).all()
        pick = (rng.integers(0, 1 << 30, size=B) % n_valid).astype(np.int64)
        tokens = want_ids[np.arange(B), pick].astype(np.int32)
        assert not o.advance_batch(states_h, data_h, len_h, tokens, v).any()
        fin = states_h < 0                                    # slot reuse
        states_h[fin], len_h[fin] = s0, 1
        lib.advance_fill_mask(torch.from_numpy(tokens).to(dev), mask_d, restart_on_eos=True)
        assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all()


def test_greedy_decode_emits_documents_the_json_module_accepts():
    """No oracle in the loop: the device decodes greedily from seeded logits (EOS favoured a little
    so that documents end), and every finished sequence's text must parse with Python's json."""
    import json
    from paper_2506_03887_amd import Pre3
    torch, dev = _torch()
    cfg = configs.get(2)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap)
    s0 = lib.initial_state(0)
    data_d = torch.zeros((B, cap), dtype=torch.int32, device=dev)
    data_d[:, 0] = s0
    len_d = torch.ones(B, dtype=torch.int32, device=dev)
    states_d = torch.full((B,), s0, dtype=torch.int32, device=dev)
    err_d = torch.zeros(B, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    tok_d = torch.empty(B, dtype=torch.int32, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed + 9)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    texts = [bytearray() for _ in range(B)]
    finished = [None] * B
    for _ in range(160):
        logits = torch.randn((B, V), generator=gen, device=dev, dtype=torch.float32)
        logits[:, v.eos_id] += 2.5
        lib.apply_mask_argmax(logits.to(torch.bfloat16), mask_d, tok_d)
        live = (states_d >= 0)
        toks = torch.where(live, tok_d, torch.full_like(tok_d, -1))      # finished sequences stay finished
        lib.advance_fill_mask(toks, mask_d)
        t_h, e_h, s_h = toks.cpu().numpy(), err_d.cpu().numpy(), states_d.cpu().numpy()
        for b in range(B):
            if t_h[b] < 0 or e_h[b] != 0:
                continue
            if t_h[b] == v.eos_id:
                assert s_h[b] < 0
                finished[b] = bytes(texts[b])
            else:
                texts[b] += v.tokens[t_h[b]]
    done = [t for t in finished if t is not None]
    assert len(done) >= B // 2, f"only {len(done)} of {B} sequences ended"
    for t in done:
        json.loads(t.decode("latin-1"))                          # raises on anything that is not JSON
    assert len({bytes(t) for t in done}) > 5
