"""Replays a seeded trajectory through the GPU library and the CPU oracle side by side."""
import time

import numpy as np

from oracle import Oracle, apply_mask as oracle_apply_mask
from workloads import configs, trajectory
from workloads.vocab import bf16_logits


def make_library(cfg, **kw):
    from paper_2506_03887_amd import Pre3
    v = cfg.vocab
    return Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cfg.cap,
                compact_cycles=cfg.compact, **kw)


def replay(cfg_idx, steps=None, full_mask_steps=None, rows_per_step=2, check_apply=True, apply_steps=None, log=print,
           **lib_options):
    """Runs `steps` decode steps of config `cfg_idx` on the GPU through the C ABI and checks,
    against the oracle on the same inputs:
      - states, len, live stack entries and err of every sequence after every advance;
      - the whole bitmask (all B*W words) on the steps in `full_mask_steps` (None = every step), and
        on those of them in `apply_steps` (None = all of them) the masked bf16 logits (all B*V raw
        patterns) through pre3_apply_mask and through the fused call;
      - the full mask rows of `rows_per_step` seeded random sequences on every other step;
      - at the end, that no kernel stopped a walk at an internal guard (the fault counter is 0).
    Returns a dict of counters."""
    import torch
    from paper_2506_03887_amd import apply_mask

    cfg = configs.get(cfg_idx)
    v = cfg.vocab
    steps = cfg.steps if steps is None else steps
    o = Oracle(cfg.grammars, compact_cycles=cfg.compact)
    gi, depths = configs.sequence_setup(cfg)
    t0 = time.time()
    traj = trajectory.generate(o, v, cfg.batch, steps, cfg.cap, cfg.seed, gi, cfg.nest_cap, None,
                               cfg.json_strings, depths, marker=cfg.marker, p_line_feed=cfg.p_line_feed)
    log(f"[cfg {cfg_idx}] trajectory of {steps} steps in {time.time() - t0:.1f}s; "
        f"{int(traj.reset.sum())} resets, {int((traj.tokens == v.eos_id).sum())} EOS", flush=True)
    lib = make_library(cfg, **lib_options)
    log(f"[cfg {cfg_idx}] token edges: {lib.token_edge_stats()}", flush=True)
    dev = torch.device("cuda:0")
    B, cap, W, V = cfg.batch, cfg.cap, v.words, v.n_tokens

    data_h, len_h = traj.init_data.copy(), traj.init_len.copy()
    states_h = data_h[np.arange(B), len_h - 1].copy()
    data_d = torch.from_numpy(data_h).to(dev)
    len_d = torch.from_numpy(len_h).to(dev)
    states_d = torch.from_numpy(states_h).to(dev)
    err_d = torch.full((B,), -7, dtype=torch.int32, device=dev)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    s0 = np.array([o.initial_state(int(g)) for g in gi], dtype=np.int32)
    rng = np.random.default_rng(cfg.seed + 1)
    full = set(range(steps)) if full_mask_steps is None else set(full_mask_steps)
    with_apply = full if apply_steps is None else set(apply_steps) & full
    n_full = n_rows = n_apply = 0

    for s in range(steps):
        rs = np.flatnonzero(traj.reset[s])
        if len(rs):                      # slot reuse: finished sequences start afresh
            data_h[rs, 0], len_h[rs], states_h[rs] = s0[rs], 1, s0[rs]
            idx = torch.from_numpy(rs).to(dev)
            data_d[idx, 0] = torch.from_numpy(s0[rs]).to(dev)
            len_d[idx] = 1
            states_d[idx] = torch.from_numpy(s0[rs]).to(dev)
        mask_d.fill_(0x5A5A5A5A)
        lib.fill_mask(states_d, data_d, len_d, mask_d)
        got = mask_d.cpu().numpy().view(np.uint32)
        if s in full:
            want = o.fill_mask(states_h, data_h, len_h, v)
            bad = np.argwhere(got != want)
            assert len(bad) == 0, f"cfg {cfg_idx} step {s}: {len(bad)} mask words differ, first (row, word) {bad[0]}"
            n_full += 1
            if check_apply and s in with_apply:
                n_apply += 1
                logits = bf16_logits(rng, B, V)
                logits_d = torch.from_numpy(logits.view(np.int16)).to(dev)
                fused_logits_d = logits_d.clone()
                apply_mask(logits_d, mask_d, V)
                oracle_apply_mask(logits, want, V)
                out = logits_d.cpu().numpy().view(np.uint16)
                assert (out == logits).all(), f"cfg {cfg_idx} step {s}: masked logits differ"
                # the fused entry point must leave exactly the same bitmask and logits
                fused_mask_d = torch.full_like(mask_d, 0x3C3C3C3C)
                lib.fill_apply_mask(states_d, data_d, len_d, fused_mask_d, fused_logits_d)
                assert (fused_mask_d.cpu().numpy().view(np.uint32) == want).all(), \
                    f"cfg {cfg_idx} step {s}: fused bitmask differs"
                assert (fused_logits_d.cpu().numpy().view(np.uint16) == logits).all(), \
                    f"cfg {cfg_idx} step {s}: fused masked logits differ"
        else:
            for b in rng.integers(0, B, size=rows_per_step):
                want = o.mask_row(data_h[b, : len_h[b]], v, done=states_h[b] < 0)
                assert (got[b] == want).all(), f"cfg {cfg_idx} step {s} row {b}: mask row differs"
                n_rows += 1
        tok = traj.tokens[s]
        lib.advance(torch.from_numpy(tok).to(dev))
        err_h = o.advance_batch(states_h, data_h, len_h, tok, v)
        assert (err_d.cpu().numpy() == err_h).all() and not err_h.any(), f"cfg {cfg_idx} step {s}: err differs"
        assert (states_d.cpu().numpy() == states_h).all(), f"cfg {cfg_idx} step {s}: states differ"
        len_g = len_d.cpu().numpy()
        assert (len_g == len_h).all(), f"cfg {cfg_idx} step {s}: len differs"
        live = np.arange(cap)[None, :] < len_h[:, None]
        data_g = data_d.cpu().numpy()
        assert (data_g[live] == data_h[live]).all(), f"cfg {cfg_idx} step {s}: stack entries differ"
        if s % 32 == 31 or s == steps - 1:
            log(f"[cfg {cfg_idx}] step {s + 1}/{steps} ok ({n_full} full masks, {n_rows} sampled rows)", flush=True)
    assert lib.fault_count() == 0, f"cfg {cfg_idx}: a kernel stopped a walk at an internal guard"
    return dict(steps=steps, full_masks=n_full, sampled_rows=n_rows, applied=n_apply, depth_hist=traj.depth_hist)


def replay_advance_fill(cfg_idx, steps=None, full_mask_steps=None, rows_per_step=2, log=print, step_call_every=0,
                        logits_pad=0, one_kernel=True, batch=None, **lib_options):
    """Same trajectory, driven through pre3_advance_fill_mask with slot reuse on EOS: after every
    call the device's states/len/live stack/err and the next mask must equal the oracle's
    advance followed by its fill (whole bitmask on `full_mask_steps`, sampled rows otherwise).
    step_call_every = k > 0: every k-th step goes through pre3_advance_fill_apply_mask (the whole step
    as one call) on fresh seeded logits whose rows are `logits_pad` elements longer than the vocabulary;
    on those steps the whole bitmask is checked, and all B * (V + pad) logit patterns against the
    oracle's apply_mask on the oracle's mask (the padding must come back untouched).  one_kernel: ask for
    the one-kernel form whatever the batch size (False: the library chooses by the batch size).
    batch: another number of sequences than the configuration's."""
    import dataclasses
    import torch

    cfg = configs.get(cfg_idx)
    if batch is not None:
        cfg = dataclasses.replace(cfg, batch=batch)
    v = cfg.vocab
    steps = cfg.steps if steps is None else steps
    o = Oracle(cfg.grammars, compact_cycles=cfg.compact)
    gi, depths = configs.sequence_setup(cfg)
    traj = trajectory.generate(o, v, cfg.batch, steps, cfg.cap, cfg.seed, gi, cfg.nest_cap, None,
                               cfg.json_strings, depths, marker=cfg.marker, p_line_feed=cfg.p_line_feed)
    # slot reuse in the trajectory == restart right after an EOS token
    assert (traj.reset[1:] == (traj.tokens[:-1] == v.eos_id)).all() and not traj.reset[0].any()
    lib = make_library(cfg, **lib_options)
    dev = torch.device("cuda:0")
    B, cap, W = cfg.batch, cfg.cap, v.words
    data_h, len_h = traj.init_data.copy(), traj.init_len.copy()
    states_h = data_h[np.arange(B), len_h - 1].copy()
    data_d = torch.from_numpy(data_h).to(dev)
    len_d = torch.from_numpy(len_h).to(dev)
    states_d = torch.from_numpy(states_h).to(dev)
    err_d = torch.full((B,), -7, dtype=torch.int32, device=dev)
    mask_d = torch.full((B, W), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    rng = np.random.default_rng(cfg.seed + 2)
    full = set(range(steps)) if full_mask_steps is None else set(full_mask_steps)
    n_full = n_rows = 0
    n_step_calls = 0
    V = v.n_tokens
    for s in range(steps):
        tok = traj.tokens[s]
        one_call = step_call_every > 0 and s % step_call_every == 0
        if one_call:
            logits = np.full((B, V + logits_pad), 0x1234, dtype=np.uint16)
            logits[:, :V] = bf16_logits(rng, B, V)
            logits_d = torch.from_numpy(logits.view(np.int16)).to(dev)
            mask_d.fill_(0x5A5A5A5A)
            lib.advance_fill_apply_mask(torch.from_numpy(tok).to(dev), mask_d, logits_d, restart_on_eos=True, one_kernel=one_kernel)
        else:
            lib.advance_fill_mask(torch.from_numpy(tok).to(dev), mask_d, restart_on_eos=True)
        err_h = o.advance_batch(states_h, data_h, len_h, tok, v)
        done = states_h < 0
        states_h[done], len_h[done] = data_h[done, 0], 1                   # restart on EOS
        assert (err_d.cpu().numpy() == err_h).all() and not err_h.any(), f"cfg {cfg_idx} step {s}: err differs"
        assert (states_d.cpu().numpy() == states_h).all(), f"cfg {cfg_idx} step {s}: states differ"
        assert (len_d.cpu().numpy() == len_h).all(), f"cfg {cfg_idx} step {s}: len differs"
        live = np.arange(cap)[None, :] < len_h[:, None]
        assert (data_d.cpu().numpy()[live] == data_h[live]).all(), f"cfg {cfg_idx} step {s}: stack entries differ"
        got = mask_d.cpu().numpy().view(np.uint32)
        if s in full or one_call:
            want = o.fill_mask(states_h, data_h, len_h, v)
            bad = np.argwhere(got != want)
            assert len(bad) == 0, f"cfg {cfg_idx} step {s}: {len(bad)} mask words differ, first (row, word) {bad[0]}"
            n_full += 1
            if one_call:
                oracle_apply_mask(logits, want, V)
                out = logits_d.cpu().numpy().view(np.uint16)
                bad = np.argwhere(out != logits)
                assert len(bad) == 0, f"cfg {cfg_idx} step {s}: {len(bad)} logits differ after the one-call step, first (row, column) {bad[0]}"
                n_step_calls += 1
        else:
            for b in rng.integers(0, B, size=rows_per_step):
                want = o.mask_row(data_h[b, : len_h[b]], v, done=states_h[b] < 0)
                assert (got[b] == want).all(), f"cfg {cfg_idx} step {s} row {b}: mask row differs"
                n_rows += 1
        if s % 32 == 31 or s == steps - 1:
            log(f"[cfg {cfg_idx}] advance+fill step {s + 1}/{steps} ok ({n_full} full masks, {n_rows} sampled rows)", flush=True)
    assert lib.fault_count() == 0, f"cfg {cfg_idx}: a kernel stopped a walk at an internal guard"
    return dict(steps=steps, full_masks=n_full, sampled_rows=n_rows, step_calls=n_step_calls)
