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


def test_cfg3_json_full_size():
    """B=256, V=128256, 256 steps: states/stacks on every step, the whole bitmask and masked
    logits on 6 steps spread over the run, two full mask rows on every other step."""
    r = replay(3, full_mask_steps=[0, 1, 50, 100, 200, 255])
    assert r["full_masks"] == 6 and r["sampled_rows"] == 500


def test_cfg4_schema_full_size():
    r = replay(4, full_mask_steps=[0, 40, 128, 255])
    assert r["full_masks"] == 4


def test_cfg5_mixed_grammars_deep_stacks():
    r = replay(5, full_mask_steps=[0, 1, 64, 256, 511])
    assert r["full_masks"] == 5
    assert max(r["depth_hist"]) >= 60 and len(r["depth_hist"]) > 40


def test_advance_fill_mask_all_configs():
    """pre3_advance_fill_mask (advance + next mask in one launch, slot reuse on EOS) on every
    configuration; config 2 also with shallow conditions (leftover walks inside the fused kernel)
    and without token-level edges (two-launch fallback)."""
    assert replay_advance_fill(1)["full_masks"] == 32
    assert replay_advance_fill(2, steps=64)["full_masks"] == 64
    assert replay_advance_fill(2, steps=12, max_condition_depth=2)["full_masks"] == 12
    assert replay_advance_fill(2, steps=12, token_edges=False)["full_masks"] == 12
    assert replay_advance_fill(3, steps=96, full_mask_steps=[0, 40, 95])["full_masks"] == 3
    assert replay_advance_fill(4, steps=64, full_mask_steps=[0, 63])["full_masks"] == 2
    assert replay_advance_fill(5, steps=96, full_mask_steps=[0, 50, 95])["full_masks"] == 3
