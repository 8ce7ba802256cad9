"""Host-side checks of the seeded workload recipes (no arithmetic of the method involved)."""

import numpy as np
import pytest
import torch

from paper_2602_00269_amd import synth


@pytest.mark.parametrize("cfg,lo,hi", [(1, 1, 256), (2, 200, 2000), (3, 500, 4000),
                                       (4, 1, 8192), (5, 64, 4096)])
def test_context_lens_ranges(cfg, lo, hi):
    s = synth._PRESETS[cfg][1]
    lens = synth.draw_context_lens(cfg, s, np.random.default_rng(synth.SEED_BASE + cfg))
    assert lens.dtype == np.int32 and lens.shape == (s,)
    assert lens.min() >= lo and lens.max() <= hi
    again = synth.draw_context_lens(cfg, s, np.random.default_rng(synth.SEED_BASE + cfg))
    assert np.array_equal(lens, again)


def test_cfg4_has_ten_percent_fresh_streams_and_lognormal_body():
    lens = synth.draw_context_lens(4, 512, np.random.default_rng(synth.SEED_BASE + 4))
    assert (lens <= 32).sum() >= 51
    body = lens[lens > 32]
    assert 800 <= np.median(body) <= 1250  # median 1000 up to sampling noise


@pytest.mark.parametrize("cfg", [1, 2])
def test_tables_are_a_partition_of_distinct_blocks(cfg):
    w = synth.make_workload(cfg)
    nb = (w.context_lens.astype(np.int64) + 15) // 16
    used = np.concatenate([w.block_tables[s, :nb[s]] for s in range(w.num_streams)])
    assert used.min() >= 0 and used.max() < w.num_blocks
    assert np.unique(used).size == used.size
    for s in range(w.num_streams):
        assert (w.block_tables[s, nb[s]:] == -1).all()
    if cfg == 2:
        assert used.size == w.num_blocks  # shuffled pool without slack
    unused = np.setdiff1d(np.arange(w.num_blocks), used)
    assert torch.isnan(w.k_pool[0][unused].float()).all()
    assert torch.isfinite(w.k_pool[0][used].float()).all()
    assert w.k_pool[0].dtype == torch.bfloat16 and w.q[0].shape == (w.num_streams, w.num_q_heads,
                                                                    w.head_dim)


def test_pool_slack_for_fragmented_presets():
    lens = synth.draw_context_lens(3, 256, np.random.default_rng(1))
    need = int(((lens.astype(np.int64) + 15) // 16).sum())
    assert synth.pool_blocks_for(3, lens) == int(np.ceil(1.25 * need))


def test_same_seed_same_bits():
    a, b = synth.make_workload(1), synth.make_workload(1)
    assert torch.equal(a.q[0].view(torch.int16), b.q[0].view(torch.int16))
    assert torch.equal(a.k_pool[0].view(torch.int16), b.k_pool[0].view(torch.int16))
    c = synth.make_workload(1, seed=7)
    assert not torch.equal(a.q[0].view(torch.int16), c.q[0].view(torch.int16))


def test_custom_workload_accepts_padded_slots():
    w = synth.make_custom([0, 5, 16, 0, 33], 8, 2, 64, seed=3)
    assert w.block_tables.shape == (5, 3)
    assert (w.block_tables[0] == -1).all() and (w.block_tables[3] == -1).all()
