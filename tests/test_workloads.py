"""The seeded input recipes: shapes, ranges, determinism, block-table validity."""
import numpy as np
import pytest

from paper_2602_12151_amd import workloads as wl


def test_counter_rng_is_deterministic_and_streams_differ():
    a, b = wl.CounterRng(7), wl.CounterRng(7)
    x, y = a.raw(1000), b.raw(1000)
    assert np.array_equal(x, y)
    assert not np.array_equal(a.raw(1000), x)          # next stream of the same rng differs
    u = wl.CounterRng(1).uniform(200000)
    assert 0.0 < u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 5e-3
    z = wl.CounterRng(2).normal(200000)
    assert abs(z.mean()) < 1e-2 and abs(z.std() - 1.0) < 1e-2
    p = wl.CounterRng(3).permutation(1000)
    assert np.array_equal(np.sort(p), np.arange(1000))
    k = wl.CounterRng(4).integers(3, 9, 50000)
    assert k.min() == 3 and k.max() == 9


@pytest.mark.parametrize("idx,lo,hi", [(1, 128, 2048), (2, 1024, 16384), (4, 65536, 131072)])
def test_uniform_length_recipes(idx, lo, hi):
    w = wl.WORKLOADS[idx]
    lens = wl.context_lens(w)
    assert lens.dtype == np.int32 and lens.shape == (w.batch,)
    assert lens.min() >= lo and lens.max() <= hi
    assert np.array_equal(lens, wl.context_lens(w))    # same seed, same draw


def test_heterogeneous_mix_recipe():
    w = wl.WORKLOADS[3]
    lens = wl.context_lens(w)
    assert lens.shape == (256,)
    long_ = lens[lens >= 8192]
    short = lens[lens <= 4096]
    assert len(long_) == 77 and len(short) == 179      # 30 % / 70 % of 256, deterministic counts
    assert short.min() >= 16 and long_.max() <= 32768
    assert 350 < np.median(short) < 750                # lognormal median 512
    # shuffled: long requests are not all at the end
    assert (lens[:179] >= 8192).any()
    # the long 30 % carry > 85 % of the tokens
    assert long_.sum() / lens.sum() > 0.85


def test_block_table_is_a_valid_scatter():
    w = wl.WORKLOADS[1]
    lens = wl.context_lens(w)
    npool = wl.pool_pages(w, lens)
    need = wl.pages_needed(lens)
    assert npool == int(np.ceil(1.25 * need.sum()))
    bt, used = wl.make_block_table(lens, npool, wl.CounterRng(5))
    assert len(np.unique(used)) == len(used) == need.sum()
    assert used.min() >= 0 and used.max() < npool
    for b in range(w.batch):
        assert (bt[b, : need[b]] >= 0).all() and (bt[b, need[b]:] == -1).all()
    assert not np.array_equal(np.sort(used), used)     # actually permuted


def test_tiny_inputs_shapes_and_bytes():
    w = wl.WORKLOADS[0]
    inp = wl.make_inputs(w)
    assert inp.q.shape == (4, 8, 64) and inp.k_pages.shape == (64, 2, 16, 64)
    assert inp.block_table.shape[0] == 4 and inp.block_table.shape[1] == 33
    assert len(inp.used_pages) == 2 + 4 + 13 + 33
    assert inp.kv_bytes == (17 + 64 + 200 + 513) * 2 * 64 * 4
    assert inp.scale == 0.125
    again = wl.make_inputs(w)
    assert (inp.k_pages.view(dtype=__import__("torch").int16) ==
            again.k_pages.view(dtype=__import__("torch").int16)).all()


def test_partial_fill_touches_only_used_pages():
    import torch
    w = wl.WORKLOADS[0]
    lens = np.array([5, 40], dtype=np.int32)
    inp = wl.make_inputs(w, lens=lens, fill_unused=False, pool_pages_override=32)
    assert inp.k_pages.shape[0] == 32 and len(inp.used_pages) == 1 + 3
    assert torch.isfinite(inp.k_pages[torch.from_numpy(inp.used_pages)].float()).all()
