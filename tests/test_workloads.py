"""The seeded input recipes: shapes, determinism and the structure each config asks for."""
import numpy as np

import workloads as W


def test_config_table_matches_the_five_named_workloads():
    got = [(c.n, c.d, c.compressor, c.k, c.block, c.layer_blocks, c.steps) for c in W.CONFIGS]
    assert got == [
        (4, 65_536, W.TOPK, 655, 0, 0, 10),
        (16, 1_199_882, W.BLOCKSIGN, 0, 4096, 0, 20),
        (16, 11_173_962, W.TOPK, 111_740, 0, 0, 20),
        (32, 25_557_032, W.BLOCKSIGN, 0, 0, 161, 10),
        (8, 110_000_000, W.TOPK, 110_000, 0, 0, 5),
    ]
    assert W.CONFIGS[1].algorithmic_bytes() == 12 * 16 * 1_199_882 + 32 * 1_199_882


def test_grads_are_a_pure_function_of_seed_step_worker():
    w = W.get(0)
    a = w.grads(3)
    b = w.grads(3, threads=1)
    assert a.dtype == np.float32 and a.shape == (4, 65_536) and a.flags.c_contiguous
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert not np.array_equal(a, w.grads(4))
    assert not np.array_equal(a[0], a[1])


def test_uniform_and_layer_block_tables():
    off = W.get(1).block_offsets()
    assert off.size == 294 and off[0] == 0 and off[-1] == 1_199_882
    assert np.all(np.diff(off)[:-1] == 4096) and np.diff(off)[-1] == 3850
    off = W.get(3).block_offsets()
    lens = np.diff(off)
    assert off.size == 162 and off[0] == 0 and off[-1] == 25_557_032 and lens.min() >= 1
    assert lens.max() > 1_000_000 and lens.min() < 5_000          # spans small and very large layers
    small = W.get(3).scaled(50_000).block_offsets()
    assert small[-1] == 50_000 and np.diff(small).min() >= 1


def test_cfg2_recipe_has_exact_zeros_and_duplicated_magnitudes():
    w = W.get(2).scaled(200_000, n=2)
    g = w.grads(0)
    assert w.k == 2000
    for i in range(2):
        assert (g[i] == 0).sum() >= 150
        mags = np.abs(g[i][g[i] != 0])
        assert mags.size - np.unique(mags).size >= 1000


def test_cfg4_recipe_is_bf16_representable():
    w = W.get(4).scaled(100_000, n=2)
    g = w.grads(1)
    assert np.all((g.view(np.uint32) & 0xFFFF) == 0)
    assert np.unique(np.abs(g)).size < 40_000
