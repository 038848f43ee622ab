"""The input generators: determinism, ranges, and the torch twin of the numpy generator."""
import numpy as np
import torch

import workloads as W


def test_uniform_is_deterministic_in_range_and_exact():
    idx = np.arange(100000, dtype=np.uint64)
    u = W.uniform_pm1(7, 1, idx, np.float64)
    assert np.array_equal(u, W.uniform_pm1(7, 1, idx, np.float64))
    assert u.min() >= -1.0 and u.max() < 1.0 and abs(u.mean()) < 0.01
    assert not np.array_equal(u, W.uniform_pm1(8, 1, idx, np.float64))
    assert not np.array_equal(u, W.uniform_pm1(7, 2, idx, np.float64))
    f = W.uniform_pm1(7, 1, idx, np.float32)
    assert f.dtype == np.float32 and f.min() >= -1.0 and f.max() < 1.0


def test_torch_generator_matches_numpy_bit_for_bit():
    for start, count in ((0, 5000), (123456789012, 4097)):
        idx = np.arange(start, start + count, dtype=np.uint64)
        for tdt, ndt in ((torch.float64, np.float64), (torch.float32, np.float32)):
            t = W.torch_uniform_pm1(W.BASE_SEED + 2, W.TAG_A, start, count, tdt, "cpu").numpy()
            assert np.array_equal(t, W.uniform_pm1(W.BASE_SEED + 2, W.TAG_A, idx, ndt))


def test_torch_integer_generator_matches_numpy():
    idx = np.arange(777, 777 + 3000, dtype=np.uint64)
    t = W.torch_uniform_pm1(5, W.TAG_B, 777, 3000, torch.float64, "cpu", dist="ints").numpy()
    assert np.array_equal(t, W.small_ints(5, W.TAG_B, idx, np.float64))
    assert t.min() == -4 and t.max() == 4


def test_config2_sample_matches_the_full_tensors():
    pf = W.config2(v=6, o=3)
    A, B, C = W.make_operands(pf)
    Am, Bm, Cm = A.reshape((36, 36), order="F"), B.reshape((36, 9), order="F"), C.reshape((36, 9), order="F")
    sub, a, b, c = W.config2_sample(pf, np.array([0, 5, 35]), np.array([1, 8]))
    assert np.array_equal(a.reshape((3, 36), order="F"), Am[[0, 5, 35], :])
    assert np.array_equal(b.reshape((36, 2), order="F"), Bm[:, [1, 8]])
    assert np.array_equal(c.reshape((3, 2), order="F"), Cm[[0, 5, 35]][:, [1, 8]])
    assert sub.sizes() == (1, 3, 2, 36)


def test_values_follow_logical_index_not_memory_order():
    e = dict(a=3, b=4, c=5)
    t1 = W.tensor("abc", e)
    t2 = W.tensor("abc", e, memory_order="cab")
    v1 = W.strided_view(W.fill(t1, 5, 0, np.float64), t1)
    v2 = W.strided_view(W.fill(t2, 5, 0, np.float64), t2)
    assert np.array_equal(v1, v2)


def test_config_shapes_match_the_stated_sizes():
    sizes = [p.sizes() for p in W.configs_full()]
    assert sizes[0] == (1, 576, 576, 576)
    assert sizes[1] == (1, 36864, 4096, 36864)
    assert sizes[2] == (1, 1961, 61, 1189)
    assert sizes[3] == (512, 96, 96, 96)
    assert sizes[4] == (1, 1024, 1024, 1024)
    assert W.config2().real_flops() == 2 * 36864 * 4096 * 36864
    assert W.config2().algorithmic_bytes() == 14495514624
    assert W.config4().real_flops() == 3623878656
    assert W.config3().D.size == 2 * 37 * 53 * 61 and W.config3().D.strides == (122, 4514, 2)
    assert W.config3().A.strides == (2173, 80401, 1, 41)


def test_config2_samples_reach_every_launch_round_and_xcd_stretch():
    """The full-size check of configuration 2 compares a grid of rows x columns of D.  The 4608
    tiles of 256 x 128 are walked in bands of 4 tile rows; a launch round is 256 consecutive tiles
    of that order (two bands), handed to the 8 XCDs in stretches of 32 consecutive tiles (4 x 8).  Every
    (round, stretch) pair must hold a sample, or a wrong tile in one of them would go unseen."""
    import bench
    p = W.config2()
    _, M, N, _ = p.sizes()
    tm, tn = 256, 128
    tiles_m, tiles_n = M // tm, N // tn
    assert (tiles_m, tiles_n) == (144, 32)
    m_idx, n_idx = bench.config2_sample_indices(p, tm, tn, np.random.default_rng(p.seed))
    assert len(m_idx) * len(n_idx) >= 65536
    # both sides of every tile boundary
    assert all({e - 1, e} <= set(int(v) for v in m_idx) for e in range(tm, M, tm))
    assert all({e - 1, e} <= set(int(v) for v in n_idx) for e in range(tn, N, tn))
    seen = set()
    for m in m_idx:
        for n in n_idx:
            row, col = int(m) // tm, int(n) // tn
            band = row // 4
            position = band * 4 * tiles_n + (row % 4) + 4 * col        # place in the tile order
            launch_round, in_round = divmod(position, 256)
            seen.add((launch_round, in_round // 32))
    assert seen == {(r, x) for r in range(tiles_m * tiles_n // 256) for x in range(8)}
    # tile-boundary rows and columns are among the samples
    assert {0, tm - 1, tm, M - 1} <= set(int(v) for v in m_idx) and {0, tn - 1, tn, N - 1} <= set(int(v) for v in n_idx)
