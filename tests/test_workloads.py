"""The seeded input generators: storage-format conversion and the shape of the index sets."""
import numpy as np
import pytest

from workloads import (CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_rng, tree_subsets,
                       zipf_subset)


def test_bf16_rounding_matches_torch_and_ties_to_even():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * s for s in (1e-3, 0.02, 1, 50)])
    x = np.concatenate([x, np.array([0.0, -0.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8)], np.float32)])
    bits = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = bf16_bits_to_f32(bits)
    assert back[-3] == 1.0 and back[-2] == 1 + 2.0 ** -6 and back[-1] == -1.0
    assert np.array_equal(f32_to_bf16_bits(back), bits)          # idempotent


def test_zipf_subset_shape_and_bias():
    rng = make_rng(9, 2)
    V, k = 20000, 1500
    idx = zipf_subset(rng, V, k)
    assert idx.dtype == np.int32 and idx.shape == (k,)
    assert np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < V
    # frequent (low-rank) tokens dominate: far more than the uniform share falls in the first 10%
    assert (idx < V // 10).mean() > 0.5
    perm = np.random.default_rng(1).permutation(V)
    idx2 = zipf_subset(make_rng(9, 2), V, k, rank_of_id=perm)
    assert (perm[idx2] < V // 10).mean() > 0.5 and (idx2 < V // 10).mean() < 0.3
    assert np.array_equal(zipf_subset(rng, 50, 50), np.arange(50))
    assert np.array_equal(zipf_subset(make_rng(9, 2), V, k), idx)   # seeded


def test_tree_subsets_share_the_step_level_set():
    rng = make_rng(9, 2)
    idx, S = tree_subsets(rng, 5000, rows=6, k=400, shared=200)
    assert idx.shape == (6, 400) and len(S) == 200
    for r in range(6):
        assert np.all(np.diff(idx[r]) > 0)
        assert np.isin(S, idx[r]).all()
    priv = [np.setdiff1d(idx[r], S) for r in range(6)]
    assert all(len(p) == 200 for p in priv)
    assert len(np.intersect1d(priv[0], priv[1])) < 200       # private parts differ


def test_config_table_matches_the_named_shapes():
    c = CONFIGS
    assert (c[1].d, c[1].V, c[1].k, c[1].kd, c[1].dtype) == (256, 8192, 512, 8, "f32")
    assert (c[2].d, c[2].V, c[2].k, c[2].rows, c[2].steps, c[2].dtype) == (4096, 128256, 8192, 1, 1000, "bf16")
    assert (c[3].rows, c[3].k, c[3].shared, c[3].kd) == (60, 4096, 2048, 10)
    assert (c[4].d, c[4].V, c[4].rows, c[4].k_sweep) == (3840, 262144, 8, (2048, 8192, 32768))
    assert (c[5].V, c[5].rows, c[5].k, c[5].d_prime, c[5].kd) == (151936, 512, 8192, 256, 10)
    idx = c[1].indices(3)
    assert idx.shape == (3, 1, 512)
    h = c[1].hidden(3)
    assert h.shape == (3, 1, 256) and h.dtype == np.float32
    assert abs(float(c[1].weights().std()) - 0.02) < 1e-3
