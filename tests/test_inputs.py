"""The seeded input generator: determinism, ranges, moments, and block/matrix agreement (no GPU)."""
import numpy as np
import pytest

from paper_1202_3173_amd import inputs


def test_block_matches_full_matrix_and_is_deterministic():
    n = 96
    for dist in inputs.DISTS:
        M = inputs.matrix(n, 5, 1, dist, chunk_rows=17)
        rows = np.array([0, 95, 40, 40])
        cols = np.array([3, 0, 77])
        assert np.array_equal(inputs.block(n, 5, 1, dist, rows, cols), M[np.ix_(rows, cols)])
        assert np.array_equal(M, inputs.matrix(n, 5, 1, dist))
        assert not np.array_equal(M, inputs.matrix(n, 5, 0, dist))
        assert not np.array_equal(M, inputs.matrix(n, 6, 1, dist))


def test_distribution_shapes():
    n = 512
    U = inputs.matrix(n, 1, 0, "uniform")
    assert U.min() >= -1.0 and U.max() < 1.0
    assert abs(U.mean()) < 0.01 and abs(U.var() - 1.0 / 3.0) < 0.01
    R = inputs.matrix(n, 1, 0, "rowscaled")
    assert np.array_equal(R, U * (1.0 + np.arange(n).reshape(-1, 1) / n))
    Z = inputs.matrix(n, 1, 0, "integer")
    assert np.array_equal(Z, np.round(Z)) and Z.min() == -8 and Z.max() == 8
    counts = np.bincount((Z + 8).astype(int).ravel(), minlength=17)
    assert counts.min() > 0.9 * n * n / 17 and counts.max() < 1.1 * n * n / 17
    G = inputs.matrix(n, 1, 0, "normal")
    assert abs(G.mean()) < 0.01 and abs(G.var() - 1.0) < 0.02 and np.isfinite(G).all()
    assert abs(np.mean(G ** 4) - 3.0) < 0.1


def test_known_first_values():
    # splitmix64 with seed 0 yields 0xE220A8397B1DCDAF first (published test vector of the generator);
    # our counter form reproduces that function, so the mixer is pinned independently of this module.
    z = inputs._mix(np.asarray(np.uint64(0) + inputs.GAMMA, dtype=np.uint64))
    assert int(z) == 0xE220A8397B1DCDAF


def test_configs_table():
    assert [c["n"] for c in inputs.CONFIGS] == [256, 4096, 16384, 23520, 94080]
    for c in inputs.CONFIGS:
        assert c["n"] % 2 ** c["levels"] == 0
        assert c["schedule"] is None or len(c["schedule"]) == c["levels"]
    with pytest.raises(ValueError):
        inputs.block(4, 0, 0, "cauchy", [0], [0])
