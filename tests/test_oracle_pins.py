"""CPU tests: the oracle against what the paper and the mathematics fix (see tests/pins.py)."""
import numpy as np
import pytest

import oracle
from paper_2402_07710_amd import synth
from tests import pins


def test_fig_subm_2d(orc):
    pins.check_fig_subm_2d(orc)


def test_fig_oft_2d(orc):
    pins.check_fig_oft_2d(orc)


def test_eq_cell_mapping(orc):
    pins.check_eq_cell_mapping(orc)


@pytest.mark.parametrize("grid,n,K,s,mode,ci,co,nb", [
    (6, 40, 3, 1, "subm", 3, 2, 1), (5, 60, 3, 1, "subm", 2, 3, 2), (7, 30, 5, 1, "subm", 2, 2, 1),
    (8, 100, 3, 1, "subm", 4, 4, 1), (5, 125, 3, 1, "subm", 1, 1, 1), (4, 1, 3, 1, "subm", 2, 2, 1),
    (6, 50, 2, 2, "strided", 3, 2, 1), (7, 40, 3, 3, "strided", 2, 2, 2), (6, 30, 3, 2, "strided", 2, 3, 1),
    (8, 200, 2, 2, "strided", 2, 2, 1), (6, 216, 2, 2, "strided", 1, 2, 1), (7, 20, 4, 2, "strided", 2, 1, 1),
    (5, 10, 1, 1, "subm", 3, 3, 1), (6, 25, 1, 2, "strided", 2, 2, 1),
])
def test_dense_brute_force(orc, grid, n, K, s, mode, ci, co, nb):
    pins.check_dense(orc, np.random.default_rng(grid * 1000 + n), grid, n, K, s, mode, ci, co, nb)


def test_empty_input(orc):
    km = orc.kmap(np.zeros((0, 4), np.int32), 3, 1, "subm")
    assert km["n_out"] == 0 and km["offset_start"][-1] == 0
    out = orc.conv(np.zeros((0, 4)), np.zeros((27, 4, 2)), km)
    assert out.shape == (0, 2)


def test_symmetry_centre(orc):
    c = synth.uniform_cells(400, 9, seed=1)
    pins.check_symmetry_and_centre(orc, c, 3)
    pins.check_symmetry_and_centre(orc, c[:150], 5)


def test_delta_weights(orc):
    rng = np.random.default_rng(2)
    c = synth.uniform_cells(300, 8, seed=2)
    pins.check_delta_weights(orc, c, rng.standard_normal((300, 4)).astype(np.float32), 3)


@pytest.mark.parametrize("n", [1, 2, 4, 5, 6])
def test_full_grid_counts(orc, n):
    pins.check_full_grid_counts(orc, n)


def test_isolated_is_matmul(orc):
    pins.check_isolated_is_matmul(orc, np.random.default_rng(3))


@pytest.mark.parametrize("s", [2, 3, 4])
def test_strided_partition(orc, s):
    c = synth.uniform_cells(500, 12, seed=4)
    c[:, 0] = np.arange(len(c)) % 3
    pins.check_strided_partition(orc, c, s)


@pytest.mark.parametrize("K,s,mode", [(3, 1, "subm"), (2, 2, "strided"), (3, 2, "strided"), (5, 1, "subm")])
def test_invariances(orc, K, s, mode):
    c = synth.uniform_cells(200, 8, seed=5)
    pins.check_invariances(orc, np.random.default_rng(5), c, K, s, mode)


@pytest.mark.parametrize("K,s,mode", [(3, 1, "subm"), (2, 2, "strided"), (3, 2, "strided")])
def test_alg2_formulation(orc, K, s, mode):
    c = synth.uniform_cells(150, 7, seed=6)
    pins.check_alg2_formulation(orc, np.random.default_rng(6), c, K, s, mode)


@pytest.mark.parametrize("K,s,mode,g", [(3, 1, "subm", 64), (3, 1, "subm", 7), (2, 2, "strided", 16), (3, 2, "strided", 5)])
def test_group_sums_by_linearity(orc, K, s, mode, g):
    """The whole-output check the full-size GPU test uses (sums over groups of output rows from a
    map and matrix products alone) against the oracle's row-by-row result."""
    c = synth.uniform_cells(300, 8, seed=11)
    pins.check_group_sums(orc, np.random.default_rng(11), c, K, s, mode, g)


@pytest.mark.parametrize("s", [2, 3])
def test_inverse_is_adjoint(orc, s):
    c = synth.uniform_cells(400, 10, seed=8)
    c[:, 0] = np.arange(len(c)) % 2
    pins.check_inverse_is_adjoint(orc, np.random.default_rng(8), c, s)


def test_expected_pairs_uniform(orc):
    pins.check_expected_pairs_uniform(orc)


def test_rejects_bad_input(orc):
    dup = np.array([[0, 1, 2, 3], [0, 1, 2, 3]], np.int32)
    with pytest.raises(oracle.OracleError):
        orc.kmap(dup, 3, 1, "subm")
    neg = np.array([[0, -1, 2, 3]], np.int32)
    with pytest.raises(oracle.OracleError):
        orc.kmap(neg, 3, 1, "subm")
    ok = np.array([[0, 1, 2, 3]], np.int32)
    with pytest.raises(oracle.OracleError):
        orc.kmap(ok, 2, 1, "subm")          # even K has no centre
    with pytest.raises(oracle.OracleError):
        orc.kmap(ok, 3, 2, "subm")          # submanifold layers have stride 1


def test_threads_do_not_change_result(orc):
    c = synth.uniform_cells(500, 10, seed=7)
    rng = np.random.default_rng(7)
    f, W = rng.standard_normal((500, 6)), rng.standard_normal((27, 6, 10))
    km = orc.kmap(c, 3, 1, "subm")
    assert np.array_equal(orc.conv(f, W, km, threads=1), orc.conv(f, W, km, threads=4))


def test_lidar_scene_statistics(orc):
    """The LiDAR-shaped generator gives what the design notes state: N in the tens of thousands,
    several pairs per voxel, and a K=s=2 layer that shrinks it by about a factor of two."""
    c = synth.lidar_scene(0)
    assert 40_000 < len(c) < 120_000
    km = orc.kmap(c, 3, 1, "subm")
    assert 3.0 < km["offset_start"][-1] / len(c) < 10.0
    km2 = orc.kmap(c, 2, 2, "strided")
    assert 1.3 < len(c) / km2["n_out"] < 3.0
