"""Pins of the CPU checker's k-nearest-neighbour graph (no GPU): a library k-d tree, exact ties on lattices,
the generator of the benchmark workloads (an independent numpy/scipy construction) and structural invariants."""
import numpy as np
import pytest
from scipy.spatial import cKDTree

from paper_2410_03462_amd import synth


def test_lists_match_a_kd_tree_on_random_points(oracle):
    rng = np.random.default_rng(0)
    pts = rng.random((3000, 3)).astype(np.float32)
    k = 9
    idx, d2 = oracle.knn_lists(pts, k)
    dist, ref = cKDTree(pts.astype(np.float64)).query(pts.astype(np.float64), k=k + 1)
    dist, ref = dist[:, 1:], ref[:, 1:]
    assert np.allclose(np.sqrt(d2.astype(np.float64)), dist, rtol=2e-6, atol=1e-9)
    # indices agree wherever consecutive distances are separated by more than fp32 rounding
    gap_ok = np.ones_like(ref, dtype=bool)
    close = np.abs(np.diff(dist, axis=1)) <= 4e-6 * dist[:, 1:]
    gap_ok[:, 1:] &= ~close
    gap_ok[:, :-1] &= ~close
    assert gap_ok.mean() > 0.99
    assert np.array_equal(idx[gap_ok], ref[gap_ok])
    assert np.all(idx != np.arange(len(pts))[:, None])
    assert np.all(np.diff(d2, axis=1) >= 0)


def test_ties_go_to_the_smaller_index(oracle):
    # points on a line at integer abscissae: left and right neighbours are equidistant
    pts = np.zeros((7, 3), np.float32); pts[:, 0] = np.arange(7)
    idx, d2 = oracle.knn_lists(pts, 2)
    assert idx.tolist() == [[1, 2], [0, 2], [1, 3], [2, 4], [3, 5], [4, 6], [5, 4]]
    assert np.array_equal(d2[3], [1.0, 1.0]) and np.array_equal(d2[0], [1.0, 4.0])
    idx1, _ = oracle.knn_lists(pts, 1)
    assert idx1[:, 0].tolist() == [1, 0, 1, 2, 3, 4, 5]
    # centre of a 3x3x3 lattice: the six face neighbours, by index
    g = np.stack(np.meshgrid(np.arange(3), np.arange(3), np.arange(3), indexing="ij"), -1).reshape(-1, 3).astype(np.float32)
    idx, d2 = oracle.knn_lists(g, 6)
    assert idx[13].tolist() == [4, 10, 12, 14, 16, 22] and np.all(d2[13] == 1.0)
    # fewer points than k
    idx, d2 = oracle.knn_lists(g[:3], 5)
    assert np.all(idx[:, 2:] == -1) and np.all(np.isinf(d2[:, 2:])) and np.all(idx[:, :2] >= 0)


@pytest.mark.parametrize("kernel,kind", [("exp", 1), ("gauss", 2)])
def test_symmetrised_graph_equals_the_workload_generator(oracle, kernel, kind):
    rng = np.random.default_rng(1)
    pts = synth.cluster_points(1500, 4, 0.05, rng).astype(np.float32)
    k = 8
    ref = synth.knn_graph(pts.astype(np.float64), k, kernel)
    dist, _ = cKDTree(pts.astype(np.float64)).query(pts.astype(np.float64), k=k + 1)
    sigma = float(np.median(dist[:, 1:]))
    rp, col, w = oracle.knn_graph(pts, k, True, kind, sigma)
    assert np.array_equal(rp, ref.row_ptr) and np.array_equal(col, ref.col)
    assert np.allclose(w, ref.w, rtol=2e-5, atol=1e-9)


def test_structure_and_other_weightings(oracle):
    rng = np.random.default_rng(2)
    pts = rng.random((400, 3)).astype(np.float32)
    n, k = len(pts), 5
    idx, d2 = oracle.knn_lists(pts, k)
    rp, col, w = oracle.knn_graph(pts, k, True, 0)
    rows = np.repeat(np.arange(n), np.diff(rp))
    A = np.zeros((n, n), bool); A[rows, col] = True
    assert np.array_equal(A, A.T) and not A.diagonal().any()
    D = np.zeros((n, n), bool); D[np.repeat(np.arange(n), k), idx.ravel()] = True
    assert np.array_equal(A, D | D.T)
    for i in range(n):
        assert np.all(np.diff(col[rp[i]:rp[i + 1]]) > 0)
    assert np.allclose(w, 1.0 / np.diff(rp)[rows], rtol=1e-15)
    # directed: exactly the lists, ascending, uniform weights 1/k
    rp, col, w = oracle.knn_graph(pts, k, False, 0)
    assert np.array_equal(rp, np.arange(n + 1) * k)
    assert np.array_equal(col.reshape(n, k), np.sort(idx, axis=1))
    assert np.allclose(w, 1.0 / k)
    # kernel weights: rows sum to one, closer is heavier
    rp, col, w = oracle.knn_graph(pts, k, False, 2, 0.1)
    assert np.allclose(np.add.reduceat(w, rp[:-1]), 1.0, rtol=1e-12)
    i = 17
    order = np.argsort(col[rp[i]:rp[i + 1]])
    d2_by_col = d2[i][np.argsort(idx[i])]
    assert np.all(np.diff(w[rp[i]:rp[i + 1]][np.argsort(d2_by_col)]) <= 0)
    assert np.allclose(w[rp[i]:rp[i + 1]], np.exp(-d2_by_col.astype(np.float64) / 0.02) / np.exp(-d2[i].astype(np.float64) / 0.02).sum(), rtol=1e-12)
