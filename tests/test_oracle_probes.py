"""Pins for the oracle's cost matrix from probes (Section 4.2: 10th-percentile RTT per ordered pair, then
c[a][b] <- max(c[a][b], c[b][a])): numpy's nearest-rank percentile, hand-worked samples, order invariance."""
import numpy as np
import pytest

import oracle
from gen import clean_hierarchy, probe_samples


def test_hand_worked():
    # N = 2, K = 10: the 10th percentile by nearest rank is the smallest sample, the 20th the second smallest
    s = np.zeros((2, 2, 10), dtype=np.int32)
    s[0, 1] = [50, 40, 90, 41, 45, 300, 42, 47, 43, 44]
    s[1, 0] = [61, 60, 65, 64, 63, 62, 900, 66, 67, 68]
    assert oracle.cost_matrix_from_probes(s, 10, False).tolist() == [[0, 40], [60, 0]]
    assert oracle.cost_matrix_from_probes(s, 20, False).tolist() == [[0, 41], [61, 0]]
    assert oracle.cost_matrix_from_probes(s, 11, False).tolist() == [[0, 41], [61, 0]]     # ceil(1.1) = 2
    assert oracle.cost_matrix_from_probes(s, 100, False).tolist() == [[0, 300], [900, 0]]
    assert oracle.cost_matrix_from_probes(s, 0, False).tolist() == [[0, 40], [60, 0]]      # rank at least 1
    assert oracle.cost_matrix_from_probes(s, 10, True).tolist() == [[0, 60], [60, 0]]      # larger direction wins
    assert oracle.cost_matrix_from_probes(s, 50, True).tolist() == [[0, 64], [64, 0]]


@pytest.mark.parametrize("n,k,q", [(5, 1, 10), (6, 7, 10), (8, 100, 10), (8, 100, 50), (4, 1000, 10), (7, 333, 90),
                                   (3, 4096, 25), (9, 10, 100)])
def test_against_numpy_nearest_rank_percentile(n, k, q):
    rng = np.random.default_rng(n * 1000 + k)
    s = rng.integers(0, 5000, size=(n, n, k)).astype(np.int32)
    want = np.percentile(s, q, axis=2, method="inverted_cdf").astype(np.int64)
    np.fill_diagonal(want, 0)
    got = oracle.cost_matrix_from_probes(s, q, False)
    assert np.array_equal(got, want)
    sym = oracle.cost_matrix_from_probes(s, q, True)
    assert np.array_equal(sym, np.maximum(want, want.T)) and np.array_equal(sym, sym.T)


def test_sample_order_does_not_matter_and_values_are_limited():
    rng = np.random.default_rng(5)
    s = rng.integers(0, 100000, size=(6, 6, 50)).astype(np.int32)
    shuffled = rng.permuted(s, axis=2)
    assert np.array_equal(oracle.cost_matrix_from_probes(s, 10, True), oracle.cost_matrix_from_probes(shuffled, 10, True))
    s[1, 2, :] = -7
    s[2, 1, :] = 1 << 30
    out = oracle.cost_matrix_from_probes(s, 10, False)
    assert out[1, 2] == 0 and out[2, 1] == (1 << 21) - 1


def test_recovers_the_base_matrix_through_interference():
    """The generator inflates 20 % of the samples heavily; the 10th percentile stays within a few percent of the
    base RTT, the mean does not (the reason Section 4.2 gives for the percentile)."""
    base = clean_hierarchy(16, 4, 300, 1500)
    s = probe_samples(base, 400, seed=11)
    c = oracle.cost_matrix_from_probes(s, 10, True)
    off = ~np.eye(16, dtype=bool)
    rel = c[off] / base[off]
    assert rel.min() >= 1.0 and rel.max() < 1.05
    assert (s.mean(axis=2)[off] / base[off]).min() > 1.2
