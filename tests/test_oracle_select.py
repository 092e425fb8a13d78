"""Pins of oracle.select (CPU only): the K distance of Sec. 4.2 and the ranking built on it."""
import numpy as np

from oracle import k_distance, top_counts, top_tokens


def test_k_distance_matches_loops_and_closed_forms():
    rng = np.random.default_rng(5)
    a, b, c = (rng.standard_normal((6, 2, 4)) for _ in range(3))
    d = k_distance(a, b)
    for t in range(6):
        acc = 0.0
        for h in range(2):
            for i in range(4):
                acc += abs(a[t][h][i] - b[t][h][i])
        assert abs(d[t] - acc) < 1e-12
    assert np.array_equal(k_distance(a, a), np.zeros(6))
    np.testing.assert_allclose(k_distance(a, a + 0.25), np.full(6, 0.25 * 8), rtol=1e-12)
    np.testing.assert_allclose(k_distance(a, b), k_distance(b, a), rtol=0, atol=0)          # symmetric
    assert (k_distance(a, c) <= k_distance(a, b) + k_distance(b, c) + 1e-12).all()          # triangle
    np.testing.assert_allclose(k_distance(3 * a, 3 * b), 3 * d, rtol=1e-12)                 # homogeneous


def test_ranking_by_hand():
    dist = [0.5, 4.0, 1.0, 4.0, 0.0, 2.5]
    assert top_tokens(dist, 1).tolist() == [1]            # tie 1 / 3: the lower index ranks first
    assert top_tokens(dist, 2).tolist() == [1, 3]
    assert top_tokens(dist, 3).tolist() == [1, 3, 5]
    assert top_tokens(dist, 4).tolist() == [1, 2, 3, 5]
    assert top_tokens(dist, 0).tolist() == [] and top_tokens(dist, 99).tolist() == [0, 1, 2, 3, 4, 5]
    layers = [dist, [9, 0, 0, 0, 0, 8], [0, 0, 7, 0, 0, 6]]
    assert top_counts(layers, 2).tolist() == [1, 1, 1, 1, 0, 2]
    assert top_counts(layers, 2).sum() == 3 * 2
