"""Pins of the deviation-predictor oracle (oracle/forest.py; paper Sec. 3.2.2-3.2.5) against things other
than itself: scikit-learn's regression tree on tie-free data, brute force over every split of a small node,
closed forms, the paper's feature length, hand-computed accuracy and cache traces."""
import itertools

import numpy as np
import pytest

from oracle import forest as orf


def make_data(seed, n, F, M, binary_from=None):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    if binary_from is not None:
        X[:, binary_from:] = (X[:, binary_from:] > 0.3).astype(np.float32)
    W = rng.standard_normal((F, M))
    score = X.astype(np.float64) @ W + 0.5 * rng.standard_normal((n, M))
    Y = np.zeros((n, M), dtype=np.uint8)
    top = np.argsort(-score, axis=1)[:, :2]                  # two active experts per sample
    np.put_along_axis(Y, top, 1, axis=1)
    return X, Y


@pytest.mark.parametrize("seed,depth,min_leaf", [(1, 3, 1), (6, 3, 4), (7, 2, 1), (2, 5, 2), (3, 8, 1), (4, 4, 5), (5, 12, 1)])
def test_tree_matches_sklearn_on_tie_free_data(seed, depth, min_leaf):
    from sklearn.tree import DecisionTreeRegressor
    X, Y = make_data(seed, 240, 7, 5)
    Xt, _ = make_data(seed + 100, 300, 7, 5)
    tree = orf.fit_tree(X, Y, np.arange(240), depth, min_leaf)
    sk = DecisionTreeRegressor(criterion="squared_error", max_depth=depth, min_samples_leaf=min_leaf,
                               max_features=None, random_state=0).fit(X, Y.astype(np.float64))
    np.testing.assert_allclose(orf.predict_tree(tree, X), sk.predict(X), rtol=0, atol=1e-12)
    assert (tree["feature"][0], tree["threshold"][0]) == (sk.tree_.feature[0], sk.tree_.threshold[0])
    # unseen points: only where nodes are large enough that no two features cut a node's samples into the
    # same two sets (such exact ties are broken differently: lowest index here, a random order there)
    if depth <= 3:
        assert (tree["feature"] >= 0).sum() == (sk.tree_.feature >= 0).sum()
        np.testing.assert_allclose(orf.predict_tree(tree, Xt), sk.predict(Xt), rtol=0, atol=1e-12)


def test_forest_is_the_mean_of_trees_grown_on_the_given_bootstrap_samples():
    from sklearn.tree import DecisionTreeRegressor
    X, Y = make_data(11, 200, 6, 4)
    Xt, _ = make_data(12, 100, 6, 4)
    rng = np.random.default_rng(0)
    boot = rng.integers(0, 200, size=(5, 200))
    f = orf.fit_forest(X, Y, boot, max_depth=3, min_leaf=8)
    ref = np.zeros((100, 4))
    for row in boot:
        ref += DecisionTreeRegressor(max_depth=3, min_samples_leaf=8, random_state=0).fit(
            X[row], Y[row].astype(np.float64)).predict(Xt)
    np.testing.assert_allclose(orf.predict_forest(f, Xt), ref / 5, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_root_split_is_the_brute_force_minimum_of_the_squared_error(seed):
    X, Y = make_data(20 + seed, 14, 3, 3, binary_from=2)
    tree = orf.fit_tree(X, Y, np.arange(14), max_depth=1, min_leaf=2)
    Yd = Y.astype(np.float64)

    def sse(mask):
        return sum(((Yd[m] - Yd[m].mean(axis=0)) ** 2).sum() for m in (mask, ~mask))

    best = None
    for f in range(3):
        vals = np.unique(X[:, f])
        for a, b in zip(vals[:-1], vals[1:]):
            thr = 0.5 * (float(a) + float(b))
            mask = X[:, f] <= thr
            if mask.sum() < 2 or (~mask).sum() < 2:
                continue
            cand = (sse(mask), f, thr)
            if best is None or cand[0] < best[0] - 1e-12:
                best = cand
    parent = ((Yd - Yd.mean(axis=0)) ** 2).sum()
    if best is None or not best[0] < parent - 1e-12:
        assert tree["feature"][0] == -1
    else:
        assert (tree["feature"][0], tree["threshold"][0]) == (best[1], best[2])
        mask = X[:, best[1]] <= best[2]
        np.testing.assert_allclose(tree["value"][tree["left"][0]], Yd[mask].mean(axis=0), atol=1e-15)
        np.testing.assert_allclose(tree["value"][tree["right"][0]], Yd[~mask].mean(axis=0), atol=1e-15)


def test_ties_go_to_the_lower_feature_then_the_lower_threshold():
    # features 0 and 1 are copies: the same partition scores the same, feature 0 must win; two thresholds of
    # feature 2 separate the labels equally well (labels 0 0 1 1 0 0 along it), the lower one must win
    X = np.array([[0, 0, 9], [0, 0, 9], [1, 1, 9], [1, 1, 9]], dtype=np.float32)
    Y = np.array([[0], [0], [1], [1]], dtype=np.uint8)
    t = orf.fit_tree(X, Y, np.arange(4), 1)
    assert t["feature"][0] == 0 and t["threshold"][0] == 0.5
    X = np.array([[0], [1], [2], [3], [4], [5]], dtype=np.float32)
    Y = np.array([[0], [0], [1], [1], [0], [0]], dtype=np.uint8)
    t = orf.fit_tree(X, Y, np.arange(6), 1)
    assert t["feature"][0] == 0 and t["threshold"][0] == 1.5


def test_stump_on_a_binary_feature_and_pure_nodes():
    X = np.array([[0.], [1.], [0.], [1.], [1.]], dtype=np.float32)
    Y = np.array([[1, 0], [0, 1], [1, 0], [0, 1], [0, 1]], dtype=np.uint8)
    t = orf.fit_tree(X, Y, np.arange(5), max_depth=4)
    assert len(t["feature"]) == 3 and t["threshold"][0] == 0.5          # children are pure: no further split
    np.testing.assert_array_equal(orf.predict_tree(t, X), Y.astype(np.float64))
    np.testing.assert_array_equal(t["count"], [5, 2, 3])


def test_unlimited_depth_interpolates_distinct_points_and_repetitions_weigh():
    X, Y = make_data(31, 60, 4, 6)
    t = orf.fit_tree(X, Y, np.arange(60), max_depth=64)
    np.testing.assert_array_equal(orf.predict_tree(t, X), Y.astype(np.float64))
    # a sample drawn three times outweighs one drawn once in a shared leaf
    X2 = np.array([[0.], [0.]], dtype=np.float32)
    Y2 = np.array([[1], [0]], dtype=np.uint8)
    t2 = orf.fit_tree(X2, Y2, np.array([0, 0, 0, 1]), max_depth=3)
    assert t2["value"][0, 0] == 0.75 and len(t2["feature"]) == 1


def test_features_follow_the_paper_layout():
    rng = np.random.default_rng(5)
    V, d, L, M = 50, 8, 4, 6
    table = rng.standard_normal((V, d)).astype(np.float32)
    toks = [3, 17, 3, 44, 9]
    actual = (rng.random((L, M)) < 0.3).astype(np.uint8)
    X, Y = orf.examples_of_request(table, toks, S=2, actual=actual)
    assert X.shape == (L, d + 2 + L * M) and Y.shape == (L, M)            # F = d + 2 + L*M, one example per layer
    np.testing.assert_allclose(X[0, :d], table[toks].astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
    for l in range(L):
        assert X[l, d] == 2 and X[l, d + 1] == l
        prev = X[l, d + 2:].reshape(L, M)
        np.testing.assert_array_equal(prev[:l], actual[:l])
        assert not prev[l:].any()
        np.testing.assert_array_equal(Y[l], actual[l])
    X2, _ = orf.examples_of_request(table, toks, S=2, actual=actual, lag=2)
    for l in range(L):
        prev = X2[l, d + 2:].reshape(L, M)
        np.testing.assert_array_equal(prev[:max(0, l - 2)], actual[:max(0, l - 2)])
        assert not prev[max(0, l - 2):].any()


def test_bit_accuracy_and_delta_mapping():
    yhat = np.array([[0.9, 0.5, 0.49, 0.0], [0.2, 0.8, 0.6, 0.1]])
    y = np.array([[1, 0, 0, 0], [0, 1, 0, 1]])
    assert orf.bit_accuracy(yhat, y) == 5 / 8                            # wrong: (0,1), (1,2), (1,3)
    rng = np.random.default_rng(2)
    z = rng.standard_normal((10, 8))
    p = rng.random((10, 8))
    dl = orf.delta_from_activation(p, 3.0)
    np.testing.assert_allclose(dl.sum(axis=-1), 0, atol=1e-5)
    np.testing.assert_array_equal(np.argsort(-(z + dl), axis=1)[:, :2], np.argsort(-(z + 3.0 * p), axis=1)[:, :2])
    assert not orf.delta_from_activation(np.full((2, 4), 0.25), 5.0).any()


def test_prediction_cache_trace():
    c = orf.PredictionCache(capacity=2)
    assert c.get([1, 2], 0, 1) is None
    c.put([1, 2], 0, 1, [0.1]); c.put([1, 2], 1, 1, [0.2])
    assert c.get([1, 2], 0, 1)[0] == np.float32(0.1)                      # refreshes (tokens, 0, 1)
    c.put([1, 2], 0, 2, [0.3])                                            # evicts (tokens, 1, 1)
    assert c.get([1, 2], 1, 1) is None and c.get([1, 2], 0, 2) is not None and c.get([2, 1], 0, 2) is None
    assert (c.hits, c.misses) == (2, 3)
