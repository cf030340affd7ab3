"""The library's deviation predictor (host code of libexpertflow.so; paper Sec. 3.2.2-3.2.5) against the CPU
oracle: identical trees (integer decisions exact, thresholds and leaf means bit-equal), identical features,
predictions to 1e-15, the same cache behaviour, and the asynchronous producer end to end.  No GPU is needed."""
import os

import numpy as np
import pytest

from paper_2510_26730_amd import binding as ef
from oracle import forest as orf


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(ef.LIB_PATH):
        from paper_2510_26730_amd import build
        build.build()
    return ef.lib()


def activation_logs(seed, n_req, L, M, k, V, d_emb, n_tok):
    """Synthetic activation logs with learnable structure: a request's experts in layer l are the top-k of a
    seeded score of (its tokens' embedding, l) plus what it activated in layer l-1 plus noise."""
    rng = np.random.default_rng(seed)
    table = rng.standard_normal((V, d_emb)).astype(np.float32)
    proj = rng.standard_normal((L, d_emb, M))
    carry = rng.standard_normal((M, M)) * 0.5
    reqs = []
    for _ in range(n_req):
        toks = rng.integers(0, V, size=n_tok).astype(np.int32)
        e = table[toks].astype(np.float64).mean(axis=0)
        actual = np.zeros((L, M), dtype=np.uint8)
        for l in range(L):
            sc = e @ proj[l] * 3.0 + (actual[l - 1] @ carry if l else 0.0) + 0.3 * rng.standard_normal(M)
            actual[l, np.argsort(-sc)[:k]] = 1
        reqs.append((toks, actual))
    return table, reqs


def dataset(table, reqs, S):
    Xs, Ys = zip(*(orf.examples_of_request(table, t, S, a) for t, a in reqs))
    return np.concatenate(Xs), np.concatenate(Ys)


@pytest.mark.parametrize("seed,L,M,k,depth,min_leaf,n_trees", [(1, 4, 8, 2, 6, 1, 3), (2, 3, 16, 4, 4, 3, 2),
                                                               (3, 6, 6, 1, 10, 1, 2), (4, 2, 64, 6, 5, 2, 2)])
def test_trees_and_predictions_equal_the_oracle(seed, L, M, k, depth, min_leaf, n_trees):
    table, reqs_all = activation_logs(seed, 55, L, M, k, V=30, d_emb=5, n_tok=4)
    reqs, reqs2 = reqs_all[:40], reqs_all[40:]
    X, Y = dataset(table, reqs, S=2)
    N = X.shape[0]
    boot = np.random.default_rng(seed).integers(0, N, size=(n_trees, N)).astype(np.int32)
    f = ef.ef_forest_create(X.shape[1], M, n_trees, depth, min_leaf, n_threads=3)
    try:
        ef.ef_forest_fit(f, X, Y, boot)
        ref = orf.fit_forest(X, Y, boot, depth, min_leaf)
        for t in range(n_trees):
            got = ef.ef_forest_tree_export(f, t, M)
            for key in ("feature", "left", "right", "count", "threshold", "value"):
                np.testing.assert_array_equal(got[key], ref[t][key], err_msg=f"tree {t} {key}")
        X2, Y2 = dataset(table, reqs2, S=2)
        p, q = ef.ef_forest_predict(f, X2, M), orf.predict_forest(ref, X2)
        np.testing.assert_allclose(p, q, rtol=0, atol=1e-15)
        assert ef.ef_forest_bit_accuracy(p, Y2) == orf.bit_accuracy(q, Y2)
    finally:
        ef.ef_forest_destroy(f)


def test_fit_without_bootstrap_and_thread_count_do_not_matter():
    table, reqs = activation_logs(7, 30, 3, 8, 2, V=20, d_emb=4, n_tok=3)
    X, Y = dataset(table, reqs, S=1)
    trees = []
    for nt in (1, 4):
        f = ef.ef_forest_create(X.shape[1], 8, 2, 5, 1, n_threads=nt)
        ef.ef_forest_fit(f, X, Y, None)
        trees.append([ef.ef_forest_tree_export(f, t, 8) for t in range(2)])
        ef.ef_forest_destroy(f)
    ref = orf.fit_tree(X, Y, np.arange(X.shape[0]), 5, 1)
    for run in trees:
        for tr in run:
            for key in ref:
                np.testing.assert_array_equal(tr[key], ref[key])


def test_features_are_bit_equal():
    rng = np.random.default_rng(3)
    V, d, L, M = 100, 16, 5, 8
    table = (rng.standard_normal((V, d)) * 3).astype(np.float32)
    for n_tok in (1, 2, 7, 33):
        toks = rng.integers(0, V, size=n_tok)
        prev = (rng.random((L, M)) < 0.25).astype(np.uint8)
        for layer in (0, 2, 4):
            x = ef.ef_delta_features(table, toks, 3, layer, prev, L, M)
            ref = orf.feature_vector(orf.pooled_embedding(table, toks), 3, layer, prev)
            np.testing.assert_array_equal(x.view(np.uint32), ref.view(np.uint32))


def test_delta_mapping_equals_the_oracle():
    rng = np.random.default_rng(4)
    y = rng.random((3, 5, 8))
    for gain in (0.0, 1.0, 0.1, 7.5):
        np.testing.assert_array_equal(ef.ef_delta_from_activation(y, gain), orf.delta_from_activation(y, gain))


def test_cache_follows_the_model_on_a_random_trace():
    rng = np.random.default_rng(5)
    M = 4
    c = ef.ef_delta_cache_create(6, M)
    model = orf.PredictionCache(6)
    seqs = [rng.integers(0, 9, size=rng.integers(1, 4)).astype(np.int32) for _ in range(5)]
    try:
        for _ in range(400):
            toks = seqs[rng.integers(0, 5)]
            layer, S = int(rng.integers(0, 3)), int(rng.integers(1, 3))
            if rng.random() < 0.45:
                y = rng.random(M)
                ef.ef_delta_cache_put(c, toks, layer, S, y)
                model.put(toks, layer, S, y)
            else:
                got, want = ef.ef_delta_cache_get(c, toks, layer, S, M), model.get(toks, layer, S)
                assert (got is None) == (want is None)
                if got is not None:
                    np.testing.assert_array_equal(got.astype(np.float32), want)
        hits, misses, entries = ef.ef_delta_cache_counts(c)
        assert (hits, misses, entries) == (model.hits, model.misses, len(model.d))
    finally:
        ef.ef_delta_cache_destroy(c)


def test_producer_fills_the_cache_and_assemble_builds_delta():
    L, M, k, d_emb, V = 5, 8, 2, 6, 40
    table, reqs = activation_logs(9, 60, L, M, k, V, d_emb, n_tok=5)
    X, Y = dataset(table, reqs, S=2)
    boot = np.random.default_rng(1).integers(0, X.shape[0], size=(4, X.shape[0])).astype(np.int32)
    f = ef.ef_forest_create(X.shape[1], M, 4, 6, 2, n_threads=2)
    ef.ef_forest_fit(f, X, Y, boot)
    ref = orf.fit_forest(X, Y, boot, 6, 2)
    cache = ef.ef_delta_cache_create(1000, M)
    prod = ef.ef_delta_producer_create(f, cache, table, L, M, n_threads=3)
    try:
        layer, H, S, gain = 1, 3, 2, 2.5
        live = reqs[:7]
        for toks, actual in live:
            prev = np.zeros((L, M), dtype=np.uint8)
            prev[:layer + 1] = actual[:layer + 1]                  # what the request has activated so far
            ef.ef_delta_submit(prod, toks, S, layer + 1, H, prev)
            ef.ef_delta_submit(prod, toks, S, layer + 1, H, prev)  # a second submission finds them queued or cached
        ef.ef_delta_drain(prod)
        _, _, entries = ef.ef_delta_cache_counts(cache)
        assert entries == 7 * H
        toks_all = np.concatenate([t for t, _ in live] + [np.array([1, 2, 3], dtype=np.int32)])
        off = np.concatenate([[0], np.cumsum([len(t) for t, _ in live] + [3])]).astype(np.int32)
        delta, hits = ef.ef_delta_assemble(cache, toks_all, off, layer, S, H, L, gain, M)
        assert delta.shape == (8, H, M) and hits == 7 * H
        assert not delta[7].any()                                    # unknown request: plain top-k fallback
        for r, (toks, actual) in enumerate(live):
            prev = np.zeros((L, M), dtype=np.uint8)
            prev[:layer + 1] = actual[:layer + 1]
            e = orf.pooled_embedding(table, toks)
            for j in range(H):
                t = layer + 1 + j
                masked = prev.copy()
                masked[max(0, t - S):] = 0                       # rows of layers >= t - S are not known S ahead
                x = orf.feature_vector(e, S, t, masked)
                want = orf.delta_from_activation(orf.predict_forest(ref, x[None])[0], gain)
                np.testing.assert_allclose(delta[r, j], want, rtol=0, atol=1e-6)
        # look-ahead past the last layer gives zero rows
        d2, h2 = ef.ef_delta_assemble(cache, toks_all, off, L - 2, S, H, L, gain, M)
        assert not d2[:, 1:].any()
    finally:
        ef.ef_delta_producer_destroy(prod)
        ef.ef_delta_cache_destroy(cache)
        ef.ef_forest_destroy(f)


def test_argument_errors():
    with pytest.raises(ef.EfError):
        ef.ef_forest_create(0, 8, 1, 3)
    with pytest.raises(ef.EfError):
        ef.ef_forest_create(4, 65, 1, 3)
    f = ef.ef_forest_create(4, 2, 1, 3)
    try:
        X = np.zeros((5, 4), dtype=np.float32)
        Y = np.zeros((5, 2), dtype=np.uint8)
        with pytest.raises(ef.EfError):
            ef.ef_forest_predict(f, X, 2)                           # before a fit
        with pytest.raises(ef.EfError):
            ef.ef_forest_fit(f, X, Y, np.full((1, 5), 5, dtype=np.int32))   # index out of range
        Xn = X.copy(); Xn[2, 1] = np.nan
        with pytest.raises(ef.EfError):
            ef.ef_forest_fit(f, Xn, Y, None)
        ef.ef_forest_fit(f, X, Y, None)
        assert ef.ef_forest_tree_size(f, 0) == 1                    # constant features: a single leaf
        with pytest.raises(ef.EfError):
            ef.ef_forest_tree_size(f, 1)
    finally:
        ef.ef_forest_destroy(f)
    with pytest.raises(ef.EfError):
        ef.ef_delta_features(np.zeros((3, 2), np.float32), [3], 1, 0, np.zeros(4, np.uint8), 2, 2)   # token id out of range
