"""CPU oracle (test infrastructure only) of the deviation predictor of Sec. 3.2.2-3.2.5.

The paper trains a random-forest regressor on activation logs: one example per (request, layer), features
x = [e, S, l, prev_act] (Sec. 3.2.4: e the mean of a fixed random embedding of the request's token ids,
S the step size, l the layer index, prev_act in {0,1}^(L*M) the experts the request activated in the
layers before l), label y in {0,1}^M (the experts it activated in layer l), squared-error criterion
(Sec. 3.2.5), accuracy = share of correctly predicted expert bits.  Its output refines the pre-gate
prediction of future layers (Sec. 3.2.2), and predictions are cached by (token sequence, layer, S).

Everything here is plain numpy / Python written from that description:

* ``pooled_embedding``, ``feature_vector``, ``examples_of_request``: Sec. 3.2.3-3.2.4.
* ``fit_tree`` / ``predict_tree``: a regression tree with the squared-error criterion over all M outputs,
  all features considered at every node (the regressor default of the library the paper names), grown to
  ``max_depth`` with at least ``min_leaf`` samples per leaf.  Labels are 0/1, so the criterion is a ratio
  of integers and the best split is decided in exact integer arithmetic: maximise
  sum_m sL[m]^2 / nL + sum_m sR[m]^2 / nR (equivalent to minimising the summed squared error); ties go to
  the lower feature index, then the lower threshold; a node is split only if that strictly beats
  sum_m s[m]^2 / n.  Threshold = midpoint of the two neighbouring feature values in fp64, x <= thr goes left.
* ``fit_forest`` / ``predict_forest``: one tree per row of the bootstrap index matrix (the random draws
  are inputs), prediction = mean over the trees, summed in tree order.
* ``bit_accuracy``: Sec. 3.2.5.  ``delta_from_activation``: the reading that turns the predicted activation
  vector into the logit-domain deviation (gain times the centred prediction; parity unpinned: the paper
  does not give the mapping).  ``PredictionCache``: Sec. 3.2.2's cache, least recently used beyond a capacity.

Pins (tests/test_forest_oracle.py): scikit-learn's DecisionTreeRegressor on tie-free data (same
predictions), brute force over every (feature, threshold) on small nodes, closed forms (a stump on one
binary feature, interpolation of distinct training points at unlimited depth), the feature length
d + 2 + L*M of Sec. 3.2.5, and hand-computed accuracy / cache traces.
"""
from __future__ import annotations

from collections import OrderedDict

import numpy as np


# ----------------------------------------------------------------------------- features (Sec. 3.2.4)

def pooled_embedding(table: np.ndarray, token_ids) -> np.ndarray:
    """e = (1/k) sum_i E[t_i]: rows summed in sequence order in fp64, divided, rounded to float32."""
    table = np.asarray(table, dtype=np.float32)
    acc = np.zeros(table.shape[1], dtype=np.float64)
    for t in token_ids:
        acc = acc + table[int(t)].astype(np.float64)
    return (acc / float(len(token_ids))).astype(np.float32)


def feature_vector(e: np.ndarray, S: int, layer: int, prev_act: np.ndarray) -> np.ndarray:
    """x = [e, S, l, prev_act] as float32, length d + 2 + L*M."""
    return np.concatenate([np.asarray(e, dtype=np.float32), np.array([S, layer], dtype=np.float32),
                           np.asarray(prev_act, dtype=np.float32).reshape(-1)])


def examples_of_request(table, token_ids, S: int, actual: np.ndarray, lag: int = 0):
    """One (x, y) per layer of one request, layers ascending.  actual [L, M] in {0,1}: the experts the
    request activated in each layer.  prev_act of layer l holds the rows of the layers before l - lag, zeros
    from there on: lag = 0 is the paper's "all previous layers"; lag = S keeps what is known when layer l is
    predicted S layers ahead (the rule the producer applies at run time)."""
    actual = np.asarray(actual, dtype=np.uint8)
    L, M = actual.shape
    e = pooled_embedding(table, token_ids)
    X, Y = [], []
    for l in range(L):
        prev = np.zeros((L, M), dtype=np.uint8)
        known = max(0, l - lag)
        prev[:known] = actual[:known]
        X.append(feature_vector(e, S, l, prev))
        Y.append(actual[l].copy())
    return np.stack(X), np.stack(Y)


# ----------------------------------------------------------------------------- one tree

def _best_split_of_feature(xs: np.ndarray, ys: np.ndarray, min_leaf: int):
    """Best split of one feature over the node's samples (xs float32 [n], ys uint8 [n, M]).
    Returns (QL*nR + QR*nL, nL*nR, thr) as Python ints + float, or None."""
    n = xs.shape[0]
    order = np.argsort(xs, kind="stable")
    xv = xs[order]
    if xv[0] == xv[-1]:
        return None
    yc = np.cumsum(ys[order].astype(np.int64), axis=0)            # sL after each prefix
    tot = yc[-1]
    nl = np.arange(1, n, dtype=np.int64)                            # split after position i-1
    ok = (xv[1:] != xv[:-1]) & (nl >= min_leaf) & (n - nl >= min_leaf)
    if not ok.any():
        return None
    sl = yc[:-1]
    ql = (sl * sl).sum(axis=1)
    qr = ((tot - sl) * (tot - sl)).sum(axis=1)
    nr = n - nl
    cand = np.nonzero(ok)[0]
    approx = ql[cand] / nl[cand] + qr[cand] / nr[cand]
    near = cand[approx >= approx.max() * (1.0 - 1e-9)]              # fp64 prefilter, exact decision below
    best = None
    for i in near:                                                  # ascending threshold
        num = int(ql[i]) * int(nr[i]) + int(qr[i]) * int(nl[i])
        den = int(nl[i]) * int(nr[i])
        if best is None or num * best[1] > best[0] * den:
            best = (num, den, 0.5 * (float(xv[i]) + float(xv[i + 1])))
    return best


def fit_tree(X: np.ndarray, Y: np.ndarray, idx: np.ndarray, max_depth: int, min_leaf: int = 1) -> dict:
    """Grow one tree on the samples idx (with repetitions).  Returns arrays in node order (a node's
    children are created left first, depth first): feature (-1 = leaf), threshold, left, right,
    value [nodes, M] (mean label of the node's samples), count."""
    X = np.asarray(X, dtype=np.float32)
    Y = np.asarray(Y, dtype=np.uint8)
    nodes = {"feature": [], "threshold": [], "left": [], "right": [], "value": [], "count": []}

    def grow(ids: np.ndarray, depth: int) -> int:
        me = len(nodes["feature"])
        ys = Y[ids]
        s = ys.astype(np.int64).sum(axis=0)
        n = ids.shape[0]
        for k, v in (("feature", -1), ("threshold", 0.0), ("left", -1), ("right", -1),
                     ("value", s.astype(np.float64) / float(n)), ("count", n)):
            nodes[k].append(v)
        if depth >= max_depth or n < 2 * min_leaf:
            return me
        best = None                                                  # (num, den, thr, feature)
        for f in range(X.shape[1]):
            r = _best_split_of_feature(X[ids, f], ys, min_leaf)
            if r is not None and (best is None or r[0] * best[1] > best[0] * r[1]):
                best = (r[0], r[1], r[2], f)
        if best is None or not (best[0] * n > int((s * s).sum()) * best[1]):
            return me
        go_left = X[ids, best[3]].astype(np.float64) <= best[2]
        nodes["feature"][me], nodes["threshold"][me] = best[3], best[2]
        nodes["left"][me] = grow(ids[go_left], depth + 1)
        nodes["right"][me] = grow(ids[~go_left], depth + 1)
        return me

    grow(np.asarray(idx, dtype=np.int64), 0)
    return {"feature": np.array(nodes["feature"], dtype=np.int32),
            "threshold": np.array(nodes["threshold"], dtype=np.float64),
            "left": np.array(nodes["left"], dtype=np.int32), "right": np.array(nodes["right"], dtype=np.int32),
            "value": np.stack(nodes["value"]), "count": np.array(nodes["count"], dtype=np.int32)}


def predict_tree(tree: dict, X: np.ndarray) -> np.ndarray:
    X = np.asarray(X, dtype=np.float32)
    out = np.empty((X.shape[0], tree["value"].shape[1]), dtype=np.float64)
    for i in range(X.shape[0]):
        nd = 0
        while tree["feature"][nd] >= 0:
            nd = tree["left"][nd] if float(X[i, tree["feature"][nd]]) <= tree["threshold"][nd] else tree["right"][nd]
        out[i] = tree["value"][nd]
    return out


# ----------------------------------------------------------------------------- the forest

def fit_forest(X, Y, bootstrap: np.ndarray, max_depth: int, min_leaf: int = 1) -> list:
    """bootstrap [n_trees, n] int: the sample indices (with repetitions) each tree is grown on."""
    return [fit_tree(X, Y, row, max_depth, min_leaf) for row in np.asarray(bootstrap)]


def predict_forest(forest: list, X) -> np.ndarray:
    acc = None
    for tree in forest:                                              # tree order
        p = predict_tree(tree, X)
        acc = p if acc is None else acc + p
    return acc / float(len(forest))


def bit_accuracy(yhat: np.ndarray, y: np.ndarray) -> float:
    """Share of expert bits predicted correctly; a bit is predicted set when yhat >= 0.5 (Sec. 3.2.5)."""
    return float(((np.asarray(yhat) >= 0.5) == (np.asarray(y) != 0)).mean())


def delta_from_activation(yhat: np.ndarray, gain: float) -> np.ndarray:
    """Delta[..., e] = gain * (yhat[..., e] - mean_e yhat): float32, fp64 inside, mean summed in expert order;
    the gain is a float32 parameter."""
    gain = float(np.float32(gain))
    yhat = np.asarray(yhat, dtype=np.float64)
    mean = np.zeros(yhat.shape[:-1], dtype=np.float64)
    for e in range(yhat.shape[-1]):
        mean = mean + yhat[..., e]
    mean = mean / float(yhat.shape[-1])
    return (gain * (yhat - mean[..., None])).astype(np.float32)


# ----------------------------------------------------------------------------- prediction cache (Sec. 3.2.2)

class PredictionCache:
    """Keyed by (token sequence, layer, step size); least recently used entry leaves beyond `capacity`.
    A hit refreshes the entry."""

    def __init__(self, capacity: int):
        self.capacity = capacity
        self.d: OrderedDict = OrderedDict()
        self.hits = self.misses = 0

    def put(self, token_ids, layer: int, S: int, value) -> None:
        key = (tuple(int(t) for t in token_ids), int(layer), int(S))
        self.d[key] = np.array(value, dtype=np.float32)
        self.d.move_to_end(key)
        while len(self.d) > self.capacity:
            self.d.popitem(last=False)

    def get(self, token_ids, layer: int, S: int):
        key = (tuple(int(t) for t in token_ids), int(layer), int(S))
        if key in self.d:
            self.d.move_to_end(key)
            self.hits += 1
            return self.d[key]
        self.misses += 1
        return None
