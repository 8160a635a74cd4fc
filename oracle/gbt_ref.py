"""Reference of the search's cost model, for tests only (like everything under oracle/).

Least-squares gradient boosting with regression trees and exact greedy splits, written out plainly
(Section 4 of arXiv 2205.13603 names a learned cost model for the evolutionary search and leaves its
form open; the algorithm itself is Friedman's gradient boosting machine, least-squares loss):

    F_0(x) = mean(y);   for t = 1..T:  r_i = y_i - F_{t-1}(x_i);  h_t = tree fitted to r;  F_t = F_{t-1} + lr * h_t

A tree node over rows R with residual sum S and count n is split on the (feature f, threshold c) that
maximises  S_L^2/n_L + S_R^2/n_R - S^2/n  over all midpoints c between consecutive distinct values of
feature f, with both sides holding at least `min_leaf` rows; the first maximum in (feature, value) order
wins, a gain must be positive; rows with x_f < c go left.  A leaf predicts the mean residual of its rows.
Sums run over rows sorted by (x_f, row index), accumulated sequentially in double.
"""
import numpy as np


def _build(X, r, rows, depth, max_depth, min_leaf):
    s = 0.0
    for i in rows:
        s += r[i]
    n = len(rows)
    node = {"value": s / n, "feature": -1}
    if depth >= max_depth or n < 2 * min_leaf:
        return node
    best = (0.0, -1, 0.0)
    for f in range(X.shape[1]):
        order = sorted(rows, key=lambda i: (X[i, f], i))
        sl = 0.0
        for k in range(n - 1):
            sl += r[order[k]]
            xa, xb = X[order[k], f], X[order[k + 1], f]
            if not xa < xb:
                continue
            nl, nr = k + 1, n - k - 1
            if nl < min_leaf or nr < min_leaf:
                continue
            sr = s - sl
            gain = sl * sl / nl + sr * sr / nr - s * s / n
            if gain > best[0]:
                best = (gain, f, 0.5 * (xa + xb))
    if best[1] < 0:
        return node
    _, f, c = best
    left = [i for i in rows if X[i, f] < c]
    right = [i for i in rows if not X[i, f] < c]
    if not left or not right:
        return node
    node.update(feature=f, threshold=c, left=_build(X, r, left, depth + 1, max_depth, min_leaf),
                right=_build(X, r, right, depth + 1, max_depth, min_leaf))
    return node


def _tree_predict(node, x):
    while node["feature"] >= 0:
        node = node["left"] if x[node["feature"]] < node["threshold"] else node["right"]
    return node["value"]


def fit(X, y, n_trees, depth, lr, min_leaf):
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = len(y)
    base = 0.0
    for v in y:
        base += v
    base /= n
    F = np.full(n, base)
    trees = []
    for _ in range(n_trees):
        r = y - F
        tree = _build(X, r, list(range(n)), 0, depth, min_leaf)
        for i in range(n):
            F[i] += lr * _tree_predict(tree, X[i])
        trees.append(tree)
    return {"base": base, "lr": lr, "trees": trees}


def predict(model, X):
    X = np.asarray(X, dtype=np.float64)
    out = np.empty(len(X))
    for i, x in enumerate(X):
        f = model["base"]
        for t in model["trees"]:
            f += model["lr"] * _tree_predict(t, x)
        out[i] = f
    return out
