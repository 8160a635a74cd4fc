"""Learned cost model of the search (Section 4, "End-to-end search"): the library's boosted trees against a plain
reference, the reference against closed forms and an independent library, and the model-guided search on a synthetic
latency.  CPU only."""
import math

import numpy as np
import pytest

from oracle import gbt_ref
from paper_2205_13603_amd import binding as B
from test_search import synthetic_latency


# ---------------------------------------------------------------- the reference, pinned to what mathematics fixes

def test_reference_zero_trees_predicts_the_mean():
    X = np.arange(12.0).reshape(6, 2)
    y = np.array([1.0, 2.0, 4.0, 8.0, 16.0, 32.0])
    m = gbt_ref.fit(X, y, n_trees=0, depth=3, lr=0.5, min_leaf=1)
    assert np.array_equal(gbt_ref.predict(m, X), np.full(6, 10.5))


def test_reference_one_stump_recovers_a_step_exactly():
    """y = 3 for x0 < 4.5, 11 otherwise; x1 is noise.  One depth-1 tree with learning rate 1: threshold at the
    midpoint 4.5 of the two neighbouring values, leaves at the class means, predictions exact."""
    X = np.array([[0, 5], [1, 3], [2, 9], [4, 1], [5, 7], [6, 2], [8, 8], [9, 4]], dtype=float)
    y = np.where(X[:, 0] < 4.5, 3.0, 11.0)
    m = gbt_ref.fit(X, y, n_trees=1, depth=1, lr=1.0, min_leaf=1)
    t = m["trees"][0]
    assert t["feature"] == 0 and t["threshold"] == 4.5
    assert t["left"]["value"] == 3.0 - 7.0 and t["right"]["value"] == 11.0 - 7.0
    assert np.array_equal(gbt_ref.predict(m, X), y)
    # min_leaf larger than the smaller side forbids that split; with min_leaf = 5 no split exists at all
    m5 = gbt_ref.fit(X, y, n_trees=1, depth=1, lr=1.0, min_leaf=5)
    assert m5["trees"][0]["feature"] == -1


def test_reference_training_error_never_increases_and_interpolates():
    g = np.random.default_rng(0)
    X = g.integers(0, 16, size=(120, 5)).astype(float)
    y = np.sin(X[:, 0]) + 0.1 * X[:, 1] * X[:, 2] + g.normal(0, 0.01, 120)
    errs = []
    for T in (0, 1, 2, 4, 8, 16, 32):
        m = gbt_ref.fit(X, y, n_trees=T, depth=3, lr=0.5, min_leaf=1)
        errs.append(float(np.mean((gbt_ref.predict(m, X) - y) ** 2)))
    assert all(a >= b - 1e-15 for a, b in zip(errs, errs[1:])), errs
    assert errs[-1] < 0.05 * errs[0]


def test_reference_agrees_with_an_independent_library():
    """scikit-learn's GradientBoostingRegressor with squared-error splits is the same algorithm (mean start, exact
    greedy midpoint splits, shrinkage).  Features are small multiples of 1/8 so that its float32 copies are exact."""
    ske = pytest.importorskip("sklearn.ensemble")
    g = np.random.default_rng(1)
    X = g.integers(0, 64, size=(150, 4)) / 8.0
    y = g.normal(0, 1, 150) + X[:, 0] - 0.5 * X[:, 3]
    for depth, lr, leaf, T in ((1, 1.0, 1, 5), (3, 0.3, 2, 20), (4, 0.1, 5, 30)):
        sk = ske.GradientBoostingRegressor(loss="squared_error", criterion="squared_error", n_estimators=T, learning_rate=lr,
                                           max_depth=depth, min_samples_leaf=leaf, subsample=1.0, random_state=0).fit(X, y)
        ref = gbt_ref.predict(gbt_ref.fit(X, y, n_trees=T, depth=depth, lr=lr, min_leaf=leaf), X)
        assert np.max(np.abs(ref - sk.predict(X))) < 1e-9, (depth, lr, leaf, T)


# ---------------------------------------------------------------- the library against the reference

@pytest.mark.parametrize("case", ["continuous", "ties", "variants"])
def test_library_model_matches_reference(case):
    g = np.random.default_rng(7)
    if case == "continuous":
        X = g.normal(0, 1, size=(200, 6))
        y = X[:, 0] * X[:, 1] + np.abs(X[:, 2]) + g.normal(0, 0.1, 200)
    elif case == "ties":
        X = g.integers(0, 4, size=(160, 5)).astype(float)      # many equal feature values
        y = (X[:, 0] > 1) * 2.0 + (X[:, 1] == 3) * 1.5 + g.integers(0, 3, 160)
    else:
        op = B.gemm_op(1024, 1024, 1024, "f16")
        sp = op.space()
        rows = [B.variant_features(op, B.trace_validate(op, sp, B.trace_sample_valid(op, sp, 5, i))) for i in range(120)]
        X = np.stack(rows)
        y = 0.5 * X[:, 16] + np.abs(X[:, 18] - 8) + 0.1 * X[:, 24]
    Xq = X[::3] + (0.0 if case == "ties" else 1e-3)
    for T, depth, lr, leaf in ((1, 1, 1.0, 1), (25, 3, 0.3, 2), (40, 4, 0.2, 3)):
        m = B.CostModel(T, depth, lr, leaf)
        m.fit(X, y)
        ref = gbt_ref.fit(X, y, n_trees=T, depth=depth, lr=lr, min_leaf=leaf)
        for Z in (X, Xq):
            got, want = m.predict(Z), gbt_ref.predict(ref, Z)
            assert np.max(np.abs(got - want)) <= 1e-12 * max(1.0, np.max(np.abs(want))), (case, T, depth)


def test_library_model_argument_errors():
    m = B.CostModel(5, 2, 0.5, 1)
    with pytest.raises(B.MsError):
        m.predict(np.zeros((2, 3)))                      # not fitted
    m.fit(np.arange(12.0).reshape(4, 3), np.arange(4.0))
    with pytest.raises(B.MsError):
        m.predict(np.zeros((2, 4)))                      # other feature count
    with pytest.raises(B.MsError):
        m.fit(np.array([[np.nan, 0.0]]), np.array([1.0]))
    with pytest.raises(B.MsError):
        B.CostModel(5, 0, 0.5, 1)


def test_features_are_finite_and_distinguish_variants():
    for mk in (lambda: B.gemm_op(128, 128, 128, "f32"), lambda: B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1),
               lambda: B.dwconv2d_op(1, 112, 112, 32)):
        op = mk()
        sp = op.space()
        seen = {}
        for i in range(60):
            p = B.trace_validate(op, sp, B.trace_sample_valid(op, sp, 2, i))
            f = B.variant_features(op, p)
            assert np.all(np.isfinite(f)) and len(f) == len(B.variant_features(op, p))
            seen.setdefault(p.key, f)
            assert np.array_equal(seen[p.key], f)
        vecs = {tuple(v) for v in seen.values()}
        assert len(vecs) > 0.9 * len(seen)                # different kernels almost always differ in some feature


# ---------------------------------------------------------------- the search with the model

def _run(seed, trials, model):
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space()
    cfg = B.search_cfg_default()
    cfg.seed, cfg.trials, cfg.cost_model = seed, trials, model
    log = []
    res = B.search(op, sp, cfg, fake_latency=synthetic_latency, on_trial=lambda t: log.append((t.status, t.us, bytes(t.trace))) and 0)
    return res, log


def test_model_guided_search_on_the_synthetic_latency():
    """Same budget of measured candidates, eight seeds.  What the model does: once it is in use (after
    model_min_trials measurements) the candidates it lets through are better than the plain search's proposals
    (median latency of the measured candidates, summed over the seeds).  It is not required to find a better
    variant or to need fewer measurements: on this function it reaches the optimum on about half of the seeds
    (the plain search on six of eight), and on the GPU workloads it showed no gain either; the bounds below only
    guard against the guided search falling far behind."""
    plain, guided, med_plain, med_guided = [], [], 0.0, 0.0
    for seed in range(8):
        r0, l0 = _run(seed, 192, 0)
        r1, l1 = _run(seed, 192, 1)
        assert r1.n_measured == 192
        plain.append(r0.best_us)
        guided.append(r1.best_us)
        med_plain += float(np.median([u for st, u, _ in l0[48:] if st == 0]))
        med_guided += float(np.median([u for st, u, _ in l1[48:] if st == 0]))
    print("plain ", plain, med_plain)
    print("guided", guided, med_guided)
    assert sum(abs(b - 1.0) < 1e-9 for b in guided) >= 3
    assert max(guided) <= 2.0 and sum(guided) <= 1.5 * sum(plain)
    assert med_guided < 0.9 * med_plain


def _pretraining_rows(n=400, seed=777):
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space()
    X, y = [], []
    for i in range(n):
        p = B.trace_validate(op, sp, B.trace_sample_valid(op, sp, seed, i))
        X.append(B.variant_features(op, p))
        y.append(np.log2(synthetic_latency(p)))
    return np.array(X), np.array(y)


def test_pretrained_model_cuts_the_trials_to_the_optimum():
    """The model fitted beforehand on 400 random variants of the same operator (another seed's draws, their
    latencies from the same function) picks half of the initial population and is in use from the first generation:
    on every one of eight seeds the search then reaches the optimum, and in fewer measurements in total than the
    plain search needs (which misses it on two of the seeds within the budget)."""
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space()
    rows = _pretraining_rows()
    first_plain, first_pre = [], []
    for seed in range(8):
        for pre, out in ((None, first_plain), (rows, first_pre)):
            cfg = B.search_cfg_default()
            cfg.seed, cfg.trials, cfg.cost_model = seed, 192, int(pre is not None)
            curve = []
            res = B.search(op, sp, cfg, fake_latency=synthetic_latency, on_trial=lambda t: curve.append(t.best_us) and 0, pretrain=pre)
            assert res.n_measured == 192 and cfg.pretrain_n == 0          # the binding drops the arrays after the call
            out.append(next((i + 1 for i, b in enumerate(curve) if b <= 1.0 + 1e-9), 193))
    print("plain", first_plain, "pre-trained", first_pre)
    assert max(first_pre) <= 192
    assert sum(first_pre) < 0.75 * sum(first_plain)
    assert sum(a <= b for a, b in zip(first_pre, first_plain)) >= 7


def test_pretraining_rows_are_checked():
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space()
    X, y = _pretraining_rows(60)
    cfg = B.search_cfg_default()
    cfg.trials, cfg.cost_model = 40, 1
    with pytest.raises(B.MsError):                       # other feature count than this operator's variants
        B.search(op, sp, cfg, fake_latency=synthetic_latency, pretrain=(X[:, :-1], y))
    bad = y.copy()
    bad[3] = np.nan
    with pytest.raises(B.MsError):
        B.search(op, sp, cfg, fake_latency=synthetic_latency, pretrain=(X, bad))
    with pytest.raises(ValueError):
        B.search(op, sp, cfg, fake_latency=synthetic_latency, pretrain=(X, y[:-1]))
    # without cost_model the rows are ignored: the run equals the plain one
    cfg.cost_model = 0
    a = B.search(op, sp, cfg, fake_latency=synthetic_latency, pretrain=(X, y))
    b = B.search(op, sp, cfg, fake_latency=synthetic_latency)
    assert bytes(a.best_trace) == bytes(b.best_trace) and a.best_us == b.best_us


def test_trace_from_decisions_round_trip():
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    sp = op.space()
    for i in range(20):
        t = B.trace_sample(sp, 4, i)
        assert bytes(B.trace_from_decisions(sp, t.decisions())) == bytes(t)
    with pytest.raises(ValueError):
        B.trace_from_decisions(sp, B.trace_sample(sp, 4, 0).decisions()[:-1])


def test_model_guided_search_is_deterministic_and_identical_before_the_model_starts():
    r1, l1 = _run(3, 96, 1)
    r2, l2 = _run(3, 96, 1)
    assert l1 == l2 and bytes(r1.best_trace) == bytes(r2.best_trace)
    _, l0 = _run(3, 96, 0)
    assert l1[:48] == l0[:48] and l1 != l0                # model_min_trials = 48 measurements run without the model


def test_model_search_bad_config():
    op = B.gemm_op(128, 128, 128, "f32")
    cfg = B.search_cfg_default()
    cfg.cost_model, cfg.model_candidates = 1, 0
    with pytest.raises(B.MsError):
        B.search(op, op.space(), cfg, fake_latency=synthetic_latency)
