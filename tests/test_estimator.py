"""Latency-estimator fit (Sec. 4.1, Eqs. 4-7): the six batch features are pinned to the oracle's own
T_pd(B), and the least-squares fit to planted coefficients."""
import numpy as np

from oracle import slidebatching as S
from paper_2512_12928_amd import estimator as E
from paper_2512_12928_amd import workloads as W
from test_sched_parity import cfg_pair


def test_features_reproduce_the_oracle_estimate():
    oc, _ = cfg_pair()
    coef = np.array([oc.a_p, oc.b_p, oc.c_p, oc.a_d, oc.b_d, oc.t_c], dtype=np.float64)
    for b in E.profiling_batches(25, 3, W.LayerShape(8, 2), 40_000):
        pre = [(b.l_q(int(r)), int(b.kv_len[r]) - b.l_q(int(r))) for r in b.prefill_reqs]
        dec = [int(b.kv_len[r]) for r in b.decode_reqs]
        want = S.t_batch_estimate(oc, pre, dec)
        got = float(E.features(b.q_start, b.kv_len) @ coef)
        assert abs(got - want) <= 1e-9 * want


def test_fit_recovers_planted_coefficients():
    batches = E.profiling_batches(80, 5, W.LayerShape(32, 8), 60_000)
    X = np.stack([E.features(b.q_start, b.kv_len) for b in batches])
    planted = np.array([3e-5, 4e-5, 2e-3, 6e-4, 0.05, 25.0])       # microseconds
    y = X @ planted
    coef = E.fit(X, y)
    assert np.allclose(coef, planted, rtol=1e-6)
    assert E.mape(coef, X, y) < 1e-9
    # 5 % multiplicative noise: the error of the fit stays of that order
    rng = np.random.default_rng(1)
    yn = y * (1 + 0.05 * rng.standard_normal(len(y)))
    assert E.mape(E.fit(X[:40], yn[:40]), X[40:], yn[40:]) < 0.08


def test_profiling_batches_are_valid_and_seeded():
    a = E.profiling_batches(10, 9, W.LayerShape(32, 8), 60_000)
    b = E.profiling_batches(10, 9, W.LayerShape(32, 8), 60_000)
    for x, y in zip(a, b):
        assert np.array_equal(x.kv_len, y.kv_len) and np.array_equal(x.block_ids, y.block_ids)
        assert x.n_req >= 1 and len(set(x.block_ids.tolist())) == len(x.block_ids)


def test_critical_path_form_recovers_a_planted_max():
    """T = max(Eq. 7, t_c + w * longest walk): planted additive coefficients and w come back from the fit, and
    the additive form alone cannot explain the same data."""
    batches = E.profiling_batches(160, 11, W.LayerShape(32, 8), 60_000)
    X = np.stack([E.features(b.q_start, b.kv_len) for b in batches])
    walk = np.array([E.longest_walk(b.q_start, b.kv_len) for b in batches])
    planted = np.array([3e-6, 2e-5, 6e-3, 5.5e-4, 0.016, 28.0])
    y = np.maximum(X @ planted, planted[5] + 1.5 * walk)
    assert (planted[5] + 1.5 * walk > X @ planted).sum() > 10          # the max binds on some batches
    coef, w = E.fit_with_critical_path(X, walk, y)
    err = np.abs(E.predict_max(coef, w, X, walk) - y) / y
    assert abs(w - 1.5) <= 0.05 and err.mean() < 0.01
    assert E.mape(E.fit(X, y), X, y) > 3 * err.mean()
    b = W.build_batch(W.LayerShape(32, 8), [(1, 100), (64, 64 + 1000), (128, 128)], [1, 1, 1], np.random.default_rng(0), seed=0)
    assert E.longest_walk(b.q_start, b.kv_len) == 17                    # ceil(1064 / 64)
    b = W.build_batch(W.LayerShape(32, 8), [(1, 100)], [1], np.random.default_rng(0), seed=0)
    assert E.longest_walk(b.q_start, b.kv_len) == 0


def test_overlap_form_recovers_planted_parameters():
    """T = t_c + max(P, D) + kappa * min(P, D) with P = max(prefill terms, w * longest walk): planted coefficients,
    kappa and w come back from the fit (to the grid's step), kappa = 1 and w = 0 reproduce Eq. 7, and the additive form
    alone cannot explain data that overlaps."""
    batches = E.profiling_batches(160, 13, W.LayerShape(32, 8), 60_000)
    X = np.stack([E.features(b.q_start, b.kv_len) for b in batches])
    walk = np.array([E.longest_walk(b.q_start, b.kv_len) for b in batches])
    planted = np.array([3e-6, 2e-5, 1.2e-2, 5.5e-4, 0.02, 24.0])
    assert np.allclose(E.predict_overlap(planted, 1.0, 0.0, X, walk), X @ planted, rtol=1e-12)
    y = E.predict_overlap(planted, 0.6, 0.5, X, walk)
    both = (X[:, 2] > 0) & (X[:, 4] > 0)
    assert both.sum() > 40 and (0.5 * walk > X[:, :3] @ planted[:3]).sum() > 5   # overlap and critical path both bind
    coef, kappa, w = E.fit_with_overlap(X, walk, y)
    err = np.abs(E.predict_overlap(coef, kappa, w, X, walk) - y) / y
    assert abs(kappa - 0.6) <= 0.05 and abs(w - 0.5) <= 0.1 and err.mean() < 0.01
    assert np.allclose(coef[3:], planted[3:], rtol=0.05)
    assert E.mape(E.fit(X, y), X, y) > 3 * err.mean()
