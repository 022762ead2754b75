"""The latency estimator of Sec. 4.1 (Eqs. 4-7) fitted to ps_step times measured on this GPU: seeded profiling
batches, least squares on one half, mean absolute percentage error on the other.  Asserted: the additive form of
Eq. 7 predicts one attention layer within 16 % on average (the paper reports about 4.5 % for a whole model's forward
pass, most of it linear layers), the form with a critical-path term (a launch ends no sooner than its longest prefill
row) is within three points of it, the form in which part of the shorter of the two kinds of work hides under the longer is no
worse than the additive one (on the 240-batch run of profiles/ it is 1.5 points better), and the fitted constants are physical."""
import numpy as np
import pytest

from paper_2512_12928_amd import estimator as E
from paper_2512_12928_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_fit_on_measured_steps():
    shape = W.LayerShape(32, 8)
    n, n_blocks = 160, 60_000
    batches = E.profiling_batches(n, 2512_12928, shape, n_blocks)
    y = E.measure(batches, shape, n_blocks, steps=12)
    X = np.stack([E.features(b.q_start, b.kv_len) for b in batches])
    walk = np.array([E.longest_walk(b.q_start, b.kv_len) for b in batches])
    half = n // 2
    coef = E.fit(X[:half], y[:half])
    coef_m, w = E.fit_with_critical_path(X[:half], walk[:half], y[:half])
    add = E.mape(coef, X[half:], y[half:])
    rel = np.abs(E.predict_max(coef_m, w, X[half:], walk[half:]) - y[half:]) / y[half:]
    print("additive form: eval MAPE %.3f; with critical path (w = %.2f us per tile): %.3f; steps %.0f-%.0f us"
          % (add, w, rel.mean(), y.min(), y.max()))
    coef_o, kappa, w_o = E.fit_with_overlap(X[:half], walk[:half], y[:half])
    rel_o = np.abs(E.predict_overlap(coef_o, kappa, w_o, X[half:], walk[half:]) - y[half:]) / y[half:]
    print("with overlap (kappa = %.2f, w = %.2f us per tile): %.3f" % (kappa, w_o, rel_o.mean()))
    assert (y > 5).all() and (y < 5000).all()
    assert add < 0.16
    assert rel.mean() <= add + 0.03
    assert rel_o.mean() <= add + 0.01 and 0.2 <= kappa <= 1.0
    # the marginal cost of a cached decode token is that of streaming its 4 KiB of K and V at a few TB/s
    assert 4096 / 9e6 < coef[3] < 4096 / 3e6                     # us per token
    assert 0 < coef[5] < 80                                      # the fixed cost of a step, us
