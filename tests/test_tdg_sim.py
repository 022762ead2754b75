"""Virtual-clock serving simulation (Eq. 3 gain over a trace driven through ps_form_batch): pinned to the
oracle's own simulation of the same trace, request by request bit-exact in integer picoseconds."""
import numpy as np
import pytest

from oracle import slidebatching as S
from paper_2512_12928_amd import tdg_sim as T
from paper_2512_12928_amd import workloads as W
from test_sched_parity import MS, cfg_pair


def test_token_gain_matches_oracle_on_random_times():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(0, 40))
        tt = np.sort(rng.integers(0, 8000 * MS, n)).tolist()
        args = (int(rng.integers(1, 3000)) * MS, int(rng.integers(1, 300)) * MS, int(rng.integers(1, 8)), int(rng.integers(1, 4)),
                int(rng.integers(1, 9)))
        assert T.token_gain(tt, *args) == S.tdg_gain(tt, *args)
        assert T.ideal_gain(n, *args[2:]) == S.ideal_gain(n, *args[2:])


@pytest.mark.parametrize("gamma", [(0, 1), (9, 10), (10 ** 6, 1)])
def test_simulation_matches_oracle_simulation(gamma):
    """Under memory pressure (evictions, reloads), for the three orderings the sweep uses."""
    oc, lc = cfg_pair(gamma_num=gamma[0], gamma_den=gamma[1])
    trace = W.make_trace(3, 150, rate_per_s=300.0, seed=8, prompt_mean=300, prompt_max=900, out_mean=20, out_max=60)
    rng = np.random.default_rng(2)
    dev, host = rng.permutation(400).astype(np.int32), rng.permutation(800).astype(np.int32)
    sb, steps = S.simulate(oc, trace, dev, host, max_steps=3000)
    g, ideal, ok, fin = S.trace_gain(sb)
    got = T.run_trace(lc, trace, dev, host, max_steps=3000)
    assert (got["gain"], got["ideal"], got["slo_attained"], got["finished"], got["steps"]) == (g, ideal, ok, fin, len(steps))
    assert fin > 50 and 0 < g <= ideal
