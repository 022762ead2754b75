"""Virtual-clock serving simulation behind the C ABI (ps_sched_simulate, ps_tdg_score) against the oracle's own
simulation of the same trace, request by request bit-exact in integer picoseconds.  The oracle's simulation
and scoring are themselves pinned to hand-worked traces in tests/test_golden_traces.py."""
import numpy as np
import pytest

from oracle import slidebatching as S
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import tdg_sim as T
from paper_2512_12928_amd import workloads as W
from test_sched_parity import MS, cfg_pair


def test_token_score_matches_oracle_on_random_times():
    rng = np.random.default_rng(0)
    oc, lc = cfg_pair()
    for _ in range(200):
        n = int(rng.integers(0, 40))
        tt = np.sort(rng.integers(0, 8000 * MS, n)).tolist()
        ttft, tpot, wf, wd = int(rng.integers(1, 3000)) * MS, int(rng.integers(1, 300)) * MS, int(rng.integers(1, 8)), int(rng.integers(1, 4))
        prio = int(rng.integers(1, 4))
        cfg = {**lc, "ttft_slo_ps": ttft, "tpot_slo_ps": tpot, "w_first": wf, "w_decode": wd}
        wc = cfg["class_weight"][prio - 1]
        g, ideal, ok = B.ps_tdg_score(cfg, prio, n, tt)
        assert g == S.tdg_gain(tt, ttft, tpot, wf, wd, wc)
        assert ideal == S.ideal_gain(n, wf, wd, wc)
        assert bool(ok) == S.slo_attained(tt, ttft, tpot)


@pytest.mark.parametrize("kw", [dict(gamma_num=0, gamma_den=1), dict(gamma_num=9, gamma_den=10),
                                dict(gamma_num=10 ** 6, gamma_den=1), dict(order_policy=1),
                                dict(t_block=40 * 10 ** 6 * 36, n_off_base=2)])
def test_simulation_matches_oracle_simulation(kw):
    """Under memory pressure (evictions, reloads, offloads discarded in flight), for the orderings the sweep uses."""
    oc, lc = cfg_pair(**kw)
    if "order_policy" in kw:
        lc["order_policy"] = kw["order_policy"]
    trace = W.make_trace(3, 150, rate_per_s=300.0, seed=8, prompt_mean=300, prompt_max=900, out_mean=20, out_max=60)
    rng = np.random.default_rng(2)
    dev, host = rng.permutation(400).astype(np.int32), rng.permutation(800).astype(np.int32)
    sb, steps = S.simulate(oc, trace, dev, host, max_steps=3000)
    g, ideal, ok, fin = S.trace_gain(sb)
    got = T.run_trace(lc, trace, dev, host, max_steps=3000)
    assert (got["gain"], got["ideal"], got["slo_attained"], got["finished"], got["steps"]) == (g, ideal, ok, fin, len(steps))
    assert fin > 50 and 0 < g <= ideal
    for i, p in enumerate(trace):
        if p.rid in sb.finished_requests:
            assert got["token_times"][i].tolist() == sb.finished_requests[p.rid].token_times
