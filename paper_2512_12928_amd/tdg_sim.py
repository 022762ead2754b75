"""Single-instance serving simulation on a virtual clock (`ps_sched_simulate`, host only, no GPU): the batch
former is driven by a synthetic arrival trace, the clock advances by the estimated batch latency T_pd(B) of
Sec. 4.1, and the token-level deadline-aware gain of Eq. 3 is summed over the finished requests (TDG ratio =
gain / ideal gain, Sec. 5.1).  This module only builds the configuration and prints the sweep; the simulation
and the scoring run in the library.  `python -m paper_2512_12928_amd.tdg_sim` sweeps the arrival rate for the
ordering SlideBatching uses (gamma = 0.9), for its two ablation arms that need nothing else -- deadline order
only (gamma = 0) and density order only (gamma very large) (Sec. 5.3) -- and for first-come-first-served.
"""
from __future__ import annotations

import json
import sys
from typing import Dict

import numpy as np

from . import binding as B
from . import workloads as W

MS, US, NS = 10 ** 9, 10 ** 6, 10 ** 3


def default_cfg(n_layers: int = 36, **kw) -> Dict:
    """Scheduler constants for a 36-layer model; the estimator terms are per layer x n_layers.  The per-layer
    values are the fit of profiles/estimator_fit_mi355x.md rounded to integer picoseconds."""
    L = n_layers
    d = dict(n_classes=3, block_tokens=16, class_weight=[4, 2, 1], w_first=4, w_decode=1, ttft_slo_ps=2000 * MS,
             tpot_slo_ps=100 * MS, a_p=2 * L, b_p=15 * L, c_p=10279 * L, a_d=558 * L, b_d=10200 * L, t_c=26670 * NS * L,
             eta_ps=10 * MS, tau_ps=30_000 * MS, gamma_num=9, gamma_den=10, beta_num=2, beta_den=1, rho_num=9,
             rho_den=10, t_block_ps=1200 * NS * L, n_off_base=8)
    d.update(kw)
    return d


def run_trace(cfg: Dict, trace, dev_order, host_order, max_steps: int) -> Dict:
    """Gain, ideal gain and SLO attainment over the finished requests of one run."""
    r = B.ps_sched_simulate(cfg, np.asarray(dev_order, np.int32), np.asarray(host_order, np.int32), trace, max_steps)
    return dict(gain=r["gain"], ideal=r["ideal_gain"], tdg_ratio=(r["gain"] / r["ideal_gain"] if r["ideal_gain"] else 0.0),
                slo_attained=r["slo_attained"], finished=r["finished"], steps=r["steps"], end_ps=r["end_ps"],
                token_times=r["token_times"])


def main(argv=None) -> int:
    n_req = int(argv[0]) if argv else 1500
    M = 40_000
    rng = np.random.default_rng(12)
    dev, host = rng.permutation(M), rng.permutation(2 * M)
    arms = {"first come first served": dict(order_policy=B.PS_ORDER_FCFS),
            "deadline order only (gamma 0)": dict(gamma_num=0, gamma_den=1),
            "SlideBatching (gamma 0.9)": dict(gamma_num=9, gamma_den=10),
            "density order only (gamma 1e6)": dict(gamma_num=10 ** 6, gamma_den=1)}
    for rate in (100.0, 200.0, 300.0, 500.0, 1000.0):
        trace = W.make_trace(2, n_req, rate_per_s=rate, out_mean=256.0)
        row = dict(rate_per_s=rate)
        for name, kw in arms.items():
            r = run_trace(default_cfg(**kw), trace, dev, host, max_steps=400_000)
            row[name] = dict(tdg_ratio=round(r["tdg_ratio"], 4), slo_attainment=round(r["slo_attained"] / max(r["finished"], 1), 4),
                             finished=r["finished"])
        print(json.dumps(row), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
