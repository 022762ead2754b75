"""Single-instance serving simulation on a virtual clock: the batch former (ps_form_batch) is driven by a
synthetic arrival trace, the clock advances by the estimated batch latency T_pd(B) of Sec. 4.1, and the
token-level deadline-aware gain of Eq. 3 is summed over the finished requests (TDG ratio = gain / ideal
gain, Sec. 5.1).  No GPU needed.  `python -m paper_2512_12928_amd.tdg_sim` sweeps the arrival rate for
the ordering SlideBatching uses (gamma = 0.9) and for its two ablation arms that need nothing else:
deadline order only (gamma = 0) and density order only (gamma very large) (Sec. 5.3).

All times are integer picoseconds, as in the scheduler.
"""
from __future__ import annotations

import json
import sys
from typing import Dict, List, Sequence

import numpy as np

from . import binding as B
from . import workloads as W

MS, US, NS = 10 ** 9, 10 ** 6, 10 ** 3


def token_gain(token_times: Sequence[int], ttft_slo: int, tpot_slo: int, w_first: int, w_decode: int, w_class: int) -> int:
    """Eq. 3: sum of the weights of the tokens delivered before their deadline TTFT_SLO + (i-1) TPOT_SLO
    (times relative to arrival; the first token weighs w_first, the others w_decode, times the class weight)."""
    g = 0
    for i, t in enumerate(token_times, start=1):
        if t < ttft_slo + (i - 1) * tpot_slo:
            g += (w_first if i == 1 else w_decode) * w_class
    return g


def ideal_gain(n_out: int, w_first: int, w_decode: int, w_class: int) -> int:
    return (w_first + (n_out - 1) * w_decode) * w_class if n_out > 0 else 0


def default_cfg(n_layers: int = 36, **kw) -> Dict:
    """Scheduler constants for a 36-layer model; the estimator terms are per layer x n_layers.  The per-layer
    values are the fit of profiles/estimator_fit_mi355x.md rounded to integer picoseconds."""
    L = n_layers
    d = dict(n_classes=3, block_tokens=16, class_weight=[4, 2, 1], w_first=4, w_decode=1, ttft_slo_ps=2000 * MS,
             tpot_slo_ps=100 * MS, a_p=3 * L, b_p=19 * L, c_p=5682 * L, a_d=554 * L, b_d=15784 * L, t_c=28 * US * L,
             eta_ps=10 * MS, tau_ps=30_000 * MS, gamma_num=9, gamma_den=10, beta_num=2, beta_den=1, rho_num=9,
             rho_den=10, t_block_ps=1200 * NS * L, n_off_base=8)
    d.update(kw)
    return d


def run_trace(cfg: Dict, trace, dev_order, host_order, max_steps: int) -> Dict:
    """Drives the batch former over the trace; returns gain, ideal gain, SLO attainment over finished requests."""
    sched = B.ps_sched_create(cfg, np.asarray(dev_order, np.int32), np.asarray(host_order, np.int32))
    pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
    info = {p.rid: p for p in pending}
    times: Dict[int, List[int]] = {}
    done: List[int] = []
    nxt = now = steps = 0
    try:
        while steps < max_steps:
            while nxt < len(pending) and pending[nxt].arrival_ps <= now:
                p = pending[nxt]
                B.ps_sched_add_request(sched, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
                nxt += 1
            if B.ps_sched_counts(sched)[0] == 0:
                if nxt >= len(pending):
                    break
                now = pending[nxt].arrival_ps
                continue
            fb = B.ps_form_batch(sched, now)
            steps += 1
            t_batch = int(fb["t_batch"])
            for rid in fb["emitted_req"].tolist():           # tokens are delivered when the batch ends
                times.setdefault(int(rid), []).append(now + t_batch - info[int(rid)].arrival_ps)
            done.extend(int(r) for r in fb["finished"].tolist())
            now += t_batch if t_batch > 0 else int(cfg["eta_ps"])
    finally:
        B.ps_sched_destroy(sched)
    gain = ideal = ok = 0
    for rid in done:
        p, tt = info[rid], times.get(rid, [])
        wc = cfg["class_weight"][p.prio - 1]
        gain += token_gain(tt, cfg["ttft_slo_ps"], cfg["tpot_slo_ps"], cfg["w_first"], cfg["w_decode"], wc)
        ideal += ideal_gain(p.out_len, cfg["w_first"], cfg["w_decode"], wc)
        n = len(tt)
        ok += bool(tt) and tt[0] < cfg["ttft_slo_ps"] and (n == 1 or tt[-1] - tt[0] < cfg["tpot_slo_ps"] * (n - 1))
    return dict(gain=gain, ideal=ideal, tdg_ratio=(gain / ideal if ideal else 0.0), slo_attained=ok, finished=len(done),
                steps=steps, end_ps=now)


def main(argv=None) -> int:
    n_req = int(argv[0]) if argv else 1500
    M = 40_000
    rng = np.random.default_rng(12)
    dev, host = rng.permutation(M), rng.permutation(2 * M)
    arms = {"deadline order only (gamma 0)": dict(gamma_num=0, gamma_den=1),
            "SlideBatching (gamma 0.9)": dict(gamma_num=9, gamma_den=10),
            "density order only (gamma 1e6)": dict(gamma_num=10 ** 6, gamma_den=1)}
    rows = []
    for rate in (100.0, 200.0, 300.0, 500.0, 1000.0):
        trace = W.make_trace(2, n_req, rate_per_s=rate, out_mean=256.0)
        row = dict(rate_per_s=rate)
        for name, kw in arms.items():
            r = run_trace(default_cfg(**kw), trace, dev, host, max_steps=400_000)
            row[name] = dict(tdg_ratio=round(r["tdg_ratio"], 4), slo_attainment=round(r["slo_attained"] / max(r["finished"], 1), 4),
                             finished=r["finished"])
        rows.append(row)
        print(json.dumps(row), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
