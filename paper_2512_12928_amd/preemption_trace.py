"""Trace mode of the preemption-heavy configuration: a 40 000-block device pool, shapes and length mix of the
Qwen3-8B-shaped configuration, three classes at 1:2:4, and an arrival rate chosen so that about 30 % of the
low-priority requests present are preempted per 100 scheduling rounds once the pool is under pressure.  The rate is
found by a seeded, documented search (a fixed grid of requests per second for workloads.make_trace, same seed
throughout; the first rate whose realised fraction lies in the band) over runs of the batch former (ps_form_batch on
a virtual clock advanced by its own T_pd(B)); the realised fraction is reported, not assumed.  The fraction is not
monotone in the rate: an open-loop trace above capacity starves its low-priority requests (they lose their blocks
once and are not admitted again for a long time), so far above capacity few of them are preempted per window.

Host only.  Every scheduling decision is the library's; this module counts.
"""
from __future__ import annotations

from typing import Dict, Sequence, Tuple

import numpy as np

from . import binding as B
from . import workloads as W

MS, US, NS = 10 ** 9, 10 ** 6, 10 ** 3
N_DEVICE_BLOCKS, N_HOST_BLOCKS = 40_000, 80_000


def default_cfg(n_layers: int = 36) -> Dict:
    """The constants of the scheduler-parity runs: TTFT 2 s, TPOT 100 ms, weights 4:2:1, estimator constants per layer
    times n_layers, t_block 1.2 us per layer."""
    return dict(n_classes=3, block_tokens=16, class_weight=[4, 2, 1], w_first=4, w_decode=1, ttft_slo_ps=2000 * MS,
                tpot_slo_ps=100 * MS, a_p=(13 * n_layers) // 2, b_p=13 * n_layers, c_p=50 * NS * n_layers,
                a_d=730 * n_layers, b_d=US * n_layers, t_c=2 * MS, eta_ps=10 * MS, tau_ps=30_000 * MS, gamma_num=9, gamma_den=10,
                beta_num=2, beta_den=1, rho_num=9, rho_den=10, t_block_ps=1200 * NS * n_layers, n_off_base=8)


def preempted_fraction(cfg: Dict, trace: Sequence, n_rounds: int, window: int = 100, low_class: int = 3,
                       n_device_blocks: int = N_DEVICE_BLOCKS, n_host_blocks: int = N_HOST_BLOCKS, seed: int = 3) -> Dict:
    """Runs the batch former over `trace` for n_rounds rounds.  Per window of `window` rounds: the low-priority requests
    evicted at least once in the window over the low-priority requests that were in the queue at some round of it.
    Returns the mean over the windows from the first one with an eviction on (the pool is under pressure from
    there) and the counts."""
    rng = np.random.default_rng(seed)
    s = B.ps_sched_create(cfg, rng.permutation(n_device_blocks).astype(np.int32), rng.permutation(n_host_blocks).astype(np.int32))
    prio = {p.rid: p.prio for p in trace}
    pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
    nxt = now = rounds = 0
    queued_low, present, hit, fracs = set(), set(), set(), []
    evictions = 0
    try:
        while rounds < n_rounds:
            while nxt < len(pending) and pending[nxt].arrival_ps <= now:
                p = pending[nxt]
                B.ps_sched_add_request(s, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
                if p.prio == low_class:
                    queued_low.add(p.rid)
                nxt += 1
            if B.ps_sched_counts(s)[0] == 0:
                if nxt >= len(pending):
                    break
                now = pending[nxt].arrival_ps
                continue
            if rounds > 0:
                B.ps_sched_offloads_done(s, rounds)        # the copy thread keeps up: every list lands before the next round
            fb = B.ps_form_batch(s, now)
            rounds += 1
            present |= queued_low
            ev = [int(r) for r in fb["evicted"].tolist()]
            evictions += len(ev)
            hit |= {r for r in ev if prio[r] == low_class}
            queued_low -= {int(r) for r in fb["finished"].tolist()}
            if rounds % window == 0:
                if present:
                    fracs.append(len(hit) / len(present))
                present, hit = set(), set()
            now += int(fb["t_batch"]) if fb["t_batch"] > 0 else int(cfg["eta_ps"])
    finally:
        B.ps_sched_destroy(s)
    first = next((k for k, f in enumerate(fracs) if f > 0), len(fracs))
    steady = fracs[first:]
    return dict(rounds=rounds, windows=len(fracs), evictions=evictions, arrived=nxt,
                fraction=float(np.mean(steady)) if steady else 0.0, per_window=[round(f, 3) for f in fracs])


RATE_GRID = (50.0, 60.0, 70.0, 80.0, 90.0, 100.0, 115.0, 130.0, 150.0)


def tune_rate(grid: Sequence[float] = RATE_GRID, band: Tuple[float, float] = (0.25, 0.35), n_requests: int = 3000,
              n_rounds: int = 1000, seed: int = 2512_12931, cfg: Dict = None, **trace_kw) -> Dict:
    """Tries the arrival rates of `grid` (requests per second, all classes together) in order, every probe with the
    same trace seed, and stops at the first whose realised fraction of preempted low-priority requests per 100 rounds
    lies in `band`.  Returns the rate, the realised fraction and the probes."""
    cfg = default_cfg() if cfg is None else cfg
    kw = dict(prompt_mean=1500.0, prompt_max=8192, out_mean=256.0, out_max=2048)
    kw.update(trace_kw)
    probes = []
    res = None
    for rate in grid:
        trace = W.make_trace(3, n_requests, rate_per_s=float(rate), seed=seed, **kw)
        res = preempted_fraction(cfg, trace, n_rounds)
        probes.append((float(rate), round(res["fraction"], 4)))
        if band[0] <= res["fraction"] <= band[1]:
            break
    return dict(rate_per_s=probes[-1][0], fraction=probes[-1][1], in_band=band[0] <= probes[-1][1] <= band[1], probes=probes,
                last=res)


if __name__ == "__main__":
    import json
    print(json.dumps(tune_rate()))
