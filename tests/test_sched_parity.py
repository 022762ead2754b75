"""The library's batch former (ps_form_batch, C++) against oracle B on synthetic traces: batch
membership, chunk sizes, order, block tables, swap lists, budgets, delivered tokens -- all bit-exact,
step by step on a virtual clock.  Host-only: runs without a GPU."""
import ctypes as C

import numpy as np
import pytest

from oracle import slidebatching as S
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W

MS, US, NS = 10 ** 9, 10 ** 6, 10 ** 3


def cfg_pair(n_layers=36, n_classes=3, **kw):
    d = dict(class_weight=[2 ** (n_classes - 1 - i) for i in range(n_classes)], ttft_slo=2000 * MS, tpot_slo=100 * MS,
             w_first=4, w_decode=1, a_p=(13 * n_layers) // 2, b_p=13 * n_layers, c_p=50 * NS * n_layers,
             a_d=730 * n_layers, b_d=1 * US * n_layers, t_c=2 * MS, eta=10 * MS, tau=30_000 * MS,
             t_block=1200 * NS * n_layers, gamma_num=9, gamma_den=10, beta_num=2, beta_den=1, rho_num=9, rho_den=10,
             n_off_base=8, order_policy=0)
    d.update(kw)
    oc = S.SchedConfig(**d)
    lib = dict(n_classes=n_classes, block_tokens=16, class_weight=d["class_weight"], w_first=d["w_first"],
               w_decode=d["w_decode"], ttft_slo_ps=d["ttft_slo"], tpot_slo_ps=d["tpot_slo"], a_p=d["a_p"], b_p=d["b_p"],
               c_p=d["c_p"], a_d=d["a_d"], b_d=d["b_d"], t_c=d["t_c"], eta_ps=d["eta"], tau_ps=d["tau"],
               gamma_num=d["gamma_num"], gamma_den=d["gamma_den"], beta_num=d["beta_num"], beta_den=d["beta_den"],
               rho_num=d["rho_num"], rho_den=d["rho_den"], t_block_ps=d["t_block"], n_off_base=d["n_off_base"],
               order_policy=d["order_policy"])
    return oc, lib


def run_both(oc, lib_cfg, trace, M, Mh, max_steps, seed, lag=0):
    """lag: how many rounds an offload list stays in flight before both sides are told that it has landed
    (0: reported before the next round; None: never reported)."""
    rng = np.random.default_rng(seed)
    dev_order, host_order = rng.permutation(M).astype(np.int32), rng.permutation(Mh).astype(np.int32)
    sb = S.SlideBatcher(oc, dev_order, host_order)
    ls = B.ps_sched_create(lib_cfg, dev_order, host_order)
    pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
    nxt, now, steps = 0, 0, 0
    stats = dict(evicted=0, swap_in=0, swap_out=0, admitted=0, partial=0, chunks=0, finished=0, dropped_pending=0)
    try:
        while steps < max_steps:
            while nxt < len(pending) and pending[nxt].arrival_ps <= now:
                p = pending[nxt]
                sb.add_request(p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
                B.ps_sched_add_request(ls, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
                nxt += 1
            if not sb.reqs:
                if nxt >= len(pending):
                    break
                now = pending[nxt].arrival_ps
                continue
            if lag is not None and steps - lag > 0:
                sb.offloads_done(steps - lag)
                B.ps_sched_offloads_done(ls, steps - lag)
            want = sb.form_batch(now)
            got = B.ps_form_batch(ls, now)
            steps += 1
            assert got["round"] == want.round == steps
            tag = "step %d now %d" % (steps, now)
            assert got["req_ids"].tolist() == [r for r, _, _ in want.batch], tag          # membership and order
            assert np.diff(got["q_start"]).tolist() == [c for _, c, _ in want.batch], tag  # chunk sizes
            assert got["kv_len"].tolist() == [k for _, _, k in want.batch], tag
            assert got["block_ids"].tolist() == [b for t in want.tables for b in t], tag   # block tables
            assert np.diff(got["bt_start"]).tolist() == [len(t) for t in want.tables], tag
            assert got["prio"].tolist() == want.prios, tag
            assert (got["t_budget"], got["phi"], got["copy_budget"], got["t_batch"]) == \
                (want.t_budget, want.phi, want.b_copy, want.t_batch), tag
            assert got["order"].tolist() == want.order and got["urgent"].tolist() == want.urgent, tag
            assert list(zip(got["swap_in_host_slots"].tolist(), got["swap_in_dev_blocks"].tolist())) == want.swap_in, tag
            assert list(zip(got["swap_out_dev_blocks"].tolist(), got["swap_out_host_slots"].tolist())) == want.swap_out, tag
            assert got["evicted"].tolist() == want.evicted, tag
            assert list(zip(got["emitted_req"].tolist(), got["emitted_index"].tolist())) == want.emitted, tag
            assert got["finished"].tolist() == want.finished, tag
            nq, ndf, nhf = B.ps_sched_counts(ls)
            assert (nq, ndf, nhf) == (len(sb.reqs), len(sb.dev_free), len(sb.host_free)), tag
            stats["dropped_pending"] += want.dropped_pending
            stats["evicted"] += len(want.evicted); stats["swap_in"] += len(want.swap_in)
            stats["swap_out"] += len(want.swap_out); stats["admitted"] += len(want.batch)
            stats["chunks"] += sum(1 for _, c, _ in want.batch if c > 1); stats["finished"] += len(want.finished)
            now += want.t_batch if want.t_batch > 0 else oc.eta
    finally:
        B.ps_sched_destroy(ls)
    return steps, stats


def test_low_load_trace_1000_steps():
    oc, lc = cfg_pair()
    tr = W.make_trace(2, 300, rate_per_s=12.0)
    steps, st = run_both(oc, lc, tr, 6000, 12000, 1000, seed=0)
    assert steps == 1000 and st["admitted"] > 1000 and st["swap_out"] > 0 and st["evicted"] == 0


def test_preemption_heavy_trace():
    """Pool sized so that admissions evict: exercises eviction from the tail, budgeted and partial reload,
    recomputation after a drop, offload thresholds per class."""
    oc, lc = cfg_pair(tau=3000 * MS)
    tr = W.make_trace(3, 250, rate_per_s=200.0, seed=1, prompt_mean=600, prompt_max=3000, out_mean=40, out_max=200)
    steps, st = run_both(oc, lc, tr, 300, 600, 1000, seed=1)
    assert steps >= 600 and st["evicted"] > 100 and st["swap_in"] > 100 and st["swap_out"] > 100 and st["chunks"] > 10


@pytest.mark.parametrize("lag", [2, 5, None])
def test_preemption_with_offloads_in_flight(lag):
    """Offload lists stay in flight for several rounds (or are never reported): evictions discard the pending
    copies (Sec. 4.3, Asynchronous Offloading) and both sides must still agree on everything."""
    oc, lc = cfg_pair(tau=3000 * MS, n_off_base=2)
    tr = W.make_trace(3, 250, rate_per_s=200.0, seed=1, prompt_mean=600, prompt_max=3000, out_mean=40, out_max=200)
    steps, st = run_both(oc, lc, tr, 300, 600, 800, seed=1, lag=lag)
    assert steps >= 500 and st["evicted"] > 50 and st["dropped_pending"] > 0
    if lag is None:
        assert st["swap_in"] == 0           # nothing was ever confirmed, so nothing can be reloaded


def test_bursty_four_class_trace():
    oc, lc = cfg_pair(n_layers=80, n_classes=4, tau=5000 * MS)
    tr = W.make_trace(5, 300, rate_per_s=40.0, seed=5, prompt_mean=2000, prompt_max=16384, out_mean=64, out_max=512,
                      class_ratios=(1, 2, 4, 8), bursty_high=True)
    steps, st = run_both(oc, lc, tr, 2500, 5000, 1000, seed=5)
    assert steps == 1000 and st["admitted"] > 1000


@pytest.mark.parametrize("kw", [dict(gamma_num=0), dict(gamma_num=10 ** 6), dict(beta_num=1, beta_den=1),
                                dict(n_off_base=1), dict(tau=200 * MS), dict(eta=3 * MS, t_c=1 * MS),
                                dict(t_block=40 * US * 36), dict(order_policy=1)])
def test_parameter_corners(kw):
    oc, lc = cfg_pair(**kw)
    tr = W.make_trace(2, 120, rate_per_s=150.0, seed=9, prompt_mean=500, prompt_max=2500, out_mean=30, out_max=120)
    steps, st = run_both(oc, lc, tr, 260, 400, 400, seed=9)
    assert steps > 100


def test_tiny_host_pool_and_single_class():
    oc, lc = cfg_pair(n_classes=1)
    tr = W.make_trace(2, 80, rate_per_s=100.0, seed=11, prompt_mean=300, prompt_max=1500, out_mean=20, out_max=60,
                      class_ratios=(1,))
    run_both(oc, lc, tr, 120, 7, 400, seed=11)          # host pool smaller than most requests: offloads are skipped


def test_create_and_add_validation():
    oc, lc = cfg_pair()
    for bad in (dict(eta_ps=lc["t_c"]), dict(n_classes=0), dict(n_classes=9), dict(gamma_den=0), dict(t_block_ps=0),
                dict(class_weight=[1, 0, 1])):
        with pytest.raises(B.PsError) as e:
            B.ps_sched_create({**lc, **bad}, [0, 1, 2], [0, 1])
        assert e.value.code == B.PS_EINVAL
    with pytest.raises(B.PsError):
        B.ps_sched_create(lc, [0, 1, 1], [0])                      # duplicate block id
    s = B.ps_sched_create(lc, [0, 1, 2], [0, 1])
    B.ps_sched_add_request(s, 7, 0, 1, 10, 3)
    for args in ((7, 0, 1, 10, 3), (8, 0, 0, 10, 3), (8, 0, 4, 10, 3), (8, 0, 1, 0, 3), (8, 0, 1, 10, 0)):
        with pytest.raises(B.PsError) as e:
            B.ps_sched_add_request(s, *args)
        assert e.value.code == B.PS_EINVAL
    empty = B.ps_form_batch(s, -5)                                  # nothing has arrived yet
    assert empty["n_req"] == 0 and empty["t_batch"] == 0 and len(empty["order"]) == 0
    B.ps_sched_destroy(s)
