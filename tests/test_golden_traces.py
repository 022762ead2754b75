"""Whole-run pins for oracle B worked by hand (tests/golden/*trace*.txt, sec43_partial_copy.txt): every round of
SlideBatching's output, the clock, the token times and the Eq. 3 totals.  The same files then check the library's
batch former and its simulation, which therefore inherit a pin that is not the oracle."""
import numpy as np
import pytest

from oracle import slidebatching as S
from paper_2512_12928_amd import binding as B
from test_golden_fixtures import MS, load

HUGE = 10 ** 6


def cfgs(g, **kw):
    d = dict(class_weight=g["class_weight"] if isinstance(g["class_weight"], list) else [g["class_weight"]],
             ttft_slo=g["ttft_slo"] * MS, tpot_slo=g["tpot_slo"] * MS, w_first=g["w_first"], w_decode=g["w_decode"],
             a_p=0, b_p=0, c_p=g["c_p"] * MS, a_d=0, b_d=g["b_d"] * MS, t_c=g["t_c"] * MS, eta=g["eta"] * MS,
             tau=g["tau"] * MS, gamma_num=1, gamma_den=1, beta_num=2, beta_den=1, rho_num=9, rho_den=10,
             t_block=g.get("t_block", 1) * MS, n_off_base=g.get("n_off_base", 8))
    d.update(kw)
    oc = S.SchedConfig(**d)
    lc = dict(n_classes=len(d["class_weight"]), block_tokens=16, class_weight=d["class_weight"], w_first=d["w_first"],
              w_decode=d["w_decode"], ttft_slo_ps=d["ttft_slo"], tpot_slo_ps=d["tpot_slo"], a_p=0, b_p=0, c_p=d["c_p"], a_d=0,
              b_d=d["b_d"], t_c=d["t_c"], eta_ps=d["eta"], tau_ps=d["tau"], gamma_num=d["gamma_num"], gamma_den=d["gamma_den"],
              beta_num=2, beta_den=1, rho_num=9, rho_den=10, t_block_ps=d["t_block"], n_off_base=d["n_off_base"])
    return oc, lc


class Tr:
    def __init__(self, v):
        self.rid, arr, self.prio, self.prompt_len, self.out_len = v
        self.arrival_ps = arr * MS


def lst(g, key):
    v = g.get(key, [])
    return v if isinstance(v, list) else [v]


def pairs(v, n=2):
    return [tuple(v[i:i + n]) for i in range(0, len(v), n)]


def expected_round(g, k):
    p = "r%d_" % k
    tabs, at = [], 0
    for n in lst(g, p + "table_lens"):
        tabs.append(lst(g, p + "tables")[at:at + n])
        at += n
    return dict(now=g[p + "now"] * MS, t_budget=g[p + "t_budget"] * MS, phi=g[p + "phi_ps"], order=lst(g, p + "order"),
                urgent=lst(g, p + "urgent") if (p + "urgent") in g else None, b_copy=g[p + "b_copy"],
                batch=pairs(lst(g, p + "batch"), 3), tables=tabs, t_batch=g[p + "t_batch"] * MS,
                swap_in=pairs(lst(g, p + "swap_in")), swap_out=pairs(lst(g, p + "swap_out")), evicted=lst(g, p + "evicted"),
                emitted=pairs(lst(g, p + "emitted")), finished=lst(g, p + "finished"),
                dropped_pending=g.get(p + "dropped_pending", 0), reported=g.get(p + "reported"))


TRACES = [("alg1_trace_three_requests.txt", dict(), list(range(16)), list(range(4)), 3),
          ("sec43_eviction_reload_trace.txt", dict(gamma_num=HUGE), None, None, 2)]


@pytest.mark.parametrize("name,kw,dev,host,n_req", TRACES)
def test_oracle_simulation_follows_the_hand_worked_trace(name, kw, dev, host, n_req):
    g = load(name)
    oc, _ = cfgs(g, **kw)
    dev = dev if dev is not None else g["dev_pool"]
    host = host if host is not None else g["host_pool"]
    trace = [Tr(g["req%d" % i]) for i in range(n_req)]
    seen = []

    def on_step(sb, res):
        k = len(seen) + 1
        e = expected_round(g, k)
        tag = "%s round %d" % (name, k)
        assert res.now == e["now"] and res.round == k, tag
        assert (res.t_budget, res.phi, res.b_copy, res.t_batch) == (e["t_budget"], e["phi"], e["b_copy"], e["t_batch"]), tag
        assert res.order == e["order"], tag
        if e["urgent"] is not None:
            assert res.urgent == e["urgent"], tag
        assert res.batch == e["batch"] and res.tables == e["tables"], tag
        assert res.swap_in == e["swap_in"] and res.swap_out == e["swap_out"], tag
        assert res.evicted == e["evicted"] and res.dropped_pending == e["dropped_pending"], tag
        assert res.emitted == e["emitted"] and res.finished == e["finished"], tag
        if e["reported"] is not None:
            assert sb.offloads_done_upto == e["reported"], tag
        seen.append(k)

    sb, steps = S.simulate(oc, trace, dev, host, max_steps=50, on_step=on_step)
    assert len(steps) == g["steps"] == len(seen)
    for i in range(n_req):
        assert sb.finished_requests[i].token_times == [t * MS for t in lst(g, "token_times_%d" % i)]
    assert S.trace_gain(sb) == (g["gain"], g["ideal"], g["slo_attained"], g["finished"])
    assert steps[-1].now + steps[-1].t_batch == g["end"] * MS


@pytest.mark.parametrize("name,kw,dev,host,n_req", TRACES)
def test_library_batch_former_follows_the_hand_worked_trace(name, kw, dev, host, n_req):
    g = load(name)
    _, lc = cfgs(g, **kw)
    dev = dev if dev is not None else g["dev_pool"]
    host = host if host is not None else g["host_pool"]
    trace = [Tr(g["req%d" % i]) for i in range(n_req)]
    s = B.ps_sched_create(lc, dev, host)
    try:
        added = set()
        for k in range(1, g["steps"] + 1):
            e = expected_round(g, k)
            for t in trace:
                if t.arrival_ps <= e["now"] and t.rid not in added:
                    B.ps_sched_add_request(s, t.rid, t.arrival_ps, t.prio, t.prompt_len, t.out_len)
                    added.add(t.rid)
            if e["reported"]:
                B.ps_sched_offloads_done(s, e["reported"])
            fb = B.ps_form_batch(s, e["now"])
            tag = "%s round %d" % (name, k)
            assert fb["round"] == k, tag
            assert (fb["t_budget"], fb["phi"], fb["copy_budget"], fb["t_batch"]) == (e["t_budget"], e["phi"], e["b_copy"], e["t_batch"]), tag
            assert fb["order"].tolist() == e["order"], tag
            if e["urgent"] is not None:
                assert fb["urgent"].tolist() == e["urgent"], tag
            got_batch = list(zip(fb["req_ids"].tolist(), np.diff(fb["q_start"]).tolist(), fb["kv_len"].tolist()))
            assert got_batch == e["batch"], tag
            assert fb["block_ids"].tolist() == [b for t in e["tables"] for b in t], tag
            assert np.diff(fb["bt_start"]).tolist() == [len(t) for t in e["tables"]], tag
            assert list(zip(fb["swap_in_host_slots"].tolist(), fb["swap_in_dev_blocks"].tolist())) == e["swap_in"], tag
            assert list(zip(fb["swap_out_dev_blocks"].tolist(), fb["swap_out_host_slots"].tolist())) == e["swap_out"], tag
            assert fb["evicted"].tolist() == e["evicted"], tag
            assert list(zip(fb["emitted_req"].tolist(), fb["emitted_index"].tolist())) == e["emitted"], tag
            assert fb["finished"].tolist() == e["finished"], tag
    finally:
        B.ps_sched_destroy(s)
    # the library's own virtual-clock run (its model of the offload thread included) reaches the same totals
    r = B.ps_sched_simulate(lc, dev, host, trace, 50)
    assert (r["gain"], r["ideal_gain"], r["slo_attained"], r["finished"], r["steps"], r["end_ps"]) == \
        (g["gain"], g["ideal"], g["slo_attained"], g["finished"], g["steps"], g["end"] * MS)
    for i in range(n_req):
        assert r["token_times"][i].tolist() == [t * MS for t in lst(g, "token_times_%d" % i)]


def test_partial_copy_rule_hand_cases():
    g = load("sec43_partial_copy.txt")
    cfg = S.SchedConfig(class_weight=[1], ttft_slo=g["ttft_slo"] * MS, tpot_slo=100 * MS, c_p=g["c_p"] * MS, b_d=2 * MS,
                        t_c=g["t_c"] * MS, eta=g["eta"] * MS, tau=10 ** 6 * MS, t_block=g["t_block"] * MS, beta_num=2, beta_den=1)
    for case in "xyz":
        sb = S.SlideBatcher(cfg, list(range(16)), list(range(40)))
        sb.add_request(0, 0, 1, g[case + "_prompt"], 3)
        r = sb.reqs[0]
        r.host_slots = list(g[case + "_host"])
        r.host_round = [0] * len(r.host_slots)
        for s in r.host_slots:
            sb.host_free.remove(s)
        r.computed = 16 * len(r.host_slots)
        n_host_free = len(sb.host_free)
        res = sb.form_batch(0)
        assert res.t_budget == 50 * MS and res.b_copy == g["b_copy"], case
        if case == "x":
            assert res.batch == [] and res.swap_in == [] and res.t_batch == 0
            assert r.host_slots == list(g["x_host"]) and r.computed == 80 and len(sb.host_free) == n_host_free
        else:
            lq, kv = g[case + "_batch"]
            assert res.batch == [(0, lq, kv)], case
            assert res.swap_in == pairs(g[case + "_swap_in"]), case
            assert r.host_slots == list(g[case + "_host"])[:2], case
            assert len(sb.host_free) == n_host_free + len(g[case + "_host"]) - 2, case      # the other slots were released
            assert len(res.tables[0]) == g.get(case + "_n_blocks", 6) and res.tables[0][:2] == [0, 1], case
            assert res.t_batch == (1 + lq) * MS, case
