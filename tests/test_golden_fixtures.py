"""The oracle against the hand-worked fixtures of tests/golden/ (see the README there)."""
import os

from oracle import slidebatching as S

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
MS = 10 ** 9


def load(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [x.strip() for x in line.split("=")]
        vals = [int(x) for x in v.split(",")]
        out[k] = vals[0] if len(vals) == 1 else vals
    return out


def test_eq3_gain():
    g = load("eq3_tdg_gain.txt")
    args = (g["ttft_slo"] * MS, g["tpot_slo"] * MS, g["w_first"], g["w_decode"], g["w_class"])
    assert [S.deadline(i + 1, args[0], args[1]) for i in range(5)] == [d * MS for d in g["deadlines"]]
    assert S.tdg_gain([t * MS for t in g["token_times"]], *args) == g["gain"]
    assert S.ideal_gain(len(g["token_times"]), *args[2:]) == g["ideal"]
    assert S.tdg_gain([g["ttft_slo"] * MS], *args) == g["gain_at_deadline"]


def test_eqs4_7_estimator():
    g = load("eqs4_7_estimator.txt")
    cfg = S.SchedConfig(class_weight=[1], ttft_slo=MS, tpot_slo=MS, a_p=g["a_p"], b_p=g["b_p"], c_p=g["c_p"], a_d=g["a_d"],
                        b_d=g["b_d"], t_c=g["t_c"])
    assert S.t_prefill(cfg, 10, 100) == g["t_prefill_10_100"]
    assert S.t_prefill(cfg, 2, 0) == g["t_prefill_2_0"]
    assert S.t_decode(cfg, 100) == g["t_decode_100"] and S.t_decode(cfg, 1) == g["t_decode_1"]
    assert S.t_batch_estimate(cfg, [(10, 100), (2, 0)], [100, 1]) == g["t_batch"]


def test_eq8_phi():
    g = load("eq8_phi.txt")
    assert S.phi(g["t_budget"] * MS, g["t_c"] * MS, g["sum_exec"] * MS) == g["phi"] * MS


def test_sec43_copy_budget():
    g = load("sec43_copy_budget.txt")
    cfg = S.SchedConfig(class_weight=[1], ttft_slo=MS, tpot_slo=MS, t_block=g["t_block"], c_p=g["c_p"])
    for case in ("case1", "case2i", "case2ii", "case2ii_b"):
        t_budget, t_fwd, miss = g[case]
        assert S.copy_budget(cfg, t_budget=t_budget, t_fwd_min=t_fwd, b_missing=miss) == g[case + "_budget"], case
