"""The closed loop of Sec. 4.3 over a multi-layer forward pass on the GPU (paper_2512_12928_amd/closed_loop.py):
ps_form_batch sets the copy budget and the reload list of every round, the list is reloaded layer by layer with one
ticket per layer while the layers compute, what the budget leaves on the host is recomputed as prefill, offloads go out
after the pass and are reported by ticket.  EVERY layer's attention output of EVERY round is compared with the fp64
oracle computed from the requests' logical K/V histories, for the three ways of ordering reload and compute and for a
link so slow that the budget cuts the reloads."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from paper_2512_12928_amd.closed_loop import ClosedLoop
from gpu_harness import check_close
from test_sched_parity import MS, US, cfg_pair

pytestmark = pytest.mark.gpu

SEEDS = {"q": 1, "k": 2, "v": 3}


_ROWS = {}


def rows(rid, pos0, n, heads, what, layer):
    """A pure function of (request, position, layer): the request's whole row history is drawn once and sliced."""
    key = (what, layer, rid, heads)
    if key not in _ROWS:
        _ROWS[key] = W.normal_bf16(np.random.default_rng([SEEDS[what], layer, rid]), (700, heads, 128))
    return _ROWS[key][pos0:pos0 + n]


@pytest.mark.parametrize("mode,t_block", [("pipelined", 1200 * 1000 * 36), ("synchronous", 1200 * 1000 * 36),
                                          ("full_reload_first", 1200 * 1000 * 36), ("pipelined", 40 * US * 36)])
def test_closed_loop_every_layer_matches_oracle(mode, t_block):
    Hq, Hkv, M, Mh, L = 8, 2, 96, 160, 3
    oc, lc = cfg_pair(tau=3000 * MS, t_block=t_block)
    tr = W.make_trace(3, 50, rate_per_s=400.0, seed=4, prompt_mean=200, prompt_max=600, out_mean=12, out_max=40)
    rng = np.random.default_rng(4)
    loop = ClosedLoop(Hq, Hkv, M, Mh, L, lc, rng.permutation(M), rng.permutation(Mh), rows, reload_mode=mode)
    worst = [0.0]
    budget_cut = [0]

    def on_layer(ell, fb, out):
        want = []
        for i, rid in enumerate(fb["req_ids"].tolist()):
            lq = int(fb["q_start"][i + 1] - fb["q_start"][i])
            Lr = int(fb["kv_len"][i])
            want.append(A.dense_attention(A.bf16_to_f64(rows(rid, Lr - lq, lq, Hq, "q", ell)),
                                          A.bf16_to_f64(rows(rid, 0, Lr, Hkv, "k", ell)), A.bf16_to_f64(rows(rid, 0, Lr, Hkv, "v", ell))))
        worst[0] = max(worst[0], check_close(out.cpu().numpy().astype(np.float64), np.concatenate(want), False))

    st = loop.run(tr, 110, on_layer)
    loop.close()
    print(mode, t_block, st, "worst abs err %.4g" % worst[0])
    assert st["evicted"] > 0 and st["blocks_offloaded"] > 0
    if t_block < 10 * US * 36:
        assert st["blocks_reloaded"] > 0
    else:
        assert st["recomputed_tokens"] > 0          # the slow link's budget leaves blocks behind: they are computed again


def test_loop_clocks_and_scores():
    """Without memory pressure (nothing is evicted, so offload reports cannot change a decision) the loop on the
    estimator's clock delivers every token at the time ps_sched_simulate says, and its Eq. 3 score is the
    simulation's.  On the measured clock (the GPU time of every pass) the same trace still finishes and scores."""
    Hq, Hkv, M, Mh, L = 8, 2, 1500, 64, 2
    _, lc = cfg_pair(tau=3000 * MS)
    tr = W.make_trace(3, 30, rate_per_s=300.0, seed=9, prompt_mean=150, prompt_max=500, out_mean=10, out_max=30)
    rng = np.random.default_rng(9)
    dev_order, host_order = rng.permutation(M), rng.permutation(Mh)
    sim = B.ps_sched_simulate(lc, dev_order, host_order, tr, 400)
    assert sim["finished"] == len(tr)
    loop = ClosedLoop(Hq, Hkv, M, Mh, L, lc, dev_order, host_order, rows)
    st = loop.run(tr, 400)
    got = loop.score(tr)
    for i, p in enumerate(tr):
        assert np.array_equal(np.asarray(loop.token_times[p.rid], np.int64) - p.arrival_ps, sim["token_times"][i]), p.rid
    loop.close()
    assert st["evicted"] == 0
    assert got["finished"] == sim["finished"] and got["tdg_ratio"] == sim["gain"] / sim["ideal_gain"]
    loop = ClosedLoop(Hq, Hkv, M, Mh, L, lc, dev_order, host_order, rows)
    loop.run(tr, 400, clock="measured")
    got_m = loop.score(tr)
    loop.close()
    print("estimator clock", got, "measured clock", got_m)
    assert got_m["finished"] == len(tr) and 0.0 < got_m["tdg_ratio"] <= 1.0
