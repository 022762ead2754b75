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
