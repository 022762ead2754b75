"""End-to-end engine loop on the GPU: ps_form_batch -> ps_swap_in (ticket) -> ps_step -> ps_swap_out, step
after step under memory pressure, every attention output compared with the fp64 oracle computed from the
requests' logical K/V histories.  Exercises eviction, budgeted reload, recomputation after a drop and the
offload path with real data."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from gpu_harness import DEV, check_close, u16_to_dev
from test_sched_parity import MS, cfg_pair

pytestmark = pytest.mark.gpu


def token_rows(rid, pos0, n, heads, seed):
    """K/V/Q rows of request rid for positions pos0..pos0+n-1: a function of (rid, position) only, so a
    recomputed token gets the same rows as the first time."""
    out = np.empty((n, heads, 128), dtype=np.uint16)
    for t in range(n):
        rng = np.random.default_rng([seed, rid, pos0 + t])
        out[t] = W.normal_bf16(rng, (heads, 128))
    return out


def test_engine_loop_matches_oracle():
    Hq, Hkv, M, Mh = 8, 2, 96, 160
    shape = W.LayerShape(Hq, Hkv)
    oc, lc = cfg_pair(tau=3000 * MS)
    tr = W.make_trace(3, 60, rate_per_s=400.0, seed=4, prompt_mean=200, prompt_max=600, out_mean=12, out_max=40)
    rng = np.random.default_rng(4)
    sched = B.ps_sched_create(lc, rng.permutation(M).astype(np.int32), rng.permutation(Mh).astype(np.int32))
    ctx = B.ps_create(Hq, Hkv, M, Mh, out_dtype=B.PS_F32)
    cache = torch.full((M, shape.block_bytes // 2), float("nan"), dtype=torch.bfloat16, device=DEV)
    host = torch.zeros((Mh, shape.block_bytes), dtype=torch.uint8).pin_memory()
    compute, side_in, side_out = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ws_bytes = B.ps_workspace_bytes(ctx, 64, 4096, M)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    pending = sorted(tr, key=lambda x: (x.arrival_ps, x.rid))
    nxt, now, steps = 0, 0, 0
    seen = dict(evicted=0, swap_in=0, swap_out=0, recomputed=0)
    hist_len = {}                                  # rid -> tokens whose KV the engine believes it holds
    out_tickets = []                               # (round, ticket) of offload lists still in flight, oldest first
    worst = 0.0
    while steps < 160:
        while nxt < len(pending) and pending[nxt].arrival_ps <= now:
            p = pending[nxt]
            B.ps_sched_add_request(sched, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
            nxt += 1
        if B.ps_sched_counts(sched)[0] == 0:
            if nxt >= len(pending):
                break
            now = pending[nxt].arrival_ps
            continue
        # the copy thread's report (Sec. 4.3, Asynchronous Offloading): offloads whose ticket has completed count
        # as host copies from now on; nobody waits for one -- an eviction discards what is still in flight
        while out_tickets and B.ps_ticket_query(ctx, out_tickets[0][1]) == B.PS_OK:
            B.ps_sched_offloads_done(sched, out_tickets.pop(0)[0])
        fb = B.ps_form_batch(sched, now)
        steps += 1
        seen["evicted"] += len(fb["evicted"]); seen["swap_in"] += len(fb["swap_in_dev_blocks"])
        seen["swap_out"] += len(fb["swap_out_dev_blocks"])
        if fb["n_req"] == 0:
            now += oc.eta
            continue
        n_in, tk_in = B.ps_swap_in(ctx, fb["swap_in_host_slots"], fb["swap_in_dev_blocks"], int(fb["copy_budget"]),
                                   host, cache, side_in)
        assert n_in == len(fb["swap_in_dev_blocks"])
        # this step's query/key/value rows
        qs, ks, vs, want = [], [], [], []
        for i, rid in enumerate(fb["req_ids"].tolist()):
            lq = int(fb["q_start"][i + 1] - fb["q_start"][i])
            L = int(fb["kv_len"][i])
            if hist_len.get(rid, 0) > L - lq:
                seen["recomputed"] += 1
            hist_len[rid] = L
            q = token_rows(rid, L - lq, lq, Hq, 1)
            qs.append(q); ks.append(token_rows(rid, L - lq, lq, Hkv, 2)); vs.append(token_rows(rid, L - lq, lq, Hkv, 3))
            want.append(A.dense_attention(A.bf16_to_f64(q), A.bf16_to_f64(token_rows(rid, 0, L, Hkv, 2)),
                                          A.bf16_to_f64(token_rows(rid, 0, L, Hkv, 3))))
        q_dev, k_dev, v_dev = (u16_to_dev(np.concatenate(x)) for x in (qs, ks, vs))
        out = torch.empty((fb["n_tokens"], Hq, 128), dtype=torch.float32, device=DEV)
        batch = B.make_batch(fb["q_start"], fb["kv_len"], fb["bt_start"], fb["block_ids"], fb["prio"])
        B.ps_step(ctx, batch, q_dev, k_dev, v_dev, cache, out, ws, ws_bytes, compute, tk_in)
        compute.synchronize()
        worst = max(worst, check_close(out.cpu().numpy().astype(np.float64), np.concatenate(want), False))
        # offload after the step (the new rows are in the cache now)
        n_out, tk = B.ps_swap_out(ctx, fb["swap_out_dev_blocks"], fb["swap_out_host_slots"], -1, cache, host, side_out)
        if n_out:
            out_tickets.append((fb["round"], tk))
        now += fb["t_batch"]
    for _, tk in out_tickets:
        B.ps_ticket_wait(ctx, tk)
    torch.cuda.synchronize()
    print("steps", steps, seen, "worst abs err %.4g" % worst)
    assert seen["evicted"] > 0 and seen["swap_in"] > 0 and seen["swap_out"] > 0
    B.ps_destroy(ctx)
    B.ps_sched_destroy(sched)
