"""Pins for oracle B (TDG, estimator, SlideBatching, copy budget).  CPU only.

Closed forms and hand examples are derived by hand from the paper's formulas (Eq. 3, Eqs. 4-8,
Sec. 4.3); the interplay of admission, eviction and partial reload is not pinned by any printed
example in the paper ("parity unpinned") and is held only by invariants here."""
import itertools

import numpy as np
import pytest

from oracle import slidebatching as S
from paper_2512_12928_amd import workloads as W

MS, US, NS = 10 ** 9, 10 ** 6, 10 ** 3


def base_cfg(**kw):
    L = 36
    d = dict(class_weight=[4, 2, 1], ttft_slo=2000 * MS, tpot_slo=100 * MS, w_first=4, w_decode=1,
             a_p=234, b_p=13 * L, c_p=50 * NS * L, a_d=730 * L, b_d=1 * US * L, t_c=2 * MS,
             eta=10 * MS, tau=30_000 * MS, t_block=43200 * NS // 1000 * 1000)
    d.update(kw)
    return S.SchedConfig(**d)


# ---------------------------------------------------------------- Eq. 3
def test_tdg_hand_example():
    # TTFT_SLO 1.0 s, TPOT_SLO 0.1 s -> deadlines 1.0/1.1/1.2/1.3/1.4 s; tokens at .90/1.05/1.25/1.29/1.45 s
    # on time: yes yes no yes no; w_p=3, w_d=1, class weight 2 -> 2*(3+1+0+1+0) = 10; ideal 2*(3+4) = 14
    times = [900 * MS, 1050 * MS, 1250 * MS, 1290 * MS, 1450 * MS]
    assert [S.deadline(i, 1000 * MS, 100 * MS) for i in range(1, 6)] == [1000 * MS, 1100 * MS, 1200 * MS, 1300 * MS, 1400 * MS]
    assert S.tdg_gain(times, 1000 * MS, 100 * MS, 3, 1, 2) == 10
    assert S.ideal_gain(5, 3, 1, 2) == 14


def test_tdg_deadline_is_strict_and_early_tokens_never_hurt():
    assert S.tdg_gain([1000 * MS], 1000 * MS, 100 * MS, 3, 1, 1) == 0      # t == deadline earns nothing
    assert S.tdg_gain([1000 * MS - 1], 1000 * MS, 100 * MS, 3, 1, 1) == 3
    rng = np.random.default_rng(0)
    for _ in range(50):
        t = np.sort(rng.integers(0, 3000, 8)) * MS
        g = S.tdg_gain(list(t), 1000 * MS, 200 * MS, 3, 1, 2)
        t2 = t.copy(); t2[rng.integers(0, 8)] -= 150 * MS
        assert S.tdg_gain(list(t2), 1000 * MS, 200 * MS, 3, 1, 2) >= g


def test_slo_attainment_needs_both():
    assert S.slo_attained([900 * MS, 950 * MS, 1000 * MS], 1000 * MS, 100 * MS)
    assert not S.slo_attained([1000 * MS, 1010 * MS], 1000 * MS, 100 * MS)          # TTFT not strictly below
    assert not S.slo_attained([100 * MS, 300 * MS, 500 * MS], 1000 * MS, 200 * MS)  # mean TPOT == SLO


# ---------------------------------------------------------------- Eqs. 4-7
def test_estimator_closed_forms():
    cfg = base_cfg(a_p=3, b_p=5, c_p=7, a_d=11, b_d=13, t_c=17)
    assert S.t_prefill(cfg, 10, 100) == 3 * 100 + 5 * 1000 + 70
    assert S.t_decode(cfg, 100) == 1113
    assert S.t_batch_estimate(cfg, [(10, 100), (2, 0)], [100, 1]) == 5370 + (12 + 14) + 1113 + 24 + 17


@pytest.mark.parametrize("l_q,l_kv,T", [(1, 0, 0), (100, 0, 10 ** 9), (8192, 4096, 3 * 10 ** 9), (500, 77, 123456789), (64, 0, 10 ** 15)])
def test_max_chunk_is_the_boundary(l_q, l_kv, T):
    cfg = base_cfg()
    c = S.max_chunk(cfg, l_q, l_kv, T)
    assert 0 <= c <= l_q and S.t_prefill(cfg, c, l_kv) <= T
    assert c == l_q or S.t_prefill(cfg, c + 1, l_kv) > T


# ---------------------------------------------------------------- Eq. 8
def test_phi_closed_form():
    # t_budget 50 ms, t_c 5 ms, sum exec 90 ms: 90/45 = 2 batches of 50 ms = 100 ms
    assert S.phi(50 * MS, 5 * MS, 90 * MS) == 100 * MS


# ---------------------------------------------------------------- copy budget
def test_copy_budget_three_cases():
    cfg = base_cfg(t_block=1000, c_p=10)
    # (1) forward time already exceeds the budget: floor(t_budget / t_block)
    assert S.copy_budget(cfg, t_budget=10_500, t_fwd_min=20_000, b_missing=500) == 10
    # (2i) compute dominates transfer: copy everything
    assert S.copy_budget(cfg, t_budget=10 ** 6, t_fwd_min=50_000, b_missing=40) == 40
    # (2ii) closed form floor((T_fwd + B_miss*16*c_p) / (t_block + 16*c_p)), clipped
    for fwd, miss in [(5_000, 40), (100, 7), (39_999, 40), (0, 3)]:
        want = min(miss, (fwd + miss * 16 * 10) // (1000 + 16 * 10))
        assert S.copy_budget(cfg, 10 ** 6, fwd, miss) == want
    # monotone in t_fwd_min
    vals = [S.copy_budget(cfg, 10 ** 6, f, 40) for f in range(0, 50_000, 777)]
    assert vals == sorted(vals)


# ---------------------------------------------------------------- Alg. 1 behaviours
def queue(cfg, specs, now=0, M=4096):
    """specs: (arrival, prio, prompt_len, out_len)."""
    sb = S.SlideBatcher(cfg, list(range(M)), list(range(2 * M)))
    for i, (a, p, pl, ol) in enumerate(specs):
        sb.add_request(i, a, p, pl, ol)
    return sb


def test_t_budget_is_max_of_tmin_and_eta_including_negative_tmin():
    cfg = base_cfg()
    sb = queue(cfg, [(0, 1, 10, 4)])
    assert sb.form_batch(now=1990 * MS).t_budget == cfg.eta          # t_min = 10 ms = eta
    sb = queue(cfg, [(0, 1, 10, 4)])
    assert sb.form_batch(now=1500 * MS).t_budget == 500 * MS         # t_min above eta
    sb = queue(cfg, [(0, 1, 10, 4)])
    assert sb.form_batch(now=2500 * MS).t_budget == cfg.eta          # t_min negative


def test_gamma_zero_is_edf_and_gamma_huge_is_density_order():
    specs = [(0, 3, 900, 4), (50 * MS, 1, 3000, 4), (100 * MS, 2, 200, 4), (120 * MS, 1, 1500, 4), (10 * MS, 3, 50, 4)]
    now = 200 * MS
    edf = queue(base_cfg(gamma_num=0), specs).form_batch(now)
    assert edf.urgent == [] and edf.order == [0, 4, 1, 2, 3]         # remain ascending == arrival ascending
    cfg = base_cfg(gamma_num=10 ** 9)
    dens = queue(cfg, specs).form_batch(now)
    assert sorted(dens.urgent) == [0, 1, 2, 3, 4]
    w = {0: 1, 1: 4, 2: 2, 3: 4, 4: 1}
    key = {i: (w[i] * 4) / S.t_prefill(cfg, specs[i][2], 0) for i in range(5)}
    assert dens.order == sorted(range(5), key=lambda i: -key[i])


def test_single_class_density_order_is_shortest_exec_first():
    cfg = base_cfg(class_weight=[1], gamma_num=10 ** 9)
    specs = [(0, 1, 700, 2), (0, 1, 30, 2), (0, 1, 5000, 2), (0, 1, 31, 2)]
    assert queue(cfg, specs).form_batch(10 * MS).order == [1, 3, 0, 2]


def test_low_load_admits_everything():
    cfg = base_cfg()
    specs = [(0, 1 + i % 3, 20 + 7 * i, 3) for i in range(12)]
    res = queue(cfg, specs).form_batch(1 * MS)
    assert sorted(r for r, _, _ in res.batch) == list(range(12))
    assert all(lq == specs[r][2] for r, lq, _ in res.batch)          # whole prompts, no chunking


def test_larger_gamma_never_shrinks_urgent_set():
    specs = [(i * 30 * MS, 1 + i % 3, 400 + 300 * i, 4) for i in range(10)]
    prev = set()
    for g in (0, 3, 9, 30, 300):
        u = set(queue(base_cfg(gamma_num=g), specs).form_batch(1900 * MS).urgent)
        assert prev <= u
        prev = u


def test_starving_request_goes_to_head():
    cfg = base_cfg(tau=500 * MS, gamma_num=10 ** 9)
    specs = [(0, 3, 8000, 2), (900 * MS, 1, 100, 2), (950 * MS, 1, 120, 2)]
    res = queue(cfg, specs).form_batch(1000 * MS)
    assert res.order[0] == 0 and res.batch[0][0] == 0


def test_greedy_matches_fractional_knapsack_lp():
    """Prefill-only, all-URGENT, memory-unconstrained, linear cost: admitted value equals the LP
    optimum of the fractional knapsack up to one token of the last (split) item."""
    linprog = pytest.importorskip("scipy.optimize").linprog
    rng = np.random.default_rng(5)
    for trial in range(20):
        n = int(rng.integers(2, 9))
        cfg = base_cfg(a_p=0, b_p=0, c_p=1 * US, t_c=1 * MS, eta=5 * MS, gamma_num=10 ** 12,
                       ttft_slo=5 * MS, class_weight=[8, 4, 2, 1])
        specs = [(0, int(rng.integers(1, 5)), int(rng.integers(200, 3000)), 2) for _ in range(n)]
        sb = queue(cfg, specs)
        res = sb.form_batch(0)
        assert res.t_budget == 5 * MS and sorted(res.urgent) == list(range(n))
        val = {i: 4 * cfg.class_weight[specs[i][1] - 1] for i in range(n)}
        got = sum(val[r] * lq / specs[r][2] for r, lq, _ in res.batch)
        size = np.array([specs[i][2] * cfg.c_p for i in range(n)], dtype=float)
        lp = linprog(-np.array([val[i] for i in range(n)], dtype=float), A_ub=size[None], b_ub=[res.t_budget - cfg.t_c],
                     bounds=[(0, 1)] * n)
        best = -lp.fun
        one_token = max(val[i] / specs[i][2] for i in range(n))
        assert best - one_token - 1e-9 <= got <= best + 1e-9


# ---------------------------------------------------------------- invariants on a preemption-heavy trace
def test_invariants_hold_under_preemption():
    cfg = base_cfg(tau=3000 * MS)
    tr = W.make_trace(2, 250, rate_per_s=200.0, seed=1, prompt_mean=600, prompt_max=3000, out_mean=40, out_max=200)
    rng = np.random.default_rng(1)
    M = 300
    seen = dict(evict=0, swap_in=0, swap_out=0, partial=0)

    def check(sb, res):
        blk = cfg.block_tokens
        held = [b for r in sb.reqs.values() for b in r.dev_blocks]
        assert len(held) == len(set(held)) and not (set(held) & set(sb.dev_free))
        assert len(held) + len(sb.dev_free) == M
        hh = [s for r in sb.reqs.values() for s in r.host_slots]
        assert len(hh) == len(set(hh)) and not (set(hh) & set(sb.host_free)) and len(hh) + len(sb.host_free) == 2 * M
        assert len(res.swap_in) <= res.b_copy
        ids = [r for r, _, _ in res.batch]
        assert len(ids) == len(set(ids)) and set(ids) <= set(res.order) and not (set(ids) & set(res.evicted))
        for (rid, lq, kv), tab in zip(res.batch, res.tables):
            assert 1 <= lq <= kv and len(tab) == -(-kv // blk) and len(set(tab)) == len(tab)
        all_tab = [b for t in res.tables for b in t]
        assert len(all_tab) == len(set(all_tab))
        dst = [d for _, d in res.swap_in]
        assert len(dst) == len(set(dst)) and set(dst) <= set(all_tab)       # reloaded blocks belong to batch members
        src = [d for d, _ in res.swap_out]
        assert len(src) == len(set(src))
        for r in sb.reqs.values():
            assert len(r.dev_blocks) == 0 or len(r.dev_blocks) >= -(-r.computed // blk)
            assert r.computed <= r.need
        seen["evict"] += len(res.evicted); seen["swap_in"] += len(res.swap_in); seen["swap_out"] += len(res.swap_out)

    sb, steps = S.simulate(cfg, tr, rng.permutation(M), rng.permutation(2 * M), 600, on_step=check)
    assert seen["evict"] > 0 and seen["swap_in"] > 0 and seen["swap_out"] > 0
    g, ideal, ok, n = S.trace_gain(sb)
    assert 0 <= g <= ideal and 0 <= ok <= n


def test_t_batch_equals_estimator_sum_without_eviction():
    cfg = base_cfg()
    tr = W.make_trace(2, 120, rate_per_s=30.0, seed=2, prompt_mean=400, prompt_max=2000, out_mean=30, out_max=100)
    emitted = set()

    def check(sb, res):
        if not res.batch:
            return
        pre = [(lq, kv - lq) for rid, lq, kv in res.batch if not (rid in emitted and lq == 1)]
        dec = [kv for rid, lq, kv in res.batch if rid in emitted and lq == 1]
        assert res.t_batch == S.t_batch_estimate(cfg, pre, dec)
        assert not res.evicted
        emitted.update(r for r, _ in res.emitted)

    S.simulate(cfg, tr, list(range(20000)), list(range(40000)), 500, on_step=check)


def test_eviction_takes_from_tail_and_spares_near_starved():
    cfg = base_cfg(tau=1000 * MS, gamma_num=10 ** 9, n_off_base=1)   # all URGENT: density order
    sb = S.SlideBatcher(cfg, list(range(12)), list(range(24)))
    sb.add_request(0, 0, 3, 64, 50)          # will hold 4 blocks
    sb.add_request(1, 0, 3, 64, 50)          # will hold 4 blocks
    r = sb.form_batch(0)
    assert sorted(x[0] for x in r.batch) == [0, 1] and len(sb.dev_free) == 4
    assert len(r.swap_out) == 8               # class 3, n_off = 1: every full block offloaded at once
    sb.offloads_done(r.round)                 # the copy thread reports those eight copies complete
    # make request 1 near-starved (waited >= 0.9 tau), request 0 recently scheduled
    sb.reqs[0].last_sched = 950 * MS
    sb.reqs[1].last_sched = 50 * MS
    sb.add_request(2, 940 * MS, 1, 7 * 16, 5)    # urgent newcomer needing 7 blocks, only 4 free
    res = sb.form_batch(960 * MS)
    assert res.order == [2, 0, 1]             # class-1 first token outweighs class-3 decode tokens
    assert res.evicted == [0]                 # the near-starved request 1 is spared, 0 is not
    assert sb.reqs[0].dev_blocks == [] and sb.reqs[0].computed == 64 and sb.reqs[0].b_miss == 4
    # when 0 comes back its 4 host blocks are reloaded, bounded by the copy budget
    sb.reqs[2].out_len = 1
    nxt = sb.form_batch(2000 * MS)
    assert len(nxt.swap_in) <= nxt.b_copy


# ---------------------------------------------------------------- hand-worked cases for the block-management readings
def test_offload_threshold_ladder_by_class():
    """n_off halves per class (8, 4, 2 for classes 1, 2, 3): a 96-token prompt (6 full blocks) is offloaded at
    once by class 3 and class 2, not yet by class 1."""
    cfg = base_cfg()
    assert [cfg.n_off(p) for p in (1, 2, 3, 4, 5)] == [8, 4, 2, 1, 1]
    sb = S.SlideBatcher(cfg, list(range(64)), list(range(64)))
    for rid, prio in ((0, 1), (1, 2), (2, 3)):
        sb.add_request(rid, 0, prio, 96, 40)
    res = sb.form_batch(0)
    out_by_req = {rid: [d for d, _ in res.swap_out if d in sb.reqs[rid].dev_blocks[:6]] for rid in (0, 1, 2)}
    assert len(out_by_req[0]) == 0 and len(out_by_req[1]) == 6 and len(out_by_req[2]) == 6
    # 32 decode steps later class 1 has 8 full blocks and offloads them in one go
    now = res.t_batch
    total = 0
    for _ in range(32):
        r = sb.form_batch(now)
        now += r.t_batch
        total += sum(1 for d, _ in r.swap_out if d in sb.reqs[0].dev_blocks)
    assert sb.reqs[0].computed == 128 and len(sb.reqs[0].host_slots) == 8 and total == 8


def test_decode_token_is_atomic_and_may_overshoot_budget():
    cfg = base_cfg(eta=3 * MS, t_c=2 * MS, ttft_slo=1 * MS, tpot_slo=1 * MS)   # every deadline already missed: t_budget = eta
    sb = S.SlideBatcher(cfg, list(range(16384)), list(range(64)))
    for rid in range(40):
        sb.add_request(rid, 0, 1, 16, 400)
    sb.form_batch(0)                                # prefill: 40 x 16 tokens
    # each request now holds a 4000-token context so that a decode costs 141 us: 8 of them exceed the 1 ms left
    for r in sb.reqs.values():
        r.prompt_len, r.computed = 4000, 4000
        r.dev_blocks = r.dev_blocks + [sb.dev_free.pop() for _ in range(250 - len(r.dev_blocks))]
    res = sb.form_batch(10 * MS)
    n = len(res.batch)
    per = S.t_decode(cfg, 4001)
    assert res.t_budget == cfg.eta and all(lq == 1 for _, lq, _ in res.batch)
    assert cfg.t_c + (n - 1) * per < cfg.eta <= cfg.t_c + n * per       # stops right after crossing the budget
    assert res.t_batch == cfg.t_c + n * per


def test_partial_reload_rule_and_recompute():
    """A victim with 8 host blocks when the copy budget works out to 0 (copying a block costs far more than
    recomputing it): nothing is reloaded, the host copies are released and the request recomputes from token
    0 -- allowed because the chunk finishes the request's outstanding tokens."""
    cfg = base_cfg(t_block=10 * MS, eta=35 * MS, ttft_slo=1 * MS, tpot_slo=1 * MS, n_off_base=1)
    sb = S.SlideBatcher(cfg, list(range(32)), list(range(32)))
    sb.add_request(0, 0, 2, 128, 50)
    r0 = sb.form_batch(0)
    assert len(r0.swap_out) == 8 and len(sb.reqs[0].host_slots) == 8
    victim = sb.reqs[0]
    for b in victim.dev_blocks:                     # evict by hand: device blocks back to the pool
        sb.dev_free.append(b)
    victim.dev_blocks = []
    victim.computed = 128
    res = sb.form_batch(1000 * MS)
    # case (1): T_fwd^min >= t_budget?  exec(decode, 129) + t_c = 2 ms + 3.4 us < 35 ms -> case 2; T_trans^max = 80 ms > T_fwd^min
    # -> case 2(ii): largest B with B*10ms <= T_fwd + (8-B)*16*c_p = 2.0394 ms + (8-B)*28.8us -> B = 0
    assert res.b_copy == 0 and res.swap_in == []
    # with budget 0 the request recomputes everything: allowed, the chunk (129 tokens) completes it
    assert res.batch == [(0, 129, 129)] and len(victim.dev_blocks) == 9
    # the 8 stale host copies were released, and the 8 recomputed full blocks were offloaded afresh (n_off = 1)
    assert len(res.swap_out) == 8 and len(victim.host_slots) == 8 and len(sb.host_free) == 32 - 8
    assert [d for d, _ in res.swap_out] == victim.dev_blocks[:8]


def test_partial_reload_is_refused_when_progress_is_too_small():
    """Same victim, but only 100 us of latency budget: the chunk that fits (55 tokens) neither finishes the
    request (129 outstanding) nor exceeds beta * (tokens left to recompute) = 2 * 8 * 16 -> the request is
    skipped this round and keeps its host copies."""
    roomy = base_cfg(t_block=10 * MS, eta=35 * MS, ttft_slo=1 * MS, tpot_slo=1 * MS, n_off_base=1)
    tight = base_cfg(t_block=10 * MS, eta=2 * MS + 100 * US, t_c=2 * MS, ttft_slo=1 * MS, tpot_slo=1 * MS, n_off_base=1)
    sb = S.SlideBatcher(roomy, list(range(32)), list(range(32)))
    sb.add_request(0, 0, 2, 128, 50)
    sb.form_batch(0)                                 # whole prompt, first token, 8 blocks offloaded
    victim = sb.reqs[0]
    assert victim.computed == 128 and victim.generated == 1 and len(victim.host_slots) == 8
    for b in victim.dev_blocks:                      # evict by hand
        sb.dev_free.append(b)
    victim.dev_blocks = []
    sb.cfg = tight
    res = sb.form_batch(1000 * MS)
    assert res.t_budget == tight.eta and res.b_copy == 0
    assert S.max_chunk(tight, 129, 0, 100 * US) == 55      # a_p c^2 + c_p c <= 100 us
    assert res.batch == [] and len(victim.host_slots) == 8 and victim.computed == 128 and res.t_batch == 0
    # with beta = 1/4 the same 55 tokens are enough progress (55 * 4 > 1 * 128): admitted, host copies released
    sb.cfg = base_cfg(t_block=10 * MS, eta=2 * MS + 100 * US, t_c=2 * MS, ttft_slo=1 * MS, tpot_slo=1 * MS,
                      n_off_base=1, beta_num=1, beta_den=4)
    res = sb.form_batch(1001 * MS)
    assert res.batch == [(0, 55, 55)] and res.swap_in == [] and len(victim.dev_blocks) == 4
