"""Oracle B: TDG gain, batch latency estimator, SlideBatching batch former, copy budget.

TEST INFRASTRUCTURE ONLY.  Follows, in the paper's order and notation:
  * Eq. 3 (Sec. 2)            token-level deadline-aware gain  f_TDG, deadline_{r,i}, w_r(i)
  * Eqs. 4-7 (Sec. 4.1)       T~_p = a_p l_q^2 + b_p l_q l_kv + c_p l_q,  T~_d = a_d l_kv + b_d,
                              T_pd(B) = sum T~ + t_c
  * Alg. 1 + Eq. 8 (Sec. 4.2) SlideBatching: metrics, t_budget = max(t_min, eta), URGENT/NORMAL
                              split by remain < gamma * phi(Q), ordering, greedy admission
  * Sec. 4.2 "Starvation Prevention", Sec. 4.3 "Eviction Policy", "Asynchronous Offloading",
    "Adaptive Copy-Budget Control", "Put it Together" (partial-copy rule).

All times are integer picoseconds; products are exact Python integers; divisions floor.
(The paper works in reals; integer time is what lets two independent implementations agree
bit for bit.)  Where the paper is silent the reading taken is written next to the step;
parity of those readings is "unpinned" by the paper -- they are pinned only by the
invariants and closed forms in tests/test_oracle_slidebatching.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------- Eq. 3: TDG
def deadline(i: int, ttft_slo: int, tpot_slo: int) -> int:
    """deadline_{r,i} = TTFT_SLO + (i-1) TPOT_SLO, measured from the request's arrival."""
    return ttft_slo + (i - 1) * tpot_slo


def token_weight(i: int, w_first: int, w_decode: int, w_class: int) -> int:
    """w_r(i) = w_p * w_{p(r)} for the first token, w_d * w_{p(r)} afterwards."""
    return (w_first if i == 1 else w_decode) * w_class


def tdg_gain(token_times: Sequence[int], ttft_slo: int, tpot_slo: int,
             w_first: int, w_decode: int, w_class: int) -> int:
    """f_TDG(r) = sum_i w_r(i) * 1[t_{r,i} < deadline_{r,i}]; times relative to arrival."""
    return sum(token_weight(i, w_first, w_decode, w_class)
               for i, t in enumerate(token_times, start=1) if t < deadline(i, ttft_slo, tpot_slo))


def ideal_gain(n_out: int, w_first: int, w_decode: int, w_class: int) -> int:
    """Gain when every one of the n_out tokens is on time (reading: the paper's Ideal_Gain,
    Sec. 5.1 Metrics, is not spelled out)."""
    return sum(token_weight(i, w_first, w_decode, w_class) for i in range(1, n_out + 1))


def slo_attained(token_times: Sequence[int], ttft_slo: int, tpot_slo: int) -> bool:
    """Both TTFT and mean TPOT strictly below their SLOs (Sec. 5.1 Metrics)."""
    if not token_times:
        return False
    if not token_times[0] < ttft_slo:
        return False
    n = len(token_times)
    return n == 1 or (token_times[-1] - token_times[0]) < tpot_slo * (n - 1)


# ----------------------------------------------------------------------------- config
@dataclass
class SchedConfig:
    class_weight: List[int]            # w_{p}, index p-1 (p = 1 is the highest class)
    ttft_slo: int
    tpot_slo: int
    w_first: int = 4                   # w_p in Eq. 3
    w_decode: int = 1                  # w_d
    a_p: int = 0
    b_p: int = 0
    c_p: int = 0
    a_d: int = 0
    b_d: int = 0
    t_c: int = 0
    eta: int = 0
    tau: int = 0
    gamma_num: int = 9
    gamma_den: int = 10
    beta_num: int = 2
    beta_den: int = 1
    rho_num: int = 9                   # "close to the starvation threshold" = waited >= rho * tau
    rho_den: int = 10
    t_block: int = 1
    block_tokens: int = 16
    n_off_base: int = 8                # offload threshold of class 1; halves per class, floor 1
    order_policy: int = 0              # 0: Alg. 1 line 13 + starvation rule; 1: arrival order only (the
                                       # first-come-first-served arm the paper compares against, Sec. 5)

    def n_off(self, prio: int) -> int:
        return max(1, self.n_off_base >> (prio - 1))


# ----------------------------------------------------------------------------- Eqs. 4-7
def t_prefill(cfg: SchedConfig, l_q: int, l_kv: int) -> int:
    return cfg.a_p * l_q * l_q + cfg.b_p * l_q * l_kv + cfg.c_p * l_q


def t_decode(cfg: SchedConfig, l_kv: int) -> int:
    return cfg.a_d * l_kv + cfg.b_d


def t_batch_estimate(cfg: SchedConfig, prefills: Sequence[Tuple[int, int]], decodes: Sequence[int]) -> int:
    """T_pd(B): prefills are (l_q, l_kv) pairs, decodes are l_kv values."""
    return sum(t_prefill(cfg, a, b) for a, b in prefills) + sum(t_decode(cfg, l) for l in decodes) + cfg.t_c


def max_chunk(cfg: SchedConfig, l_q: int, l_kv: int, T: int) -> int:
    """GetMaxChunk for a prefill: the largest c in [0, l_q] whose estimated cost fits in T.
    Plain scan over every candidate (vectorised)."""
    if l_q <= 0 or T < 0:
        return 0
    assert t_prefill(cfg, l_q, l_kv) < 2 ** 62          # int64 is enough for every candidate
    xs = np.arange(l_q + 1, dtype=np.int64)
    cost = cfg.a_p * xs * xs + cfg.b_p * xs * l_kv + cfg.c_p * xs
    return int(np.nonzero(cost <= T)[0].max())


# ----------------------------------------------------------------------------- Eq. 8
def phi(t_budget: int, t_c: int, sum_exec: int) -> int:
    """phi(Q) = t_budget / (t_budget - t_c) * sum exec   (floored)."""
    assert t_budget > t_c
    return (t_budget * sum_exec) // (t_budget - t_c)


# ----------------------------------------------------------------------------- copy budget
def copy_budget(cfg: SchedConfig, t_budget: int, t_fwd_min: int, b_missing: int) -> int:
    """Adaptive copy-budget control (Sec. 4.3), the three cases in the paper's order.
    Reading of case 2(ii): blocks that are not copied are recomputed, so the batch latency
    as a function of the budget is Lat(B) = T_fwd^min + (B_missing - B) * s_blk * c_p, which
    falls towards T_fwd^min as B grows while the transfer time B * t_block rises; the answer
    is the largest B whose transfer time does not exceed Lat(B).  Equality in the case
    conditions (unassigned in the text) goes to the earlier case."""
    t_trans_max = b_missing * cfg.t_block
    if t_fwd_min >= t_budget:
        return t_budget // cfg.t_block
    if t_fwd_min >= t_trans_max:
        return b_missing
    best = 0
    for B in range(b_missing + 1):           # plain scan; the library uses bisection
        if B * cfg.t_block <= t_fwd_min + (b_missing - B) * cfg.block_tokens * cfg.c_p:
            best = B
    return best


# ----------------------------------------------------------------------------- state
@dataclass
class Request:
    rid: int
    arrival: int
    prio: int
    prompt_len: int
    out_len: int
    computed: int = 0                  # tokens whose KV exists (device, or host if evicted)
    generated: int = 0                 # output tokens delivered
    last_sched: int = 0
    dev_blocks: List[int] = field(default_factory=list)     # logical order
    host_slots: List[int] = field(default_factory=list)     # host copies of logical blocks 0..n-1 (issued)
    host_round: List[int] = field(default_factory=list)     # scheduling round that issued each of them
    token_times: List[int] = field(default_factory=list)    # relative to arrival

    @property
    def need(self) -> int:
        """Tokens whose KV must exist before the next output token can be produced."""
        return self.prompt_len + self.generated

    @property
    def b_miss(self) -> int:
        """max(0, b_host - b_device): blocks that exist only on the host."""
        return max(0, len(self.host_slots) - len(self.dev_blocks))


@dataclass
class StepResult:
    now: int
    round: int = 0                                     # 1-based count of form_batch calls; names this round's offloads
    t_budget: int = 0
    phi: int = 0
    b_copy: int = 0
    t_batch: int = 0                                   # T_pd(B); 0 if the queue was empty
    order: List[int] = field(default_factory=list)     # sorted queue (request ids)
    urgent: List[int] = field(default_factory=list)
    batch: List[Tuple[int, int, int]] = field(default_factory=list)  # (rid, l_q, kv_len after)
    tables: List[List[int]] = field(default_factory=list)            # device block ids per member
    prios: List[int] = field(default_factory=list)
    swap_in: List[Tuple[int, int]] = field(default_factory=list)     # (host_slot, dev_block)
    swap_out: List[Tuple[int, int]] = field(default_factory=list)    # (dev_block, host_slot)
    evicted: List[int] = field(default_factory=list)
    dropped_pending: int = 0                           # host copies still in flight that evictions discarded
    emitted: List[Tuple[int, int]] = field(default_factory=list)     # (rid, token index)
    finished: List[int] = field(default_factory=list)


class SlideBatcher:
    """Single-instance PD co-located engine state + Alg. 1.

    Block pools are LIFO stacks.  ``dev_free_order[0]`` is handed out first.  Blocks of a
    request are released in logical order (so its last block is reused first)."""

    def __init__(self, cfg: SchedConfig, dev_free_order: Sequence[int], host_free_order: Sequence[int]):
        assert cfg.eta > cfg.t_c, "eta must exceed t_c (Eq. 8 denominator)"
        self.cfg = cfg
        self.dev_free = list(reversed([int(x) for x in dev_free_order]))
        self.host_free = list(reversed([int(x) for x in host_free_order]))
        self.n_dev = len(self.dev_free)
        self.n_host = len(self.host_free)
        self.reqs: Dict[int, Request] = {}
        self.finished_requests: Dict[int, Request] = {}
        self.round = 0                 # scheduling rounds so far
        self.offloads_done_upto = 0    # every offload issued in a round <= this has completed

    # -- Sec. 4.3 "Asynchronous Offloading": the copy thread reports completion
    def offloads_done(self, upto_round: int) -> None:
        """The device-to-host copies issued by rounds <= upto_round have all landed (copies on the
        offload stream complete in issue order, so a watermark is enough)."""
        self.offloads_done_upto = max(self.offloads_done_upto, int(upto_round))

    def confirmed(self, r: Request) -> int:
        """Leading host copies of r whose transfer is known to be complete."""
        n = 0
        while n < len(r.host_round) and r.host_round[n] <= self.offloads_done_upto:
            n += 1
        return n

    # -- queue
    def add_request(self, rid: int, arrival: int, prio: int, prompt_len: int, out_len: int) -> None:
        assert rid not in self.reqs and 1 <= prio <= len(self.cfg.class_weight)
        assert prompt_len >= 1 and out_len >= 1
        self.reqs[rid] = Request(rid, arrival, prio, prompt_len, out_len, last_sched=arrival)

    # -- Alg. 1, lines 2-6
    def _metrics(self, r: Request, now: int):
        cfg = self.cfg
        l_q = r.need - r.computed
        if r.generated >= 1 and l_q == 1:
            ex = t_decode(cfg, r.need)          # l_kv of a decode = its context incl. this token
        else:
            ex = t_prefill(cfg, l_q, r.computed)  # whole remaining prompt (the chunk is chosen later)
        i = r.generated + 1
        remain = deadline(i, cfg.ttft_slo, cfg.tpot_slo) - (now - r.arrival)
        w = token_weight(i, cfg.w_first, cfg.w_decode, cfg.class_weight[r.prio - 1])
        return ex, remain, w

    def _evict(self, v: Request, res: StepResult) -> None:
        """Free every device block of v at once (Sec. 4.3, Asynchronous Offloading: evict directly
        and discard the pending transfer, no on-demand synchronisation).  Host copies whose transfer
        has completed stay; a copy still in flight is discarded (its host slot is released, in
        logical order) and the tokens it would have covered, like those never offloaded, are
        recomputed."""
        for b in v.dev_blocks:
            self.dev_free.append(b)
        v.dev_blocks = []
        conf = self.confirmed(v)
        for s in v.host_slots[conf:]:
            self.host_free.append(s)
        res.dropped_pending += len(v.host_slots) - conf
        v.host_slots = v.host_slots[:conf]
        v.host_round = v.host_round[:conf]
        v.computed = min(v.computed, conf * self.cfg.block_tokens)
        res.evicted.append(v.rid)

    def form_batch(self, now: int) -> StepResult:
        cfg, blk = self.cfg, self.cfg.block_tokens
        self.round += 1
        res = StepResult(now=now, round=self.round)
        Q = [r for r in self.reqs.values() if r.arrival <= now]
        if not Q:
            return res
        # lines 1-6: per-request metrics and t_min
        met = {r.rid: self._metrics(r, now) for r in Q}
        t_min = min(m[1] for m in met.values())
        # line 7
        t_budget = max(t_min, cfg.eta)
        # lines 8-12 with Eq. 8
        sum_exec = sum(m[0] for m in met.values())
        ph = phi(t_budget, cfg.t_c, sum_exec)
        urgent = {r.rid for r in Q if met[r.rid][1] * cfg.gamma_den < cfg.gamma_num * ph}
        # line 13 + starvation rule: starving first (longest wait first), then URGENT by
        # density descending, then NORMAL by remain ascending; ties by arrival, then id.
        starving = [r for r in Q if now - r.last_sched > cfg.tau]
        st_ids = {r.rid for r in starving}
        starving.sort(key=lambda r: (-(now - r.last_sched), r.arrival, r.rid))
        urg = [r for r in Q if r.rid in urgent and r.rid not in st_ids]
        urg.sort(key=lambda r: (-Fraction(met[r.rid][2], max(met[r.rid][0], 1)), r.arrival, r.rid))
        nor = [r for r in Q if r.rid not in urgent and r.rid not in st_ids]
        nor.sort(key=lambda r: (met[r.rid][1], r.arrival, r.rid))
        order = starving + urg + nor
        if cfg.order_policy == 1:
            order = sorted(Q, key=lambda r: (r.arrival, r.rid))
        # line 14
        t_fwd_min = cfg.t_c + sum_exec
        b_missing = sum(r.b_miss for r in Q)
        b_rem = copy_budget(cfg, t_budget, t_fwd_min, b_missing)
        res.t_budget, res.phi, res.b_copy = t_budget, ph, b_rem
        res.order = [r.rid for r in order]
        res.urgent = [r.rid for r in order if r.rid in urgent]
        # lines 15-23
        t_batch = cfg.t_c
        members: List[Tuple[Request, int]] = []
        in_batch = set()
        evicted_now = set()
        idx = 0
        while idx < len(order) and t_batch < t_budget:
            r = order[idx]
            idx += 1
            if r.rid in evicted_now:
                continue
            T = t_budget - t_batch
            miss = r.b_miss
            if miss > 0:
                k = miss if b_rem >= miss else b_rem
                comp = k * blk                     # blocks beyond the copied prefix are recomputed
            else:
                k, comp = 0, r.computed
            partial = miss > 0 and k < miss
            l_q = r.need - comp
            is_dec = r.generated >= 1 and l_q == 1
            if is_dec:
                c, t = 1, t_decode(cfg, r.need)    # a decode token is atomic
            else:
                c = max_chunk(cfg, l_q, comp, T)
                if c == 0:
                    continue
                t = t_prefill(cfg, c, comp)
            if partial:
                # partial copy only if it still finishes the request's outstanding tokens, or
                # the progress is more than beta times the tokens left to recompute
                ok = (c == l_q) or (c * cfg.beta_den > cfg.beta_num * (miss - k) * blk)
                if not ok:
                    continue
            held = len(r.dev_blocks)
            want = -(-(comp + c) // blk) - held
            if want > len(self.dev_free):
                # evict from the tail of the sorted queue, never a near-starved request
                j = len(order) - 1
                while want > len(self.dev_free) and j >= idx:
                    v = order[j]
                    j -= 1
                    if v.rid in in_batch or v.rid in evicted_now or not v.dev_blocks:
                        continue
                    if (now - v.last_sched) * cfg.rho_den >= cfg.rho_num * cfg.tau:
                        continue
                    self._evict(v, res)
                    evicted_now.add(v.rid)
            if want > len(self.dev_free):
                c_fit = (held + len(self.dev_free)) * blk - comp
                if is_dec or c_fit <= 0:
                    break                           # "memory is enough" is false
                c = min(c, c_fit)
                t = t_prefill(cfg, c, comp)
                want = -(-(comp + c) // blk) - held
            # commit
            if miss > 0:
                new_dev = [self.dev_free.pop() for _ in range(k)]
                for b in range(k):
                    res.swap_in.append((r.host_slots[b], new_dev[b]))
                for s in r.host_slots[k:]:
                    self.host_free.append(s)
                r.host_slots = r.host_slots[:k]
                r.host_round = r.host_round[:k]
                r.dev_blocks = new_dev
                r.computed = comp
                b_rem -= k
                want -= k
            for _ in range(want):
                r.dev_blocks.append(self.dev_free.pop())
            r.computed += c
            r.last_sched = now
            t_batch += t
            members.append((r, c))
            in_batch.add(r.rid)
        res.t_batch = t_batch if members else 0
        # what the attention layer receives, in admission order
        for r, c in members:
            res.batch.append((r.rid, c, r.computed))
            res.tables.append(list(r.dev_blocks[: -(-r.computed // blk)]))
            res.prios.append(r.prio)
        # token delivery at now + T_pd(B); completion
        done_at = now + t_batch
        for r, c in members:
            if r.computed == r.need:
                r.generated += 1
                r.token_times.append(done_at - r.arrival)
                res.emitted.append((r.rid, r.generated))
                if r.generated == r.out_len:
                    for b in r.dev_blocks:
                        self.dev_free.append(b)
                    for s in r.host_slots:
                        self.host_free.append(s)
                    r.dev_blocks, r.host_slots, r.host_round = [], [], []
                    res.finished.append(r.rid)
        for rid in res.finished:
            self.finished_requests[rid] = self.reqs.pop(rid)
        # asynchronous offload trigger: every n_off^r newly completed full blocks of r
        for r, c in members:
            if r.rid not in self.reqs:
                continue
            full = r.computed // blk
            pending = full - len(r.host_slots)
            if pending >= cfg.n_off(r.prio) and len(self.host_free) >= pending:
                for b in range(len(r.host_slots), full):
                    s = self.host_free.pop()
                    r.host_slots.append(s)
                    r.host_round.append(self.round)
                    res.swap_out.append((r.dev_blocks[b], s))
        return res


# ----------------------------------------------------------------------------- trace driver
def simulate(cfg: SchedConfig, trace, dev_free_order, host_free_order, max_steps: int,
             on_step=None):
    """Virtual-clock run: requests join the queue at their arrival; the clock advances by
    T_pd(B) per step, or jumps to the next arrival when the queue is empty.  The offload thread
    is modelled on the same clock: the copies a round issues start when its batch has been
    computed and the earlier copies are through, take t_block per block (the paper profiles
    one per-block copy time), and are reported complete at the first round that starts at or
    after their end."""
    sb = SlideBatcher(cfg, dev_free_order, host_free_order)
    pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
    nxt = 0
    now = 0
    steps: List[StepResult] = []
    inflight: List[Tuple[int, int]] = []      # (round, completion time) of offload lists, oldest first
    copy_free_at = 0
    while len(steps) < max_steps:
        while nxt < len(pending) and pending[nxt].arrival_ps <= now:
            p = pending[nxt]
            sb.add_request(p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
            nxt += 1
        if not sb.reqs:
            if nxt >= len(pending):
                break
            now = pending[nxt].arrival_ps
            continue
        while inflight and inflight[0][1] <= now:
            sb.offloads_done(inflight.pop(0)[0])
        res = sb.form_batch(now)
        steps.append(res)
        if res.swap_out:
            copy_free_at = max(copy_free_at, now + res.t_batch) + len(res.swap_out) * cfg.t_block
            inflight.append((res.round, copy_free_at))
        if on_step is not None:
            on_step(sb, res)
        now += res.t_batch if res.t_batch > 0 else cfg.eta
    return sb, steps


def trace_gain(sb: SlideBatcher):
    """(sum f_TDG, Ideal_Gain, SLO-attained count, finished count) over finished requests."""
    cfg = sb.cfg
    g = ideal = ok = 0
    for r in sb.finished_requests.values():
        wc = cfg.class_weight[r.prio - 1]
        g += tdg_gain(r.token_times, cfg.ttft_slo, cfg.tpot_slo, cfg.w_first, cfg.w_decode, wc)
        ideal += ideal_gain(r.out_len, cfg.w_first, cfg.w_decode, wc)
        ok += slo_attained(r.token_times, cfg.ttft_slo, cfg.tpot_slo)
    return g, ideal, ok, len(sb.finished_requests)
