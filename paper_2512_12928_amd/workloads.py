"""Seeded synthetic inputs for the mixed-batch paged-attention step.

This module only *draws* inputs: shapes, context lengths, block tables, priorities and
N(0,1) tensors rounded to bf16.  It holds none of the method's arithmetic (no softmax,
no scheduling rule, no copy rule) and is the one module both the CPU oracle's tests and
the HIP path's tests/bench may import.  It imports neither of them.

The five workloads stand in for the paper's trace-driven runs (Sec. 5.1, "Datasets and
Workloads"): none of those datasets is reproduced; only their structure is borrowed
(Poisson arrivals, random priority assignment, a 2:1-style weight ladder).

bf16 tensors are carried as numpy ``uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 2512_12928_0  # seed of workload k is BASE_SEED + k


# --------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns uint16 bit patterns.
    NaN stays NaN (quiet)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """N(0,1) drawn in float32, rounded to bf16 bits."""
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


BF16_NAN = np.uint16(0x7FC0)


# --------------------------------------------------------------------------- shapes
@dataclass
class LayerShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    block_tokens: int = 16

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def block_bytes(self) -> int:  # K and V of one block, bf16
        return 2 * self.n_kv_heads * self.block_tokens * self.head_dim * 2


@dataclass
class MixedBatch:
    """One engine iteration's batch as the scheduler hands it to the attention layer:
    per request the number of new query tokens (1 = decode, >1 = prefill chunk), the
    cached length *including* these tokens, and its block table (CSR)."""
    shape: LayerShape
    n_device_blocks: int
    q_start: np.ndarray        # int32 [n_req+1]
    kv_len: np.ndarray         # int32 [n_req]
    bt_start: np.ndarray       # int32 [n_req+1]
    block_ids: np.ndarray      # int32 [sum ceil(kv_len/blk)]
    prio: np.ndarray           # uint8 [n_req] (1 = highest)
    name: str = ""
    seed: int = 0

    @property
    def n_req(self) -> int:
        return int(self.kv_len.shape[0])

    @property
    def n_tokens(self) -> int:
        return int(self.q_start[-1])

    def l_q(self, r: int) -> int:
        return int(self.q_start[r + 1] - self.q_start[r])

    def table(self, r: int) -> np.ndarray:
        return self.block_ids[self.bt_start[r]:self.bt_start[r + 1]]

    @property
    def decode_reqs(self) -> np.ndarray:
        lq = np.diff(self.q_start)
        return np.nonzero(lq == 1)[0]

    @property
    def prefill_reqs(self) -> np.ndarray:
        lq = np.diff(self.q_start)
        return np.nonzero(lq > 1)[0]

    def causal_pairs(self) -> int:
        """(query, key) pairs the prefill chunks attend over."""
        total = 0
        for r in self.prefill_reqs:
            lq = self.l_q(int(r))
            p = int(self.kv_len[r]) - lq
            total += lq * p + lq * (lq + 1) // 2
        return total

    def decode_kv_tokens(self) -> int:
        return int(self.kv_len[self.decode_reqs].astype(np.int64).sum())


def build_batch(shape: LayerShape, items: Sequence[Tuple[int, int]], prios: Sequence[int],
                rng: np.random.Generator, pool_factor: float = 1.25,
                n_device_blocks: Optional[int] = None, name: str = "", seed: int = 0,
                order: Optional[Sequence[int]] = None) -> MixedBatch:
    """items: (l_q, kv_len) per request.  Physical block ids are handed out from a seeded
    permutation of [0, M) so tables are neither contiguous nor monotone."""
    blk = shape.block_tokens
    if order is not None:
        items = [items[i] for i in order]
        prios = [prios[i] for i in order]
    lq = np.array([it[0] for it in items], dtype=np.int64)
    kv = np.array([it[1] for it in items], dtype=np.int64)
    assert (lq >= 1).all() and (kv >= lq).all()
    nblk = (kv + blk - 1) // blk
    need = int(nblk.sum())
    M = int(n_device_blocks) if n_device_blocks is not None else max(need + 1, int(np.ceil(need * pool_factor)))
    assert M >= need
    perm = rng.permutation(M).astype(np.int32)
    q_start = np.zeros(len(items) + 1, dtype=np.int32)
    q_start[1:] = np.cumsum(lq)
    bt_start = np.zeros(len(items) + 1, dtype=np.int32)
    bt_start[1:] = np.cumsum(nblk)
    return MixedBatch(shape=shape, n_device_blocks=M, q_start=q_start, kv_len=kv.astype(np.int32),
                      bt_start=bt_start, block_ids=perm[:need].copy(),
                      prio=np.asarray(prios, dtype=np.uint8), name=name, seed=seed)


def _lognormal_lengths(rng, n, mean, sigma, lo, hi):
    mu = np.log(mean) - 0.5 * sigma * sigma
    x = np.rint(rng.lognormal(mean=mu, sigma=sigma, size=n))
    return np.clip(x, lo, hi).astype(np.int64)


def _classes(rng, n, ratios):
    p = np.asarray(ratios, dtype=np.float64)
    p = p / p.sum()
    return (rng.choice(len(ratios), size=n, p=p) + 1).astype(np.uint8)


def make_workload(index: int, scale: float = 1.0, seed: Optional[int] = None) -> MixedBatch:
    """The five single-layer workloads (index 1..5).  ``scale`` < 1 shrinks request
    counts and context lengths proportionally (same structure) so that a CPU oracle can
    finish in seconds; scale == 1 is the full size that is timed."""
    seed = BASE_SEED + index if seed is None else seed
    rng = np.random.default_rng(seed)

    def sc(n, lo=1):
        return max(lo, int(round(n * scale)))

    if index == 1:
        shape = LayerShape(8, 2)
        items = [(1, 17), (1, 64), (1, 130), (1, 200), (64, 64)]
        prios = [1, 2, 1, 2, 1]
        return build_batch(shape, items, prios, rng, n_device_blocks=64, name="cfg1-tiny", seed=seed)
    if index in (2, 3):
        shape = LayerShape(32, 8)
        n_dec = sc(256, 4)
        kv = _lognormal_lengths(rng, n_dec, 1500 * max(scale, 0.05), 0.8, 16, sc(8192, 64))
        prios = list(_classes(rng, n_dec, (1, 2, 4)))
        items = [(1, int(x)) for x in kv]
        chunk = sc(512, 16)
        for p in (0, 1, 3, 7):  # chunk prefixes {0, 512, 1536, 3584} at full scale
            items.append((chunk, p * chunk + chunk))
        prios += list(_classes(rng, 4, (1, 2, 4)))
        nd = 40_000 if (index == 3 and scale == 1.0) else None
        return build_batch(shape, items, prios, rng, n_device_blocks=nd,
                           name="cfg%d-qwen3-8b" % index + ("-preempt" if index == 3 else ""), seed=seed)
    if index == 4:
        shape = LayerShape(32, 8)
        n_dec = sc(32, 2)
        lo, hi = sc(16384, 64), sc(32768, 128)
        kv = rng.integers(lo, hi + 1, size=n_dec)
        items = [(1, int(x)) for x in kv]
        prios = list(_classes(rng, n_dec, (1, 2, 4)))
        chunk = sc(4096, 32)
        items.append((chunk, lo + chunk))  # last chunk of a (lo + chunk)-token prompt
        prios.append(1)
        return build_batch(shape, items, prios, rng, pool_factor=1.1, name="cfg4-long-context", seed=seed)
    if index == 5:
        shape = LayerShape(64, 8)
        n_dec = sc(512, 4)
        kv = _lognormal_lengths(rng, n_dec, 2000 * max(scale, 0.05), 0.8, 16, sc(16384, 64))
        items = [(1, int(x)) for x in kv]
        prios = list(_classes(rng, n_dec, (1, 2, 4, 8)))
        chunk = sc(2048, 16)
        for p in (0, 1, 2, 4):  # prefixes {0, 2048, 4096, 8192} at full scale
            items.append((chunk, p * chunk + chunk))
        prios += [1, 2, 3, 4]
        return build_batch(shape, items, prios, rng, name="cfg5-llama-70b", seed=seed)
    raise ValueError("workload index must be 1..5")


# --------------------------------------------------------------------------- tensors
@dataclass
class StepTensors:
    """Logical (layout-free) tensors of one step: queries for every batch token and the
    full K/V history of every request, including this step's new rows at the tail."""
    q: np.ndarray                       # uint16 [n_tokens, Hq, d]
    k: List[np.ndarray] = field(default_factory=list)   # per request uint16 [kv_len, Hkv, d]
    v: List[np.ndarray] = field(default_factory=list)

    def new_rows(self, batch: MixedBatch):
        """K/V rows appended in this step, concatenated in batch token order."""
        ks, vs = [], []
        for r in range(batch.n_req):
            lq = batch.l_q(r)
            ks.append(self.k[r][-lq:])
            vs.append(self.v[r][-lq:])
        return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


def make_tensors(batch: MixedBatch, seed: Optional[int] = None) -> StepTensors:
    rng = np.random.default_rng((batch.seed if seed is None else seed) + 7919)
    s = batch.shape
    q = normal_bf16(rng, (batch.n_tokens, s.n_q_heads, s.head_dim))
    t = StepTensors(q=q)
    for r in range(batch.n_req):
        L = int(batch.kv_len[r])
        t.k.append(normal_bf16(rng, (L, s.n_kv_heads, s.head_dim)))
        t.v.append(normal_bf16(rng, (L, s.n_kv_heads, s.head_dim)))
    return t


# --------------------------------------------------------------------------- swap lists
def make_swap_lists(n: int, n_device_blocks: int, n_host_blocks: int, rng: np.random.Generator,
                    exclude_device: Optional[np.ndarray] = None, host_run: int = 1):
    """n distinct device block ids (avoiding ``exclude_device``) and n distinct host slots.  host_run > 1:
    the host slots come in runs of that many consecutive slots (a host pool handed out in extents, one
    per offloaded request), the runs themselves scattered; the device blocks stay scattered."""
    pool = np.arange(n_device_blocks, dtype=np.int32)
    if exclude_device is not None and len(exclude_device):
        mask = np.ones(n_device_blocks, dtype=bool)
        mask[np.asarray(exclude_device)] = False
        pool = pool[mask]
    assert len(pool) >= n and n_host_blocks >= n
    dev = rng.permutation(pool)[:n].astype(np.int32)
    if host_run <= 1:
        host = rng.permutation(n_host_blocks)[:n].astype(np.int32)
    else:
        n_runs = -(-n // host_run)
        assert n_host_blocks // host_run >= n_runs
        starts = rng.permutation(n_host_blocks // host_run)[:n_runs] * host_run
        host = (starts[:, None] + np.arange(host_run)[None, :]).reshape(-1)[:n].astype(np.int32)
    return dev, host


# --------------------------------------------------------------------------- request traces
@dataclass
class TraceRequest:
    rid: int
    arrival_ps: int
    prio: int
    prompt_len: int
    out_len: int


def make_trace(index: int, n_requests: int, rate_per_s: float, seed: Optional[int] = None,
               prompt_mean: float = 1500.0, prompt_max: int = 8192, out_mean: float = 256.0,
               out_max: int = 2048, class_ratios: Sequence[float] = (1, 2, 4),
               bursty_high: bool = False) -> List[TraceRequest]:
    """Arrival trace for scheduler parity runs: Poisson arrivals per class at the given
    ratios (or, with ``bursty_high``, class-1 arrivals from a two-state on/off process:
    10x rate for 2 s, silent for 18 s), lognormal prompt and output lengths."""
    seed = BASE_SEED + 100 + index if seed is None else seed
    rng = np.random.default_rng(seed)
    ratios = np.asarray(class_ratios, dtype=np.float64)
    ratios = ratios / ratios.sum()
    reqs = []
    t = 0.0
    while len(reqs) < n_requests:
        t += rng.exponential(1.0 / rate_per_s)
        c = int(rng.choice(len(ratios), p=ratios)) + 1
        if bursty_high and c == 1:
            phase = t % 20.0
            if phase >= 2.0:       # off period: the arrival slides into the next burst
                t_arr = t - phase + 20.0 + rng.uniform(0.0, 2.0)
            else:
                t_arr = t
        else:
            t_arr = t
        pl = int(_lognormal_lengths(rng, 1, prompt_mean, 0.8, 1, prompt_max)[0])
        ol = int(_lognormal_lengths(rng, 1, out_mean, 0.8, 1, out_max)[0])
        reqs.append((t_arr, c, pl, ol))
    reqs.sort(key=lambda x: x[0])
    return [TraceRequest(rid=i, arrival_ps=int(round(a * 1e12)), prio=c, prompt_len=pl, out_len=ol)
            for i, (a, c, pl, ol) in enumerate(reqs)]


# --------------------------------------------------------------------------- "needle" inputs
NEEDLE_TILE = 32
NEEDLE_K_GAINS = (0.6875, 0.6953125, 0.703125, 0.7109375, 0.71875)   # bf16-exact


@dataclass
class NeedlePlan:
    """A second input recipe for long contexts.  With plain N(0,1) inputs an attention output over n keys is
    an average of ~n values and shrinks like 1/sqrt(n): losing a whole 32-token tile of a 24 k context moves
    it by less than any usable tolerance.  Here every 32-token tile of every request holds one planted token
    whose key is aligned with a direction u (per request and kv-head) that is also added to the request's
    queries, so that its score stands out (q.k/sqrt(d) about +8), and whose value row is a +-A sign pattern
    of its own, with A growing with the request's tile count so that every single tile carries a visible
    share of every output row that can see it.  Only draws and sizes: no attention arithmetic here."""
    pos: List[np.ndarray]        # per request: planted token positions, one per tile, increasing
    gain: List[np.ndarray]       # per request: float32 key gain of each planted token
    amp: np.ndarray              # per request: float32 amplitude A of its planted value rows
    u: np.ndarray                # float32 [n_req, Hkv, d] of +-1
    vsign: List[np.ndarray]      # per request: int8 [n_planted, Hkv, d] of +-1

    def k_rows(self, r: int) -> np.ndarray:
        """bf16 bits [n_planted, Hkv, d] of request r's planted keys."""
        return f32_to_bf16_bits(self.gain[r][:, None, None] * self.u[r][None])

    def v_rows(self, r: int) -> np.ndarray:
        return f32_to_bf16_bits(self.amp[r] * self.vsign[r].astype(np.float32))


def make_needle_plan(batch: MixedBatch, seed: Optional[int] = None) -> NeedlePlan:
    rng = np.random.default_rng((batch.seed if seed is None else seed) + 104729)
    s = batch.shape
    pos, gain, vsign = [], [], []
    amp = np.empty(batch.n_req, dtype=np.float32)
    u = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=(batch.n_req, s.n_kv_heads, s.head_dim))
    for r in range(batch.n_req):
        L = int(batch.kv_len[r])
        nt = -(-L // NEEDLE_TILE)
        first = np.arange(nt, dtype=np.int64) * NEEDLE_TILE
        width = np.minimum(NEEDLE_TILE, L - first)
        pos.append(first + rng.integers(0, width))
        gain.append(rng.choice(np.array(NEEDLE_K_GAINS, dtype=np.float32), size=nt))
        vsign.append(rng.choice(np.array([-1, 1], dtype=np.int8), size=(nt, s.n_kv_heads, s.head_dim)))
        amp[r] = bf16_bits_to_f32(f32_to_bf16_bits(np.array([max(1.0, nt / 48.0)], dtype=np.float32)))[0]
    return NeedlePlan(pos=pos, gain=gain, amp=amp, u=u, vsign=vsign)


def make_needle_tensors(batch: MixedBatch, seed: Optional[int] = None) -> Tuple[StepTensors, NeedlePlan]:
    """CPU-sized form of the needle recipe: N(0,1) tensors as make_tensors draws them, the request's direction
    added to its queries, the planted rows written over the plain ones."""
    plan = make_needle_plan(batch, seed)
    rng = np.random.default_rng((batch.seed if seed is None else seed) + 7919)
    s = batch.shape
    q = rng.standard_normal(size=(batch.n_tokens, s.n_q_heads, s.head_dim), dtype=np.float32)
    for r in range(batch.n_req):
        a, b = int(batch.q_start[r]), int(batch.q_start[r + 1])
        q[a:b] += np.repeat(plan.u[r], s.group, axis=0)[None]
    t = StepTensors(q=f32_to_bf16_bits(q))
    for r in range(batch.n_req):
        L = int(batch.kv_len[r])
        k = normal_bf16(rng, (L, s.n_kv_heads, s.head_dim))
        v = normal_bf16(rng, (L, s.n_kv_heads, s.head_dim))
        k[plan.pos[r]] = plan.k_rows(r)
        v[plan.pos[r]] = plan.v_rows(r)
        t.k.append(k)
        t.v.append(v)
    return t, plan


# --------------------------------------------------------------------------- full-size device inputs
def device_inputs(batch: MixedBatch, seed: int, device: str = "cuda:0", recipe: str = "normal"):
    """Full-size inputs generated on the GPU with torch's seeded generator (plumbing, not the HIP
    path): the whole device pool, q, and this step's k_new / v_new, all N(0,1) rounded to bf16.
    Returns (pool [M, block_elems], q, k_new, v_new) as bf16 tensors.  Filling the raw pool with
    i.i.d. values makes every logical K/V entry N(0,1) whatever the in-block layout.
    recipe "needle": on top of that, the planted tokens of make_needle_plan (the cached ones written
    into the pool through the block tables, this step's own into k_new / v_new) and each request's
    direction added to its queries."""
    import torch
    from .kvlayout import scatter_token_rows
    s = batch.shape
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    pool_elems = batch.n_device_blocks * (s.block_bytes // 2)
    pool = torch.empty(pool_elems, dtype=torch.bfloat16, device=device)
    step = 1 << 28
    for a in range(0, pool_elems, step):       # N(0,1) in fp32, rounded to bf16, in slabs
        n = min(step, pool_elems - a)
        pool[a:a + n] = torch.randn(n, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    pool = pool.view(batch.n_device_blocks, -1)

    def rows(heads):
        return torch.randn((batch.n_tokens, heads, s.head_dim), generator=g, device=device)

    q, kn, vn = rows(s.n_q_heads), rows(s.n_kv_heads).to(torch.bfloat16), rows(s.n_kv_heads).to(torch.bfloat16)
    if recipe == "needle":
        plan = make_needle_plan(batch, seed)
        lq = np.diff(batch.q_start)
        req_of_token = np.repeat(np.arange(batch.n_req), lq)
        u_dev = torch.from_numpy(plan.u).to(device)                                  # [n_req, Hkv, d]
        q += u_dev[torch.from_numpy(req_of_token).to(device)].repeat_interleave(s.group, dim=1)
        blocks, slots, krows, vrows, new_at, new_k, new_v = [], [], [], [], [], [], []
        for r in range(batch.n_req):
            L, p = int(batch.kv_len[r]), int(batch.kv_len[r]) - int(lq[r])
            pos, kr, vr = plan.pos[r], plan.k_rows(r), plan.v_rows(r)
            old = pos < p
            blocks.append(batch.table(r)[pos[old] // s.block_tokens])
            slots.append(pos[old] % s.block_tokens)
            krows.append(kr[old]); vrows.append(vr[old])
            new_at.append(int(batch.q_start[r]) + (pos[~old] - p))
            new_k.append(kr[~old]); new_v.append(vr[~old])

        def bits(a):
            return torch.from_numpy(np.ascontiguousarray(np.concatenate(a)).view(np.int16)).to(device).view(torch.bfloat16)
        scatter_token_rows(pool, s.n_kv_heads, torch.from_numpy(np.concatenate(blocks).astype(np.int64)).to(device),
                           torch.from_numpy(np.concatenate(slots).astype(np.int64)).to(device), bits(krows), bits(vrows))
        at = torch.from_numpy(np.concatenate(new_at).astype(np.int64)).to(device)
        kn[at] = bits(new_k)
        vn[at] = bits(new_v)
    elif recipe != "normal":
        raise ValueError("recipe must be 'normal' or 'needle'")
    return pool, q.to(torch.bfloat16), kn, vn
