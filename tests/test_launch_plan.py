"""Host logic of the mixed attention launch (no GPU): how many compute units the decode workgroups of a batch
get next to its prefill workgroups, and when prefill rows are split along their KV range.  Checked through
ps_plan_launch on the benchmark workloads and on seeded random batches."""
import numpy as np
import pytest

from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W


def plan(b, n_cus=256, **kw):
    s = b.shape
    return B.ps_plan_launch(s.n_q_heads, s.n_kv_heads, b.n_device_blocks, b, n_cus, **kw)


def decode_tiles(b):
    return int(sum(-(-int(b.kv_len[r]) // 32) for r in b.decode_reqs))


def test_decode_only_batch_gets_one_wave_per_simd():
    b = W.build_batch(W.LayerShape(32, 8), [(1, 4000)] * 300, [1] * 300, np.random.default_rng(1), seed=1)
    p = plan(b)
    assert p["decode_waves"] == 1024 and p["decode_slots"] == 128 and p["decode_workgroups"] == 256
    assert p["prefill_workgroups"] == 0 and p["prefill_split_tiles"] == 0
    p = plan(b, n_cus=64)
    assert p["decode_waves"] == 256 and p["decode_workgroups"] == 64
    p = plan(b, decode_waves=512)
    assert p["decode_waves"] == 512


def test_prefill_only_batch_has_no_decode_workgroups():
    b = W.build_batch(W.LayerShape(32, 8), [(512, 512), (256, 4096)], [1, 1], np.random.default_rng(2), seed=2)
    p = plan(b, prefill_split_tiles=-1)
    assert p["decode_workgroups"] == 0 and p["decode_waves"] == 0
    # 64-token query tiles for four heads per kv-head: (8 + 4) tiles x 8 kv-heads
    assert p["prefill_workgroups"] == 12 * 8 and p["partial_slots"] == 0


def test_shares_of_the_benchmark_workloads():
    """Decode-heavy batch: the share at which both kinds of work end together, a little under t_d / (t_d + t_p)
    of the chip.  One long chunk of equally long workgroups that outweighs the decode work: decode gets most
    of the chip first and leaves it to the prefill workgroups.  Many prefill workgroups of all lengths next to
    moderate decode work: the proportional share again."""
    p2, p4, p5 = (plan(W.make_workload(i), mixed_launch=1) for i in (2, 4, 5))
    assert 170 <= p2["decode_workgroups"] <= 200 and p2["prefill_split_tiles"] > 0      # 64-tile rows cut in two
    assert 160 <= p4["decode_workgroups"] <= 248 and p4["prefill_workgroups"] == 512 and p4["prefill_split_tiles"] == 0
    assert 64 <= p5["decode_workgroups"] <= 128 and p5["prefill_workgroups"] == 2048
    for p in (p2, p4, p5):
        assert p["decode_waves"] == p["decode_slots"] * 8
        assert p["decode_workgroups"] == -(-p["decode_slots"] // 4) * 8


def test_which_mixed_batches_get_workgroups_that_carry_both_kinds_of_work():
    """Left to the library (mixed_launch = 0), a launch in which neither kind of work dwarfs the other and which has at
    least one prefill workgroup per compute unit is laid out that way (workloads 4 and 5: the prefill work priced at 2.6
    and 1.9 times the decode work; not workload 2, mostly decode work, nor workload 5 with an eighth of its decode
    requests); with short KV walks the prefill work has to be the larger of the two; forced (2), any mixed batch is,
    and every prefill workgroup then walks at most two decode slots of its kv-head."""
    p2, p4, p5 = (plan(W.make_workload(i)) for i in (2, 4, 5))
    assert p2["decode_workgroups"] > 0 and p2 == plan(W.make_workload(2), mixed_launch=1)
    assert p4["decode_workgroups"] == 0 and p4["prefill_workgroups"] == 512 and p4 == plan(W.make_workload(4), mixed_launch=2)
    assert p5["decode_workgroups"] == 0 and p5["prefill_workgroups"] == 2048 and p5 == plan(W.make_workload(5), mixed_launch=2)
    b5 = W.make_workload(5)
    few = [(1, int(b5.kv_len[r])) for r in b5.decode_reqs[:64]] + [(b5.l_q(int(r)), int(b5.kv_len[r])) for r in b5.prefill_reqs]
    bf = W.build_batch(b5.shape, few, [1] * len(few), np.random.default_rng(3), seed=3)
    assert plan(bf)["decode_workgroups"] > 0 and plan(bf, mixed_launch=2)["decode_workgroups"] == 0
    # one chunk next to 192 decode requests of 857 tokens, 256 prefill workgroups: long walks and twice the decode work
    # -> both in every workgroup; short walks and half the decode work -> disjoint units; a ratio of 0.8: by walk length
    def small(pre, n_dec):
        items = [(1, 857)] * n_dec + pre
        return plan(W.build_batch(W.LayerShape(32, 8), items, [1] * len(items), np.random.default_rng(5), n_device_blocks=60_000, seed=5))
    assert small([(2048, 2048 + 4096)], 192)["decode_workgroups"] == 0 and small([(2048, 2048 + 4096)], 192)["prefill_workgroups"] == 256
    assert small([(1024, 1024 + 2048)], 192)["decode_workgroups"] > 0
    assert small([(2048, 2048 + 4096)], 384)["decode_workgroups"] == 0        # a ratio of 0.9, walks of 96 tiles on average
    assert small([(4096, 4096)], 384)["decode_workgroups"] > 0                # 0.7, walks of 32 tiles on average
    for i in (2, 4, 5):
        b = W.make_workload(i)
        p = plan(b, mixed_launch=2)
        assert p["decode_workgroups"] == 0 and p["decode_waves"] == p["decode_slots"] * 8
        assert p["decode_slots"] == 2 * p["prefill_workgroups"] // 8      # some of them may be empty
        assert p["prefill_workgroups"] == plan(b, mixed_launch=1)["prefill_workgroups"]
    # decode-only and prefill-only batches are not affected, nor is a batch with fixed decode partitions or wave count
    b = W.build_batch(W.LayerShape(32, 8), [(1, 4000)] * 300, [1] * 300, np.random.default_rng(1), seed=1)
    assert plan(b, mixed_launch=2) == plan(b)
    b = W.make_workload(4)
    assert plan(b, mixed_launch=2, decode_chunk=256)["decode_workgroups"] > 0
    assert plan(b, mixed_launch=2, decode_waves=512)["decode_workgroups"] > 0
    with pytest.raises(B.PsError):
        plan(b, mixed_launch=3)


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_keep_the_launch_within_bounds(seed):
    rng = np.random.default_rng(9000 + seed)
    Hq, Hkv = [(32, 8), (64, 8), (8, 2), (16, 1)][seed % 4]
    n_cus = [256, 128, 304, 64][seed % 4]
    items = [(1, int(rng.integers(1, 20000))) for _ in range(int(rng.integers(0, 200)))]
    n_pre = int(rng.integers(0 if items else 1, 5))
    for _ in range(n_pre):
        lq = int(rng.integers(2, 3000))
        items.append((lq, lq + int(rng.integers(0, 20000))))
    b = W.build_batch(W.LayerShape(Hq, Hkv), items, [1] * len(items), rng, seed=seed)
    p = plan(b, n_cus, mixed_launch=1)
    n_dec, T = len(b.decode_reqs), decode_tiles(b)
    assert (p["decode_slots"] > 0) == (n_dec > 0)
    if n_dec:
        assert p["decode_slots"] <= max(1, T // 4)                     # no slot shorter than four tiles
        assert p["decode_waves"] <= 4 * n_cus                           # never more than one wave per SIMD
        if n_pre:                                                       # prefill keeps at least 8 compute units
            assert p["decode_waves"] <= 4 * max(8, n_cus - 8)
    G = Hq // Hkv
    hw = 8 if G % 8 == 0 else 4 if G % 4 == 0 else 2 if G % 2 == 0 else 1
    tt = (8 // hw) * 32
    tiles = sum(-(-b.l_q(int(r)) // tt) for r in b.prefill_reqs)
    assert p["prefill_workgroups"] >= tiles * Hkv * (G // hw)          # more only when rows are split
    assert (p["prefill_workgroups"] > tiles * Hkv * (G // hw)) == (p["prefill_split_tiles"] > 0)
    # partial slots: cut decode requests (at most one cut per slot boundary) and split prefill rows
    assert p["partial_slots"] >= 0
    if p["prefill_split_tiles"] == 0:
        assert p["partial_slots"] <= 2 * max(0, p["decode_slots"] - 1)
    # the plan is a function of the batch alone
    assert plan(b, n_cus, mixed_launch=1) == p
    # every workgroup carrying both kinds of work: same prefill work items, at most two decode slots for each
    f = plan(b, n_cus, mixed_launch=2)
    if n_dec and n_pre:
        assert f["decode_workgroups"] == 0 and f["prefill_workgroups"] == p["prefill_workgroups"]
        assert f["decode_slots"] == 2 * f["prefill_workgroups"] // Hkv     # some of them may be empty
        if f["prefill_split_tiles"] == 0:
            assert f["partial_slots"] <= 2 * max(0, min(f["decode_slots"], -(-T // 4)) - 1)   # a cut every four tiles at most
    else:
        assert f == p
    assert plan(b, n_cus) in (p, f)


def test_bad_arguments():
    b = W.make_workload(1)
    with pytest.raises(B.PsError):
        plan(b, n_cus=0)
    with pytest.raises(B.PsError):
        B.ps_plan_launch(8, 3, 64, b)                                   # Hq not a multiple of Hkv
    bad = W.make_workload(1)
    bad.kv_len = bad.kv_len.copy()
    bad.kv_len[0] += 100
    with pytest.raises(B.PsError):
        plan(bad)


def test_planner_constants_move_the_share_and_the_split():
    """The machine constants the planner prices with are configuration (ps_layer_cfg.plan_*; 0 = the MI355X default):
    a faster cache stream shrinks the decode share, a slower prefill tile step shrinks it too, the defaults written
    out give the default plan, a dear merge forbids the row split."""
    b = W.make_workload(2)
    base = plan(b)
    same = plan(b, plan_stream_TBps=6.3, plan_tile_step_us=1.78, plan_merge_launch_steps=4.0, plan_merge_row_steps=0.0047,
                plan_decode_share=0.95, plan_decode_knee_cus=176)
    assert same == base
    assert plan(b, plan_stream_TBps=12.6)["decode_workgroups"] < base["decode_workgroups"]
    assert plan(b, plan_tile_step_us=3.84)["decode_workgroups"] < base["decode_workgroups"]
    assert plan(b, plan_decode_share=0.5)["decode_workgroups"] < base["decode_workgroups"]
    assert base["prefill_split_tiles"] > 0 and plan(b, plan_merge_launch_steps=1000.0)["prefill_split_tiles"] == 0
    for bad in (dict(plan_stream_TBps=-1.0), dict(plan_decode_share=1.5), dict(plan_decode_knee_cus=-3),
                dict(plan_tile_step_us=float("inf"))):
        with pytest.raises(B.PsError) as e:
            plan(b, **bad)
        assert e.value.code == B.PS_EINVAL
