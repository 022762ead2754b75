"""GPU parity of the mixed launch whose workgroups carry both kinds of work (cfg.mixed_launch = 2: a prefill tile
walk on eight waves, two waves that fetch its tiles into LDS, two that walk decode slots) against the fp64 oracle,
element by element through the C ABI, at the tolerance of the other step tests (max-abs 1e-2 on the f32 output).  The
hand-over between the waves goes through flags in LDS with bounded waits: after all cases no wave may have given
one up (ps_mixed_launch_faults)."""
import numpy as np
import pytest
import torch

from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from gpu_harness import DEV, Layer, check_close, dev_to_u16, oracle_cache, run_prefilled, u16_to_dev
from paper_2512_12928_amd.kvlayout import from_device_layout, to_device_layout
from test_gpu_step import custom_batch, drifting_batch, oracle_out

pytestmark = pytest.mark.gpu
KW = dict(mixed_launch=2)


def check(b, t, **kw):
    got, cache = run_prefilled(b, t, **KW, **kw)
    return check_close(got, oracle_out(b, t, cache), False)


def test_walks_shorter_and_longer_than_the_ring():
    """One to many tiles per walk (the ring holds eight), with and without decode slots for the workgroup."""
    check(*custom_batch(8, 2, [(1, 40), (33, 33)], seed=1))
    check(*custom_batch(8, 2, [(1, 40), (300, 2100), (1, 7), (1, 900), (64, 64 + 48)], seed=5))
    check(*custom_batch(8, 2, [(1, 9000), (20, 20)], seed=6))          # decode slots outlast the walk by far
    check(*custom_batch(8, 2, [(1, 3), (500, 4000)], seed=8))          # and the other way round


def test_ragged_and_degenerate_shapes():
    items = [(1, 1), (1, 15), (1, 16), (1, 17), (1, 31), (1, 32), (1, 33), (1, 511), (1, 512), (1, 513),
             (2, 2), (33, 33), (95, 95 + 13), (64, 64 + 48), (31, 31 + 16), (129, 129 + 7), (5, 700)]
    check(*custom_batch(8, 2, items, seed=7))


@pytest.mark.parametrize("split", [1, 2, 3, -1])
def test_prefill_kv_partitions(split):
    items = [(1, 40), (64, 64), (200, 200), (70, 70 + 333), (129, 129 + 1000), (5, 700), (33, 33 + 64), (1, 900)]
    check(*custom_batch(8, 2, items, seed=21), prefill_split_tiles=split)
    check(*custom_batch(16, 2, items[:5], seed=22), prefill_split_tiles=split)


@pytest.mark.parametrize("split", [1, 3, -1])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 1), (64, 8)])
def test_leaping_row_maxima_with_partitions(Hq, Hkv, split):
    """Scores that leap by 65 to 163 powers of two along the walk (more than fp32 holds against a reference that lags),
    with the prefill rows' KV ranges cut into partitions or not, for several group sizes: the MFMA waves take a tile's
    maximum only when their row sums tell them to, and the partials they hand to the merge carry whatever reference
    they ended with."""
    b, t = drifting_batch("leaps", Hq, Hkv, seed=90 + Hq)
    check(b, t, prefill_split_tiles=split)


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (2, 1), (4, 1), (8, 1), (16, 1), (6, 2), (12, 4), (64, 8)])
def test_group_sizes(Hq, Hkv):
    items = [(1, 1), (1, 16), (1, 33), (1, 300), (7, 7), (40, 77), (1, 1)]
    check(*custom_batch(Hq, Hkv, items, seed=100 + Hq))


@pytest.mark.parametrize("seed", range(8))
def test_random_mixed_batches(seed):
    """Seeded random mixed batches (odd seeds through the append path, pool checked bit for bit afterwards)."""
    rng = np.random.default_rng(4000 + seed)
    Hq, Hkv = [(8, 2), (32, 8), (16, 1), (64, 8)][seed % 4]
    items = [(1, int(rng.integers(1, 3000))) for _ in range(int(rng.integers(1, 40)))]
    for _ in range(int(rng.integers(1, 4))):
        lq = int(rng.integers(2, 300))
        items.append((lq, lq + int(rng.integers(0, 1500))))
    items = [items[i] for i in rng.permutation(len(items))]
    b, t = custom_batch(Hq, Hkv, items, seed=4000 + seed)
    full = oracle_cache(b, t)
    want = oracle_out(b, t, full)
    if seed % 2 == 0:
        got, _ = run_prefilled(b, t, **KW)
        check_close(got, want, False)
    else:
        pre = oracle_cache(b, t, upto_prefix=True)
        cache_dev = u16_to_dev(to_device_layout(pre.pool))
        k_new, v_new = t.new_rows(b)
        lay = Layer(b, **KW)
        out = lay.step(b, u16_to_dev(t.q), cache_dev, u16_to_dev(k_new), u16_to_dev(v_new))
        lay.close()
        check_close(out.cpu().numpy().astype(np.float64), want, False)
        assert np.array_equal(from_device_layout(dev_to_u16(cache_dev), b.shape.n_kv_heads), full.pool)


@pytest.mark.parametrize("idx,scale", [(2, 0.08), (4, 0.04), (5, 0.06)])
def test_scaled_workloads(idx, scale):
    b = W.make_workload(idx, scale=scale)
    print(b.name, "max err", check(b, W.make_tensors(b)))


def test_walk_longer_than_the_id_table():
    """A chunk over a 36 000-token prefix, unsplit (a walk of more than a thousand ring tiles by one workgroup), next
    to a 70 000-token decode request."""
    check(*custom_batch(2, 1, [(40, 40 + 36_000), (1, 70_000), (1, 5)], seed=31), prefill_split_tiles=-1)


def test_next_layer_reuses_the_plan_and_block_relabelling_changes_nothing():
    """ps_step_next_layer runs the same launch from the stored plan: the step's own output again, bit for bit.  And
    the launch is deterministic in the logical batch: with the physical blocks relabelled (another seeded permutation
    of the pool) every output bit stays."""
    items = [(1, 700)] * 30 + [(256, 256 + 1024), (100, 100)]
    outs = []
    for seed in (9, 9, 10):
        rng = np.random.default_rng(seed)
        b = W.build_batch(W.LayerShape(32, 8), items, [1] * len(items), rng, seed=9)   # same tensors, other block ids
        t = W.make_tensors(b)
        cache = oracle_cache(b, t)
        cache_dev = u16_to_dev(to_device_layout(cache.pool))
        q = u16_to_dev(t.q)
        lay = Layer(b, **KW)
        out = lay.step(b, q, cache_dev)
        again = torch.full_like(out, float("nan"))
        B.ps_step_next_layer(lay.ctx, q, None, None, cache_dev, again, lay.ws, lay.ws_bytes, torch.cuda.current_stream())
        torch.cuda.synchronize()
        lay.close()
        assert torch.equal(again, out)
        check_close(out.cpu().numpy().astype(np.float64), oracle_out(b, t, cache), False)
        outs.append(out)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_profiled_step_reports_both_clocks():
    b, t = custom_batch(32, 8, [(1, 2000)] * 64 + [(512, 512 + 2048)], seed=10)
    cache_dev = u16_to_dev(to_device_layout(oracle_cache(b, t).pool))
    lay = Layer(b, **KW)
    B.ps_set_profiling(lay.ctx, 1)
    lay.step(b, u16_to_dev(t.q), cache_dev)
    st = B.ps_get_step_times(lay.ctx)
    lay.close()
    print(st)
    assert st["attention_ms"] > 0 and 500 < st["prefill_mhz"] < 2600 and 500 < st["decode_mhz"] < 2600


def test_zz_no_wave_gave_up_a_wait():
    assert B.ps_mixed_launch_faults() == 0
