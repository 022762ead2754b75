"""Host logic of the decode work list (ps_plan_decode; no GPU needed): the segments tile every decode
request exactly, the slots are equally long, and the list is what the kernel's indexing assumes."""
import numpy as np
import pytest

from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W


def random_batch(rng, n_dec, n_pre, max_len, hkv=8):
    shape = W.LayerShape(4 * hkv, hkv)
    items = []
    for _ in range(n_dec):
        items.append((1, int(rng.integers(1, max_len + 1))))
    for _ in range(n_pre):
        lq = int(rng.integers(2, 200))
        items.append((lq, lq + int(rng.integers(0, max_len))))
    order = rng.permutation(len(items))
    items = [items[i] for i in order]
    return W.build_batch(shape, items, [0] * len(items), rng, n_device_blocks=None, seed=int(rng.integers(1 << 30)))


def check_plan(batch, seg, n_slots, waves, hkv, chunk=0):
    dec = [int(r) for r in batch.decode_reqs]
    by_req = {r: [] for r in dec}
    for r, t0, t1, x, part in seg:
        assert r in by_req, "a segment of a request that is not a decode request"
        by_req[int(r)].append((int(t0), int(t1), int(x), int(part)))
    parts_seen = []
    for r in dec:
        L = int(batch.kv_len[r])
        s = sorted(by_req[r])
        assert s[0][0] == 0 and s[-1][1] == L
        for (a0, a1, _, _), (b0, _, _, _) in zip(s, s[1:]):
            assert a1 == b0 and a1 % 32 == 0          # contiguous, cut on a tile boundary
        if len(s) == 1:
            assert s[0][3] == -1
        else:
            ps = [p for _, _, _, p in s]
            assert ps == list(range(ps[0], ps[0] + len(s))) and ps[0] >= 0   # consecutive partial slots
            parts_seen += ps
    assert sorted(parts_seen) == list(range(len(parts_seen)))   # partial slots are used exactly once
    # slots: numbered in launch order, none empty
    xs = [int(x) for _, _, _, x, _ in seg]
    assert xs == sorted(xs) and (not xs or (xs[0] == 0 and xs[-1] == n_slots - 1 and len(set(xs)) == n_slots))
    tiles = np.zeros(max(n_slots, 1), dtype=np.int64)
    for _, t0, t1, x, _ in seg:
        tiles[x] += -(-(int(t1) - int(t0)) // 32)
    T = int(sum(-(-int(batch.kv_len[r]) // 32) for r in dec))
    if chunk == 0:
        assert n_slots == (max(1, min(waves // hkv, T // 4)) if dec else 0)
        if dec:
            assert tiles.sum() == T and tiles.max() - tiles.min() <= 1
            assert sum(len(v) > 1 for v in by_req.values()) <= n_slots - 1 or n_slots == 1
    else:
        assert n_slots == len(seg)
        lens = [int(t1) - int(t0) for _, t0, t1, _, _ in seg]
        assert all(l <= chunk for l in lens) and lens == sorted(lens, reverse=True)


@pytest.mark.parametrize("seed", range(12))
def test_balanced_slots_tile_the_requests(seed):
    rng = np.random.default_rng(1000 + seed)
    hkv = [1, 2, 4, 8][seed % 4]
    batch = random_batch(rng, n_dec=int(rng.integers(1, 300)), n_pre=int(rng.integers(0, 4)),
                         max_len=[40, 700, 9000][seed % 3], hkv=hkv)
    for waves in (1, 7, 64, 1024, 4096):
        seg, n_slots = B.ps_plan_decode(hkv, batch.n_device_blocks, batch, waves)
        check_plan(batch, seg, n_slots, waves, hkv)


@pytest.mark.parametrize("chunk", [32, 64, 256, 4096])
def test_fixed_partitions(chunk):
    rng = np.random.default_rng(77 + chunk)
    batch = random_batch(rng, n_dec=50, n_pre=2, max_len=3000)
    seg, n_slots = B.ps_plan_decode(8, batch.n_device_blocks, batch, 1024, decode_chunk=chunk)
    check_plan(batch, seg, n_slots, 1024, 8, chunk=chunk)


def test_edge_cases():
    shape = W.LayerShape(32, 8)
    # one token of context; no decode request at all; one very long request cut many times
    rng = np.random.default_rng(9)
    b1 = W.build_batch(shape, [(1, 1)], [0], rng, n_device_blocks=64, seed=1)
    seg, n = B.ps_plan_decode(8, 64, b1, 1024)
    assert n == 1 and seg.tolist() == [[0, 0, 1, 0, -1]]
    b2 = W.build_batch(shape, [(64, 64)], [0], rng, n_device_blocks=64, seed=2)
    seg, n = B.ps_plan_decode(8, 64, b2, 1024)
    assert n == 0 and len(seg) == 0
    b3 = W.build_batch(shape, [(1, 50_000)], [0], rng, n_device_blocks=4096, seed=3)
    seg, n = B.ps_plan_decode(8, 4096, b3, 1024)
    check_plan(b3, seg, n, 1024, 8)
    assert n == 128 and len(seg) == 128          # 1563 tiles: 1024 / 8 slots of 12 or 13 tiles
    seg, n = B.ps_plan_decode(8, 4096, b3, 4096)
    check_plan(b3, seg, n, 4096, 8)
    assert n == 390 and len(seg) == 390          # no slot shorter than 4 tiles: 1563 / 4 slots (fewer than 4096 / 8)
    # the headline workload at full size, with the wave count ps_step uses on a 256-CU device
    b4 = W.make_workload(2)
    seg, n = B.ps_plan_decode(8, b4.n_device_blocks, b4, 1024)
    check_plan(b4, seg, n, 1024, 8)
    assert n == 128


def test_rejects_bad_batches():
    shape = W.LayerShape(32, 8)
    b = W.build_batch(shape, [(1, 100), (1, 17)], [0, 0], np.random.default_rng(5), n_device_blocks=64, seed=5)
    bad = W.build_batch(shape, [(1, 100), (1, 17)], [0, 0], np.random.default_rng(5), n_device_blocks=64, seed=5)
    bad.kv_len = bad.kv_len.copy()
    bad.kv_len[1] = 40                                   # table has 2 entries, 40 tokens need 3
    with pytest.raises(B.PsError) as e:
        B.ps_plan_decode(8, 64, bad, 1024)
    assert e.value.code == B.PS_EINVAL
    with pytest.raises(B.PsError) as e:
        B.ps_plan_decode(8, 4, b, 1024)                  # block ids outside a pool of 4 blocks
    assert e.value.code == B.PS_EINVAL
    with pytest.raises(B.PsError) as e:
        B.ps_plan_decode(8, 64, b, 0)                    # no waves
    assert e.value.code == B.PS_EINVAL
    with pytest.raises(B.PsError) as e:
        B.ps_plan_decode(8, 64, b, 1024, decode_chunk=48)
    assert e.value.code == B.PS_EINVAL
