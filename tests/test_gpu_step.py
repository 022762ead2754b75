"""GPU parity of ps_step (append + decode split-K + merge + prefill MFMA) against the fp64 oracle,
element by element, through the C ABI.  Tolerance: max-abs 1e-2 on the f32 output path (bf16
inputs, fp32 accumulation); on the bf16 output path 1e-2 + 2^-8 |o| (half an ulp of the output
format), plus o_bf16 == RNE(o_f32) bit for bit."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from gpu_harness import DEV, Layer, check_close, dev_to_u16, oracle_cache, run_prefilled, u16_to_dev
from paper_2512_12928_amd.kvlayout import from_device_layout, to_device_layout

pytestmark = pytest.mark.gpu


def oracle_out(batch, tens, cache):
    return A.paged_attention(tens.q, cache, batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids)


def custom_batch(Hq, Hkv, items, seed, prios=None, M=None):
    rng = np.random.default_rng(seed)
    b = W.build_batch(W.LayerShape(Hq, Hkv), items, prios or [1] * len(items), rng, n_device_blocks=M, seed=seed)
    return b, W.make_tensors(b)


def test_cfg1_prefilled_f32():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    got, cache = run_prefilled(b, t)
    print("cfg1 max err", check_close(got, oracle_out(b, t, cache), False))


def test_cfg1_bf16_output_is_rounded_f32_output():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    g32, cache = run_prefilled(b, t, out_f32=True)
    cache_dev = u16_to_dev(to_device_layout(cache.pool))
    lay = Layer(b, out_f32=False)
    o16 = lay.step(b, u16_to_dev(t.q), cache_dev)
    lay.close()
    bits = dev_to_u16(o16.view(torch.int16))
    assert np.array_equal(bits, W.f32_to_bf16_bits(g32.astype(np.float32)))
    check_close(W.bf16_bits_to_f32(bits).astype(np.float64), oracle_out(b, t, cache), True)


def test_cfg1_append_path_matches_and_pool_is_bit_exact():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    full = oracle_cache(b, t)
    pre = oracle_cache(b, t, upto_prefix=True)
    cache_dev = u16_to_dev(to_device_layout(pre.pool))
    k_new, v_new = t.new_rows(b)
    lay = Layer(b)
    out = lay.step(b, u16_to_dev(t.q), cache_dev, u16_to_dev(k_new), u16_to_dev(v_new))
    lay.close()
    check_close(out.cpu().numpy().astype(np.float64), oracle_out(b, t, full), False)
    # the append is a copy: the whole pool (NaN-filled elsewhere) must equal the oracle's bit for bit
    assert np.array_equal(from_device_layout(dev_to_u16(cache_dev), b.shape.n_kv_heads), full.pool)


@pytest.mark.parametrize("chunk", [32, 64, 256])
def test_split_k_partitions_and_merge(chunk):
    b = W.make_workload(1)
    t = W.make_tensors(b)
    got, cache = run_prefilled(b, t, decode_chunk=chunk)
    check_close(got, oracle_out(b, t, cache), False)


@pytest.mark.parametrize("waves", [8, 64, 1024, 4096])
def test_balanced_decode_slots(waves):
    """Decode-only batch, balanced slots: one wave walking every request (8 waves = one slot), a long
    request cut into more than 8 partials (the merge kernel's second round), requests of one token."""
    lens = [1, 3, 16, 17, 31, 32, 33, 64, 100, 257, 700, 1, 48, 9000, 2, 511, 1025]
    b, t = custom_batch(16, 8, [(1, L) for L in lens], seed=99)
    got, cache = run_prefilled(b, t, decode_waves=waves)
    check_close(got, oracle_out(b, t, cache), False)
    seg, n_slots = B.ps_plan_decode(8, b.n_device_blocks, b, waves)
    assert n_slots == max(1, min(waves // 8, 380 // 4))     # 380 tiles, no slot shorter than 4
    if waves >= 1024:
        assert max(np.bincount(seg[:, 0])) > 8     # the 9000-token request has more than 8 segments


def test_mixed_batch_decode_share_extremes():
    """Mixed batches whose decode share of the chip clamps at either end: a sliver of decode work next
    to a long prefill chunk, and a sliver of prefill next to heavy decode."""
    b, t = custom_batch(8, 2, [(1, 40), (300, 2100), (1, 7)], seed=5)
    got, cache = run_prefilled(b, t)
    check_close(got, oracle_out(b, t, cache), False)
    b, t = custom_batch(8, 2, [(1, 6000), (2, 2), (1, 5000), (1, 4000)], seed=6)
    got, cache = run_prefilled(b, t)
    check_close(got, oracle_out(b, t, cache), False)


def test_prefill_heavy_mixed_batch():
    """A long chunk of equally long workgroups that outweighs the decode work next to it: the case in which the
    host prices larger decode shares by simulation (decode first at full speed, prefill inheriting its CUs)."""
    rng = np.random.default_rng(77)
    items = [(1, int(x)) for x in rng.integers(200, 900, size=40)] + [(768, 768 + 3072)]
    b, t = custom_batch(32, 8, items, seed=77)
    got, cache = run_prefilled(b, t)
    check_close(got, oracle_out(b, t, cache), False)


@pytest.mark.parametrize("seed", range(8))
def test_random_mixed_batches(seed):
    """Seeded random mixed batches (head shapes, request counts, lengths, chunk sizes and prefixes drawn at
    random; odd seeds go through the append path) against the oracle, pool checked bit for bit after an append."""
    rng = np.random.default_rng(4000 + seed)
    Hq, Hkv = [(8, 2), (32, 8), (16, 1), (64, 8)][seed % 4]
    items = [(1, int(rng.integers(1, 3000))) for _ in range(int(rng.integers(0, 40)))]
    for _ in range(int(rng.integers(0 if items else 1, 4))):
        lq = int(rng.integers(2, 300))
        items.append((lq, lq + int(rng.integers(0, 1500))))
    items = [items[i] for i in rng.permutation(len(items))]
    b, t = custom_batch(Hq, Hkv, items, seed=4000 + seed)
    full = oracle_cache(b, t)
    want = oracle_out(b, t, full)
    if seed % 2 == 0:
        got, _ = run_prefilled(b, t)
        check_close(got, want, False)
    else:
        pre = oracle_cache(b, t, upto_prefix=True)
        cache_dev = u16_to_dev(to_device_layout(pre.pool))
        k_new, v_new = t.new_rows(b)
        lay = Layer(b)
        out = lay.step(b, u16_to_dev(t.q), cache_dev, u16_to_dev(k_new), u16_to_dev(v_new))
        lay.close()
        check_close(out.cpu().numpy().astype(np.float64), want, False)
        assert np.array_equal(from_device_layout(dev_to_u16(cache_dev), b.shape.n_kv_heads), full.pool)


def test_own_copy_stream_matches():
    """cfg.own_streams: the batch description is uploaded on the context's copy stream; several steps
    back to back on a non-default stream, each equal to the oracle."""
    b = W.make_workload(2, scale=0.08)
    t = W.make_tensors(b)
    cache = oracle_cache(b, t)
    want = oracle_out(b, t, cache)
    lay = Layer(b, own_streams=1, decode_chunk=64, prefill_split_tiles=1)
    cache_dev, q = u16_to_dev(to_device_layout(cache.pool)), u16_to_dev(t.q)
    st = torch.cuda.Stream()
    outs = []
    ws = lay.workspace(b)
    for _ in range(4):
        o = torch.full((b.n_tokens, b.shape.n_q_heads, 128), float("nan"), dtype=torch.float32, device=DEV)
        B.ps_step(lay.ctx, b, q, None, None, cache_dev, o, ws, lay.ws_bytes, st)
        outs.append(o)
    st.synchronize()
    for o in outs:
        check_close(o.cpu().numpy().astype(np.float64), want, False)
    lay.close()


@pytest.mark.parametrize("split", [1, 2, 3, -1])
def test_prefill_kv_partitions(split):
    """Prefill rows whose KV range is cut into partitions of `split` 64-token tiles and merged: same result
    as unsplit (-1), for chunks with and without prefix, ragged ends, rows that see nothing in a partition."""
    items = [(1, 40), (64, 64), (200, 200), (70, 70 + 333), (129, 129 + 1000), (5, 700), (33, 33 + 64), (1, 900)]
    b, t = custom_batch(8, 2, items, seed=21)
    got, cache = run_prefilled(b, t, prefill_split_tiles=split)
    check_close(got, oracle_out(b, t, cache), False)
    b, t = custom_batch(16, 2, items[:5], seed=22)          # G = 8: two head groups per workgroup tile
    got, cache = run_prefilled(b, t, prefill_split_tiles=split)
    check_close(got, oracle_out(b, t, cache), False)


@pytest.mark.parametrize("idx,scale", [(2, 0.08), (4, 0.04), (5, 0.06)])
def test_scaled_workloads(idx, scale):
    b = W.make_workload(idx, scale=scale)
    t = W.make_tensors(b)
    got, cache = run_prefilled(b, t)
    print(b.name, "n_req", b.n_req, "tokens", b.n_tokens, "max err", check_close(got, oracle_out(b, t, cache), False))


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (2, 1), (4, 1), (8, 1), (16, 1), (6, 2), (12, 4)])
def test_group_sizes(Hq, Hkv):
    items = [(1, 1), (1, 16), (1, 33), (1, 300), (7, 7), (40, 77), (1, 1)]
    b, t = custom_batch(Hq, Hkv, items, seed=100 + Hq)
    got, cache = run_prefilled(b, t, decode_chunk=64)
    check_close(got, oracle_out(b, t, cache), False)


def test_ragged_and_degenerate_shapes():
    # kv_len 1; one-token prompt (l_q = 1, p = 0: o == v_0); lengths on and off block / tile
    # boundaries; chunks whose prefix is not a multiple of 16 or 32; chunk sizes that leave a
    # ragged last query tile
    items = [(1, 1), (1, 15), (1, 16), (1, 17), (1, 31), (1, 32), (1, 33), (1, 511), (1, 512), (1, 513),
             (2, 2), (33, 33), (95, 95 + 13), (64, 64 + 48), (31, 31 + 16), (129, 129 + 7), (5, 700)]
    b, t = custom_batch(8, 2, items, seed=7)
    got, cache = run_prefilled(b, t)
    want = oracle_out(b, t, cache)
    check_close(got, want, False)
    # single visible key: output is exactly v_0 of the matching kv-head (P = 1 exactly)
    v0 = A.bf16_to_f64(t.v[0])[0]
    assert np.array_equal(got[0], np.repeat(v0, 4, axis=0))


@pytest.mark.parametrize("split", [-1, 0])
def test_very_long_contexts(split):
    """A chunk over a 36 000-token prefix and a decode request of 70 000 tokens.  Unsplit, the chunk's KV
    walk is one partition of more than 512 tiles, whose block ids do not fit the kernel's LDS table and are
    read through the scalar cache instead; with the default split the partitions are short again."""
    b, t = custom_batch(2, 1, [(40, 40 + 36_000), (1, 70_000), (1, 5)], seed=31)
    got, cache = run_prefilled(b, t, prefill_split_tiles=split)
    check_close(got, oracle_out(b, t, cache), False)


@pytest.mark.parametrize("mixed_launch", [1, 2])
@pytest.mark.parametrize("shape", ["rising", "falling", "steps", "leaps"])
def test_row_maxima_that_drift_along_the_context(shape, mixed_launch):
    """Scores whose row maximum keeps moving along the KV walk: every request's queries and keys share a +-1
    direction, the keys with a gain that rises (0 to 2), falls (2 to 0) or jumps every 100 tokens, which moves
    the scaled score by up to 32 powers of two over the walk, by a fraction of one per tile on the long rows and
    by several per tile on the short ones; "leaps" jumps between gains 0, 4 and 10, 65 to 163 powers of two at
    once, more than fp32 holds.  The online softmax has to follow that whatever its policy for renewing the
    reference maximum (a kernel may let the reference lag behind, and has to notice when it lags too far)."""
    b, t = drifting_batch(shape)
    got, cache = run_prefilled(b, t, mixed_launch=mixed_launch)
    check_close(got, oracle_out(b, t, cache), False)


def drifting_batch(shape, Hq=8, Hkv=2, seed=77):
    """The batch of the test above: N(0,1) tensors with a shared +-1 direction in queries and keys (draws only)."""
    items = [(1, 90), (1, 700), (1, 4000), (40, 140), (200, 900), (64, 64 + 3000), (33, 33)]
    b, t = custom_batch(Hq, Hkv, items, seed=seed)
    rng = np.random.default_rng(seed + 1)
    s = b.shape
    q = W.bf16_bits_to_f32(t.q)
    for r in range(b.n_req):
        u = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=(s.n_kv_heads, s.head_dim))
        L = int(b.kv_len[r])
        pos = np.arange(L, dtype=np.float32) / max(L - 1, 1)
        gain = {"rising": 2 * pos, "falling": 2 - 2 * pos,
                "steps": rng.choice(np.array([0.0, 0.5, 1.0, 2.0], dtype=np.float32), size=L // 100 + 1)[np.arange(L) // 100],
                "leaps": rng.choice(np.array([0.0, 4.0, 10.0], dtype=np.float32), size=L // 100 + 1)[np.arange(L) // 100]}[shape]
        t.k[r] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(t.k[r]) + gain[:, None, None] * u[None])
        a, e = int(b.q_start[r]), int(b.q_start[r + 1])
        q[a:e] += np.repeat(u, s.group, axis=0)[None]
    t.q = W.f32_to_bf16_bits(q)
    return b, t


@pytest.mark.parametrize("mixed_launch", [1, 2])
def test_lone_chunk_over_a_long_prefix_is_cut_into_many_partitions(mixed_launch):
    """A 40-token chunk over 20 000 cached tokens (a walk of 314 KV tiles) with a few decode requests: left alone the
    planner cuts every query tile's walk into more than eight partitions (the merge then folds a row's partials eight
    at a time), in either layout of the mixed launch."""
    b, t = custom_batch(8, 2, [(1, 300), (40, 40 + 20_000), (1, 5000), (1, 17)], seed=55)
    p = B.ps_plan_launch(8, 2, b.n_device_blocks, b, mixed_launch=mixed_launch)
    assert 0 < p["prefill_split_tiles"] < 314 // 8          # more than eight partitions of the 314-tile walk
    got, cache = run_prefilled(b, t, mixed_launch=mixed_launch)
    check_close(got, oracle_out(b, t, cache), False)


@pytest.mark.parametrize("mixed_launch", [1, 2])
def test_rows_that_one_key_dominates(mixed_launch):
    """Two planted keys per request in the prefix (queries and planted keys share a +-1 direction): the first stands
    20 powers of two above the other keys, the second, later in the context, 7 more, so every row is the second key's
    value row but for 0.6 % of the first's.  The kernels round the probabilities to bf16 for the output product, and a
    kernel whose reference for the exponentials is not the row's true maximum (it may lag by a few powers of two)
    gives the dominant key a probability with an arbitrary 8-bit significand instead of 1: unless the row sum carries
    the same rounding, the output is off by up to 2^-8 of a value of 3.5, more than the 1e-2 bound allows.  Asserted to
    5e-3 (score noise leaves some rows a mixture of the two planted values, where the roundings of two probabilities
    show)."""
    items = [(1, 700), (1, 4000), (1, 300), (40, 40 + 1000), (200, 200 + 700), (64, 64 + 3000)]
    b, t = custom_batch(8, 2, items, seed=91)
    rng = np.random.default_rng(92)
    s = b.shape
    q = W.bf16_bits_to_f32(t.q)
    pm = np.array([-1.0, 1.0], dtype=np.float32)
    for r in range(b.n_req):
        u = rng.choice(pm, size=(s.n_kv_heads, s.head_dim))
        prefix = int(b.kv_len[r]) - b.l_q(r)
        first = int(rng.integers(40, prefix // 2))
        second = int(rng.integers(first + 70, prefix))       # a few tiles on, inside the prefix: every row sees both
        k = W.bf16_bits_to_f32(t.k[r])
        k[first] += 1.2 * u
        k[second] += 1.65 * u
        t.k[r] = W.f32_to_bf16_bits(k)
        for pos in (first, second):
            t.v[r][pos] = W.f32_to_bf16_bits(np.float32(3.5) * rng.choice(pm, size=(s.n_kv_heads, s.head_dim)))
        a, e = int(b.q_start[r]), int(b.q_start[r + 1])
        q[a:e] += np.repeat(u, s.group, axis=0)[None]
    t.q = W.f32_to_bf16_bits(q)
    got, cache = run_prefilled(b, t, mixed_launch=mixed_launch)
    want = oracle_out(b, t, cache)
    assert np.median(np.abs(want)) > 3.3                     # the rows are what was planted
    check_close(got, want, False, tol=5e-3)


def test_block_relabelling_is_bit_identical():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    g1, _ = run_prefilled(b, t)
    rng = np.random.default_rng(3)
    relabel = rng.permutation(b.n_device_blocks).astype(np.int32)
    b2 = W.MixedBatch(**{**b.__dict__, "block_ids": relabel[b.block_ids]})
    g2, _ = run_prefilled(b2, t)
    assert np.array_equal(g1, g2)


def test_chunk_split_invariance_on_gpu():
    """64-token chunk == 32 + 32 (second with prefix 32) == 63 prefill + 1 decode, within tolerance."""
    b = W.make_workload(1)
    t = W.make_tensors(b)
    whole, cache = run_prefilled(b, t)
    rows = whole[int(b.q_start[4]):int(b.q_start[5])]
    want = oracle_out(b, t, cache)[int(b.q_start[4]):]
    for cut in (32, 63):
        shape = b.shape
        # same physical table for the chunk request, processed as two requests sharing its blocks is not
        # allowed (a block belongs to one request), so run two steps over the same cache instead
        tab = b.table(4)
        cache_dev = u16_to_dev(to_device_layout(cache.pool))
        outs = []
        for (lo, hi) in ((0, cut), (cut, 64)):
            nb = -(-hi // 16)
            bb = W.MixedBatch(shape=shape, n_device_blocks=b.n_device_blocks, q_start=np.array([0, hi - lo], np.int32),
                              kv_len=np.array([hi], np.int32), bt_start=np.array([0, nb], np.int32),
                              block_ids=tab[:nb].copy(), prio=np.array([1], np.uint8))
            lay = Layer(bb)
            q = t.q[int(b.q_start[4]) + lo:int(b.q_start[4]) + hi]
            outs.append(lay.step(bb, u16_to_dev(q), cache_dev).cpu().numpy().astype(np.float64))
            lay.close()
        got = np.concatenate(outs)
        check_close(got, want, False)
        assert np.abs(got - rows).max() < 2e-3


def test_empty_batch_and_validation_errors():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    lay = Layer(b)
    ws = lay.workspace(b)
    cache_dev = u16_to_dev(to_device_layout(oracle_cache(b, t).pool))
    q = u16_to_dev(t.q)
    out = torch.zeros((b.n_tokens, 8, 128), dtype=torch.float32, device=DEV)
    empty = W.MixedBatch(shape=b.shape, n_device_blocks=64, q_start=np.zeros(1, np.int32), kv_len=np.zeros(0, np.int32),
                         bt_start=np.zeros(1, np.int32), block_ids=np.zeros(0, np.int32), prio=np.zeros(0, np.uint8))
    B.ps_step(lay.ctx, empty, q, None, None, cache_dev, out, ws, lay.ws_bytes)   # successful no-op

    def expect(code, **chg):
        d = {**b.__dict__}
        d.update(chg)
        with pytest.raises(B.PsError) as e:
            B.ps_step(lay.ctx, W.MixedBatch(**d), q, None, None, cache_dev, out, ws, lay.ws_bytes)
        assert e.value.code == code, str(e.value)

    bad = b.block_ids.copy(); bad[5] = 64
    expect(B.PS_EINVAL, block_ids=bad)
    bad = b.block_ids.copy(); bad[0] = -1
    expect(B.PS_EINVAL, block_ids=bad)
    kv = b.kv_len.copy(); kv[0] = 33
    expect(B.PS_EINVAL, kv_len=kv)                       # table length no longer matches
    qs = b.q_start.copy(); qs[1] = 0
    expect(B.PS_EINVAL, q_start=qs)                      # l_q = 0
    kv = b.kv_len.copy(); kv[4] = 63
    expect(B.PS_EINVAL, kv_len=kv)                       # l_q > kv_len
    small = Layer(b, decode_chunk=32)                    # split-K partials need a workspace
    with pytest.raises(B.PsError) as e:
        B.ps_step(small.ctx, b, q, None, None, cache_dev, out, ws, 1024)
    assert e.value.code == B.PS_ENOMEM
    small.close()
    with pytest.raises(B.PsError) as e:
        B.ps_step(lay.ctx, b, q, q, None, cache_dev, out, ws, lay.ws_bytes)
    assert e.value.code == B.PS_EINVAL
    with pytest.raises(B.PsError) as e:
        B.ps_step(lay.ctx, b, q, None, None, cache_dev, out, ws, lay.ws_bytes, None, 12345)
    assert e.value.code == B.PS_ESTATE
    # after all the rejected calls a good one still works
    B.ps_step(lay.ctx, b, q, None, None, cache_dev, out, ws, lay.ws_bytes)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    lay.close()


def test_profiling_times_are_reported():
    """Mode 1 times the phases as they run (one attention launch); mode 2 gives the decode and the
    prefill work launches of their own.  Both leave the results unchanged."""
    b = W.make_workload(2, scale=0.08)
    t = W.make_tensors(b)
    cache = oracle_cache(b, t)
    lay = Layer(b)
    ref = lay.step(b, u16_to_dev(t.q), u16_to_dev(to_device_layout(cache.pool))).clone()
    B.ps_set_profiling(lay.ctx, 1)
    got = lay.step(b, u16_to_dev(t.q), u16_to_dev(to_device_layout(cache.pool)))
    tm = B.ps_get_step_times(lay.ctx)
    assert tm["total_ms"] > 0 and tm["attention_ms"] > 0 and tm["decode_ms"] == 0 and tm["prefill_ms"] == 0
    assert 500 < tm["decode_mhz"] < 2600 and 500 < tm["prefill_mhz"] < 2600      # the shader clock the roles ran at
    assert torch.equal(got, ref)
    B.ps_set_profiling(lay.ctx, 2)
    got = lay.step(b, u16_to_dev(t.q), u16_to_dev(to_device_layout(cache.pool)))
    tm = B.ps_get_step_times(lay.ctx)
    assert tm["decode_ms"] > 0 and tm["prefill_ms"] > 0
    assert 500 < tm["decode_mhz"] < 2600 and 500 < tm["prefill_mhz"] < 2600
    assert abs(tm["attention_ms"] - tm["decode_ms"] - tm["prefill_ms"]) < 1e-3
    # the decode slots are cut differently in mode 2 (whole chip), so only closeness is asserted
    assert (got.float() - ref.float()).abs().max().item() < 2e-2
    with pytest.raises(B.PsError) as e:
        B.ps_set_profiling(lay.ctx, 3)
    assert e.value.code == B.PS_EINVAL
    # Many steps back to back, read once: the mean over the steps since the last read (the library keeps the events
    # of the last 64).  It lies between the fastest and the slowest step read one at a time, give or take what running
    # back to back changes; a second read with no step in between repeats the first.
    B.ps_set_profiling(lay.ctx, 1)
    q_dev, c_dev = u16_to_dev(t.q), u16_to_dev(to_device_layout(cache.pool))
    singles = []
    for _ in range(5):
        lay.step(b, q_dev, c_dev)
        singles.append(B.ps_get_step_times(lay.ctx)["attention_ms"])
    for _ in range(70):
        lay.step(b, q_dev, c_dev)
    mean = B.ps_get_step_times(lay.ctx)
    assert 0.5 * min(singles) < mean["attention_ms"] < 2.0 * max(singles)
    assert mean["total_ms"] >= mean["attention_ms"] > 0
    assert B.ps_get_step_times(lay.ctx) == mean
    with pytest.raises(B.PsError) as e:          # switching the mode restarts the series
        B.ps_set_profiling(lay.ctx, 1)
        B.ps_get_step_times(lay.ctx)
    assert e.value.code == B.PS_ESTATE
    lay.close()
