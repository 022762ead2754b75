"""Pins for oracle A (paged causal attention, fp64).  Each test checks the oracle against
something other than itself: a pure-Python brute force of the definition, a closed form,
an invariant, or a library routine as a third opinion.  CPU only."""
import math

import numpy as np
import pytest

from oracle import attention as A
from paper_2512_12928_amd import workloads as W


def brute_force(q, k, v, scale):
    """The definition with Python loops and math.exp; q [l_q,Hq,d], k/v [L,Hkv,d] lists/arrays."""
    l_q, Hq, d = q.shape
    L, Hkv, _ = k.shape
    G = Hq // Hkv
    p = L - l_q
    out = np.zeros((l_q, Hq, d))
    for i in range(l_q):
        n = p + i + 1
        for h in range(Hq):
            g = h // G
            s = [sum(float(q[i, h, x]) * float(k[j, g, x]) for x in range(d)) * scale for j in range(n)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            z = sum(e)
            for x in range(d):
                out[i, h, x] = sum(e[j] * float(v[j, g, x]) for j in range(n)) / z
    return out


def small_case(seed, l_q, L, Hq=4, Hkv=2, d=8):
    rng = np.random.default_rng(seed)
    q = A.bf16_to_f64(W.normal_bf16(rng, (l_q, Hq, d)))
    k = A.bf16_to_f64(W.normal_bf16(rng, (L, Hkv, d)))
    v = A.bf16_to_f64(W.normal_bf16(rng, (L, Hkv, d)))
    return q, k, v


def test_bf16_decode_exact():
    # bit patterns with known values: 1.0, -2.0, 0.5, 3.140625 (0x4049), smallest normal
    bits = np.array([0x3F80, 0xC000, 0x3F00, 0x4049, 0x0080], dtype=np.uint16)
    want = np.array([1.0, -2.0, 0.5, 3.140625, 2.0 ** -126])
    assert (A.bf16_to_f64(bits) == want).all()


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 (even) and 1+2^-7 -> 1.0; 1 + 3*2^-8 ties up to 1+2^-6
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = A.bf16_to_f64(W.f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


@pytest.mark.parametrize("l_q,L", [(1, 1), (1, 7), (3, 3), (4, 9), (5, 21)])
def test_dense_matches_brute_force(l_q, L):
    q, k, v = small_case(10 + l_q + L, l_q, L)
    scale = 1.0 / math.sqrt(q.shape[-1])
    got = A.dense_attention(q, k, v)
    want = brute_force(q, k, v, scale)
    assert np.abs(got - want).max() < 1e-13


def test_scale_is_inverse_sqrt_d_and_overridable():
    q, k, v = small_case(3, 2, 6)
    a = A.dense_attention(q, k, v)
    b = A.dense_attention(q, k, v, scale=1.0 / math.sqrt(8))
    c = A.dense_attention(q, k, v, scale=0.5)
    assert np.array_equal(a, b) and not np.allclose(a, c)
    assert np.abs(c - brute_force(q, k, v, 0.5)).max() < 1e-13


def test_softmax_rows_sum_to_one_and_causal_zeros():
    q, k, v = small_case(4, 6, 20)
    _, P = A.dense_attention(q, k, v, return_probs=True)
    assert np.abs(P.sum(-1) - 1.0).max() < 1e-12
    p = 20 - 6
    for i in range(6):
        assert (P[i, :, p + i + 1:] == 0).all() and (P[i, :, :p + i + 1] > 0).all()


def test_single_visible_key_returns_v0_exactly():
    q, k, v = small_case(5, 3, 3)
    o = A.dense_attention(q, k, v)
    G = 2
    for h in range(4):
        assert np.array_equal(o[0, h], v[0, h // G])


def test_constant_v_and_equal_keys():
    q, k, v = small_case(6, 2, 11)
    vc = np.full_like(v, 0.625)
    assert np.abs(A.dense_attention(q, k, vc) - 0.625).max() < 1e-15
    ke = np.broadcast_to(k[:1], k.shape).copy()   # all keys equal -> uniform weights -> running mean of V
    o = A.dense_attention(q, ke, v)
    p = 11 - 2
    for i in range(2):
        for h in range(4):
            assert np.abs(o[i, h] - v[:p + i + 1, h // 2].mean(0)).max() < 1e-14


def test_gqa_equals_mha_after_replication():
    q, k, v = small_case(7, 3, 10, Hq=6, Hkv=2)
    o = A.dense_attention(q, k, v)
    o2 = A.dense_attention(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1))
    assert np.array_equal(o, o2)
    # the grouping is "consecutive q heads share a kv head": head 2 must use kv head 0, head 3 kv head 1
    v2 = v.copy(); v2[:, 1] += 1.0
    d = A.dense_attention(q, k, v2) - o
    assert np.abs(d[:, :3]).max() == 0 and np.abs(d[:, 3:] - 1.0).max() < 1e-12


def test_chunk_split_invariance():
    """One 12-token chunk == chunks 5+7 == 11 prefill + 1 decode, row by row."""
    q, k, v = small_case(8, 12, 12)
    whole = A.dense_attention(q, k, v)
    a = A.dense_attention(q[:5], k[:5], v[:5])
    b = A.dense_attention(q[5:], k, v)
    assert np.abs(np.concatenate([a, b]) - whole).max() < 1e-14
    c = A.dense_attention(q[:11], k[:11], v[:11])
    dcode = A.dense_attention(q[11:], k, v)
    assert np.abs(np.concatenate([c, dcode]) - whole).max() < 1e-14


def test_library_third_opinion_sdpa():
    torch = pytest.importorskip("torch")
    q, k, v = small_case(9, 5, 5, Hq=4, Hkv=4, d=16)   # p = 0 so torch's causal flag applies
    o = A.dense_attention(q, k, v)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(o - ref).max() < 1e-12


def _fill_cache(batch, tens, fill):
    s = batch.shape
    c = A.PagedKV(batch.n_device_blocks, s.n_kv_heads, s.block_tokens, s.head_dim, fill=fill)
    for r in range(batch.n_req):
        c.append(batch.table(r), 0, tens.k[r], tens.v[r])
    return c


def test_paged_equals_dense_exactly_on_cfg1():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    cache = _fill_cache(b, t, W.BF16_NAN)   # unreferenced blocks and tail slots are NaN
    got = A.paged_attention(t.q, cache, b.q_start, b.kv_len, b.bt_start, b.block_ids)
    assert np.isfinite(got).all()
    for r in range(b.n_req):
        a, e = b.q_start[r], b.q_start[r + 1]
        want = A.dense_attention(A.bf16_to_f64(t.q[a:e]), A.bf16_to_f64(t.k[r]), A.bf16_to_f64(t.v[r]))
        assert np.array_equal(got[a:e], want)


def test_paged_slot_addressing_by_hand():
    """Token j must come from block table[j // 16], slot j % 16 (checked with a hand-built pool)."""
    c = A.PagedKV(4, 1, 16, 2)
    table = np.array([3, 1], dtype=np.int32)
    L = 20
    kbits = W.f32_to_bf16_bits(np.arange(L * 2, dtype=np.float32).reshape(L, 1, 2))
    vbits = W.f32_to_bf16_bits(-np.arange(L * 2, dtype=np.float32).reshape(L, 1, 2))
    c.append(table, 0, kbits, vbits)
    assert np.array_equal(c.pool[3, 0, 0, 5], kbits[5, 0]) and np.array_equal(c.pool[1, 0, 0, 3], kbits[19, 0])
    assert np.array_equal(c.pool[1, 1, 0, 0], vbits[16, 0]) and (c.pool[[0, 2]] == 0).all()
    k2, v2 = c.gather(table, L)
    assert np.array_equal(k2, kbits) and np.array_equal(v2, vbits)


def test_block_id_reshuffle_leaves_output_bit_identical():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    o1 = A.paged_attention(t.q, _fill_cache(b, t, 0), b.q_start, b.kv_len, b.bt_start, b.block_ids)
    rng = np.random.default_rng(1)
    relabel = rng.permutation(b.n_device_blocks).astype(np.int32)
    b2 = W.MixedBatch(**{**b.__dict__, "block_ids": relabel[b.block_ids]})
    o2 = A.paged_attention(t.q, _fill_cache(b2, t, W.BF16_NAN), b2.q_start, b2.kv_len, b2.bt_start, b2.block_ids)
    assert np.array_equal(o1, o2)


def test_append_in_two_steps_equals_one():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    c1 = _fill_cache(b, t, 0)
    s = b.shape
    c2 = A.PagedKV(b.n_device_blocks, s.n_kv_heads, s.block_tokens, s.head_dim)
    for r in range(b.n_req):
        cut = int(b.kv_len[r]) - b.l_q(r)
        c2.append(b.table(r), 0, t.k[r][:cut], t.v[r][:cut])
        c2.append(b.table(r), cut, t.k[r][cut:], t.v[r][cut:])
    assert np.array_equal(c1.pool, c2.pool)


@pytest.mark.parametrize("cuts", [[0, 40], [0, 1, 40], [0, 16, 32, 40], [0, 7, 8, 33, 40]])
def test_split_k_merge_identity(cuts):
    rng = np.random.default_rng(11)
    q = rng.standard_normal(16)
    k = rng.standard_normal((40, 16)) * 3
    v = rng.standard_normal((40, 16))
    scale = 0.25
    parts = [A.partial_softmax(q, k[a:b], v[a:b], scale) for a, b in zip(cuts[:-1], cuts[1:])]
    got = A.merge_partials(parts)
    want = A.dense_attention(q[None, None], k[:, None], v[:, None], scale)[0, 0]
    assert np.abs(got - want).max() < 1e-13


def test_attention_rows_matches_full():
    b = W.make_workload(1)
    t = W.make_tensors(b)
    r = 4                                   # the 64-token prefill chunk, prefix 0
    a = int(b.q_start[r])
    full = A.dense_attention(A.bf16_to_f64(t.q[a:a + 64]), A.bf16_to_f64(t.k[r]), A.bf16_to_f64(t.v[r]))
    rows = np.array([0, 15, 16, 63])
    got = A.attention_rows(t.q[a + rows], t.k[r], t.v[r], rows + 1)
    assert np.abs(got - full[rows]).max() < 1e-14


def test_workload_shapes_match_config_text():
    b = W.make_workload(1)
    assert b.kv_len.tolist() == [17, 64, 130, 200, 64] and b.n_tokens == 68 and len(b.block_ids) == 32
    assert len(set(b.block_ids.tolist())) == 32 and b.block_ids.max() < 64
    for idx, (nd, nt) in {2: (256, 2304), 4: (32, 4128), 5: (512, 8704)}.items():
        w = W.make_workload(idx)
        assert len(w.decode_reqs) == nd and w.n_tokens == nt
        assert len(set(w.block_ids.tolist())) == len(w.block_ids)
    assert W.make_workload(4).causal_pairs() == 4096 * 16384 + 4096 * 4097 // 2
