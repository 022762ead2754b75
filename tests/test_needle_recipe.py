"""The second input recipe of the long-context parity tests (workloads.make_needle_plan), checked with the
oracle alone: at the longest context of every timed workload, taking ANY one 32-token tile away from what a row
attends over moves that row's output by more than the 1e-2 parity tolerance -- so a kernel that loses a tile, a
split-K partial or a KV partition cannot pass -- whereas with plain N(0,1) inputs it does not."""
import numpy as np
import pytest

from oracle import attention as A
from paper_2512_12928_amd import workloads as W

TOL = 1e-2


def single_request(index):
    """A one-request batch with the shape and the longest decode context of workload `index`."""
    full = W.make_workload(index)
    L = int(full.kv_len[full.decode_reqs].max())
    rng = np.random.default_rng(index)
    return W.build_batch(full.shape, [(1, L)], [1], rng, seed=full.seed), L


def leave_one_tile_out(q, k, v, tiles):
    """min over the given tiles of max|o_full - o_without_tile| (one kv-head's query heads, one query row)."""
    full = A.dense_attention(q, k, v)
    worst = np.inf
    for t in tiles:
        keep = np.ones(k.shape[0], dtype=bool)
        keep[t * 32:(t + 1) * 32] = False
        o = A.dense_attention(q, k[keep], v[keep])
        worst = min(worst, float(np.abs(o - full).max()))
    return worst


@pytest.mark.parametrize("index", [2, 4, 5])
def test_every_tile_of_the_longest_decode_context_is_visible(index):
    b, L = single_request(index)
    t, plan = W.make_needle_tensors(b)
    G = b.shape.group
    q = A.bf16_to_f64(t.q[:, :G])                       # the query heads of kv-head 0
    k, v = A.bf16_to_f64(t.k[0][:, :1]), A.bf16_to_f64(t.v[0][:, :1])
    n_tiles = -(-L // 32)
    worst = leave_one_tile_out(q, k, v, range(n_tiles))
    print("workload %d: kv_len %d, %d tiles, amplitude %.4g, smallest change %.4g" % (index, L, n_tiles, plan.amp[0], worst))
    assert worst > TOL


def test_plain_normal_inputs_would_not_show_a_lost_tile():
    b, L = single_request(4)
    t = W.make_tensors(b)
    G = b.shape.group
    q = A.bf16_to_f64(t.q[:, :G])
    k, v = A.bf16_to_f64(t.k[0][:, :1]), A.bf16_to_f64(t.v[0][:, :1])
    n_tiles = -(-L // 32)
    worst = leave_one_tile_out(q, k, v, range(0, n_tiles, 64))
    assert worst < TOL          # this is why the needle recipe exists


def test_every_tile_of_a_long_prefill_row_is_visible():
    """Workload 4's chunk: 4096 query tokens over a 16384-token prefix; rows in the middle and at the end."""
    full = W.make_workload(4)
    r = int(full.prefill_reqs[0])
    lq, L = full.l_q(r), int(full.kv_len[r])
    b = W.build_batch(full.shape, [(lq, L)], [1], np.random.default_rng(0), seed=full.seed)
    t, plan = W.make_needle_tensors(b)
    G = b.shape.group
    k, v = A.bf16_to_f64(t.k[0][:, :1]), A.bf16_to_f64(t.v[0][:, :1])
    for row in (lq // 2, lq - 1):
        n = L - lq + row + 1
        q = A.bf16_to_f64(t.q[row:row + 1, :G])
        worst = leave_one_tile_out(q, k[:n], v[:n], range(0, -(-n // 32), 3))
        assert worst > TOL, row


def test_needle_tensors_match_the_plan():
    b = W.make_workload(2, scale=0.1)
    t, plan = W.make_needle_tensors(b)
    for r in range(b.n_req):
        L = int(b.kv_len[r])
        assert len(plan.pos[r]) == -(-L // 32) and (plan.pos[r] // 32 == np.arange(len(plan.pos[r]))).all() and plan.pos[r].max() < L
        assert np.array_equal(t.k[r][plan.pos[r]], plan.k_rows(r)) and np.array_equal(t.v[r][plan.pos[r]], plan.v_rows(r))
        vv = W.bf16_bits_to_f32(plan.v_rows(r))
        assert (np.abs(vv) == plan.amp[r]).all()
