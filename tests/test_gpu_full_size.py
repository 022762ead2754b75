"""Parity at the full workload sizes, in the configuration bench.py times (bf16 output, append on,
library-chosen partition size): sampled outputs against the fp64 oracle, one request / one row at a time.
Oracle inputs are the pool as generated (read back BEFORE the step) plus the step's own k_new / v_new rows;
nothing the HIP path wrote is fed to the oracle.  The appended cache rows are checked bit for bit."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from paper_2512_12928_amd.kvlayout import request_kv
from gpu_harness import DEV

pytestmark = pytest.mark.gpu


def bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("idx", [2, 4, 5])
def test_full_size_sampled_parity(idx):
    batch = W.make_workload(idx)
    s = batch.shape
    pool, q, kn, vn = W.device_inputs(batch, batch.seed, DEV)
    rng = np.random.default_rng(idx)
    dec, pre = batch.decode_reqs, batch.prefill_reqs
    by_len = dec[np.argsort(batch.kv_len[dec])]
    sample_dec = sorted(set([int(by_len[0]), int(by_len[-1]), int(by_len[len(by_len) // 2])] +
                            [int(x) for x in rng.choice(dec, 5, replace=False)]))
    # logical K/V of the sampled requests before the step, with the step's new rows overlaid
    def logical(r):
        tab = torch.from_numpy(batch.table(r).astype(np.int64)).to(DEV)
        L, lq, a = int(batch.kv_len[r]), batch.l_q(r), int(batch.q_start[r])
        k, v = request_kv(bits(pool[tab]), s.n_kv_heads, L)
        k[L - lq:] = bits(kn[a:a + lq])
        v[L - lq:] = bits(vn[a:a + lq])
        return k, v
    kv = {r: logical(r) for r in sample_dec + [int(r) for r in pre]}

    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, 0, out_dtype=B.PS_BF16)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out = torch.full((batch.n_tokens, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.ps_step(ctx, batch, q, kn, vn, pool, out, ws, nbytes, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()          # every row of the full batch was written
    q_bits = bits(q)

    def close(got, want, what):
        err = np.abs(got - want)
        bad = err > 1e-2 + 2.0 ** -8 * np.abs(want)
        assert not bad.any(), "%s: max abs err %.4g" % (what, err.max())
        return float(err.max())

    worst = 0.0
    for r in sample_dec:
        a = int(batch.q_start[r])
        k, v = kv[r]
        want = A.dense_attention(A.bf16_to_f64(q_bits[a:a + 1]), A.bf16_to_f64(k), A.bf16_to_f64(v))
        worst = max(worst, close(out[a:a + 1].float().cpu().numpy().astype(np.float64), want, "decode req %d" % r))
    for r in [int(x) for x in pre]:
        a, lq, L = int(batch.q_start[r]), batch.l_q(r), int(batch.kv_len[r])
        rows = np.unique(np.concatenate([np.arange(4), np.arange(lq - 4, lq), [31, 32, 63, 64, lq // 2],
                                         rng.integers(0, lq, 12)]))
        k, v = kv[r]
        want = A.attention_rows(q_bits[a + rows], k, v, (L - lq) + rows + 1)
        got = out[a + torch.from_numpy(rows).to(DEV)].float().cpu().numpy().astype(np.float64)
        worst = max(worst, close(got, want, "prefill req %d" % r))
        # the appended rows: cache == generated prefix + new rows, bit for bit
        tab = torch.from_numpy(batch.table(r).astype(np.int64)).to(DEV)
        k2, v2 = request_kv(bits(pool[tab]), s.n_kv_heads, L)
        assert np.array_equal(k2, k) and np.array_equal(v2, v)
    for r in sample_dec:
        tab = torch.from_numpy(batch.table(r).astype(np.int64)).to(DEV)
        k2, v2 = request_kv(bits(pool[tab]), s.n_kv_heads, int(batch.kv_len[r]))
        assert np.array_equal(k2, kv[r][0]) and np.array_equal(v2, kv[r][1])
    print(batch.name, "sampled %d decode requests, %d prefill chunks; worst abs err %.4g" % (len(sample_dec), len(pre), worst))
    B.ps_destroy(ctx)


def test_workload3_swaps_under_attention():
    """Workload 3 at full size: per step 512 blocks out and 512 in under a copy budget on side streams while
    the attention step runs; copied blocks bit-exact against the copy oracle, every other byte untouched,
    attention on a sampled decode request unaffected."""
    from oracle import blockcopy as C
    batch = W.make_workload(3)
    s = batch.shape
    assert batch.n_device_blocks == 40_000
    pool, q, kn, vn = W.device_inputs(batch, batch.seed, DEV)
    Mh, bb = 1200, s.block_bytes
    rng = np.random.default_rng(33)
    out_ids, out_slots = W.make_swap_lists(512, batch.n_device_blocks, Mh, rng, exclude_device=batch.block_ids)
    free = np.setdiff1d(np.arange(batch.n_device_blocks, dtype=np.int32), np.concatenate([batch.block_ids, out_ids]))
    in_ids = rng.permutation(free)[:512].astype(np.int32)
    in_slots = np.setdiff1d(np.arange(Mh, dtype=np.int32), out_slots)[:512].astype(np.int32)
    host_np = rng.integers(0, 256, (Mh, bb), dtype=np.uint8)
    host = torch.from_numpy(host_np.copy()).pin_memory()
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, Mh)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out = torch.empty((batch.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    compute, so, si = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    touched = np.concatenate([out_ids, in_ids])
    before = pool.view(torch.uint8)[torch.from_numpy(touched.astype(np.int64)).to(DEV)].cpu().numpy()
    torch.cuda.synchronize()
    cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
    for budget in (300, -1):
        n_o, tk_o = B.ps_swap_out(ctx, out_ids, out_slots, budget, pool, host, so)
        n_i, tk_i = B.ps_swap_in(ctx, in_slots, in_ids, budget, host, pool, si)
        B.ps_step(ctx, cb, q, None, None, pool, out, ws, nbytes, compute)
        B.ps_ticket_wait(ctx, tk_o); B.ps_ticket_wait(ctx, tk_i)
        torch.cuda.synchronize()
        # oracle on host copies of exactly the touched device blocks
        dev_small = {int(b): before[i].copy() for i, b in enumerate(touched)}
        want_host = host_np.copy()
        m_o = C.n_moved(512, budget)
        assert n_o == m_o and n_i == m_o
        for k in range(m_o):
            want_host[out_slots[k]] = dev_small[int(out_ids[k])]
        for k in range(m_o):
            dev_small[int(in_ids[k])] = host_np[in_slots[k]]
        assert np.array_equal(host.numpy(), want_host)
        after = pool.view(torch.uint8)[torch.from_numpy(touched.astype(np.int64)).to(DEV)].cpu().numpy()
        for i, b in enumerate(touched):
            assert np.array_equal(after[i], dev_small[int(b)])
        host_np = want_host
        before = after
    # every block outside the reload list is unchanged: compare with the pool generated again from the seed
    idx_in = torch.from_numpy(in_ids.astype(np.int64)).to(DEV)
    mask = torch.ones(batch.n_device_blocks, dtype=torch.bool, device=DEV)
    mask[idx_in] = False
    pool0, _, _, _ = W.device_inputs(batch, batch.seed, DEV)
    assert torch.equal(pool[mask], pool0[mask])
    del pool0
    # attention output of one decode request equals the oracle's
    r = int(batch.decode_reqs[7])
    tab = torch.from_numpy(batch.table(r).astype(np.int64)).to(DEV)
    k, v = request_kv(bits(pool[tab]), s.n_kv_heads, int(batch.kv_len[r]))
    a = int(batch.q_start[r])
    want = A.dense_attention(A.bf16_to_f64(bits(q[a:a + 1])), A.bf16_to_f64(k), A.bf16_to_f64(v))
    got = out[a:a + 1].float().cpu().numpy().astype(np.float64)
    assert (np.abs(got - want) <= 1e-2 + 2.0 ** -8 * np.abs(want)).all()
    B.ps_destroy(ctx)
