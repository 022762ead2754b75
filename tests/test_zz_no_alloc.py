"""ps_step_static -- the entry point for callers that cannot allocate -- against ps_step: two calls in a row on one
context, the second with a smaller batch, each compared with ps_step's output on the same inputs (same kernels;
bit-identical unless the two plan the launch differently, never further apart than the parity tolerance of 1e-2 on
the f32 output path) and with the fp64 oracle.  Also: a batch too large for the fixed array is refused with
PS_ENOMEM and nothing is enqueued."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from gpu_harness import DEV, check_close, oracle_cache, u16_to_dev
from paper_2512_12928_amd.kvlayout import to_device_layout

pytestmark = pytest.mark.gpu


def device_args(batch, tens, M):
    """Cache holding every request's prefix (NaN elsewhere), q, this step's new rows; on the device."""
    pre = oracle_cache(batch, tens, upto_prefix=True).pool
    pool = np.full((M,) + pre.shape[1:], W.BF16_NAN, dtype=np.uint16)
    pool[:pre.shape[0]] = pre
    k_new, v_new = tens.new_rows(batch)
    return u16_to_dev(to_device_layout(pool)), u16_to_dev(tens.q), u16_to_dev(k_new), u16_to_dev(v_new)


def test_static_entry_point_two_calls_second_smaller():
    big = W.make_workload(2, scale=0.25)                 # 64 decode requests (several cut into split-K partials) + 4 chunks
    small = W.make_workload(2, scale=0.06, seed=77)      # 15 decode requests + 4 short chunks, same head counts
    assert small.n_tokens < big.n_tokens and len(small.block_ids) < len(big.block_ids)
    s = big.shape
    M = max(big.n_device_blocks, small.n_device_blocks)
    ctx_ref = B.ps_create(s.n_q_heads, s.n_kv_heads, M, 0, out_dtype=B.PS_F32)
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, M, 0, out_dtype=B.PS_F32)
    nbytes = B.ps_workspace_bytes(ctx_ref, big.n_req, big.n_tokens, len(big.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    results = []
    for batch in (big, small):                           # two static calls in a row on ctx, the second smaller
        tens = W.make_tensors(batch)
        want = A.paged_attention(tens.q, oracle_cache(batch, tens), batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids)
        cache_ref, q, kn, vn = device_args(batch, tens, M)
        cache = cache_ref.clone()
        ref = torch.full((batch.n_tokens, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.float32, device=DEV)
        got = torch.full_like(ref, float("nan"))
        B.ps_step(ctx_ref, batch, q, kn, vn, cache_ref, ref, ws, nbytes)
        B.ps_step_static(ctx, batch, q, kn, vn, cache, got)
        torch.cuda.synchronize()
        results.append((batch, want, ref.cpu().numpy().astype(np.float64), got.cpu().numpy().astype(np.float64),
                        cache_ref.cpu().numpy(), cache.cpu().numpy()))
    for batch, want, ref, got, cache_ref, cache in results:
        check_close(ref, want, False)
        check_close(got, want, False)                    # the oracle's bar: max-abs 1e-2 on the f32 path
        assert np.abs(got - ref).max() <= 1e-2           # and against the existing entry point
        assert np.array_equal(cache, cache_ref)          # the append wrote the same bytes
    B.ps_destroy(ctx_ref)
    B.ps_destroy(ctx)


def test_static_entry_point_rejects_what_does_not_fit():
    shape = W.LayerShape(8, 2)
    n = 70_000                                   # 70 000 one-token requests: the description alone exceeds 2 MiB
    rng = np.random.default_rng(0)
    batch = W.build_batch(shape, [(1, 1)] * n, [1] * n, rng, pool_factor=1.0, seed=0)
    ctx = B.ps_create(shape.n_q_heads, shape.n_kv_heads, batch.n_device_blocks, 0)
    q = torch.zeros((n, 8, 128), dtype=torch.bfloat16, device=DEV)
    kv = torch.zeros((n, 2, 128), dtype=torch.bfloat16, device=DEV)
    cache = torch.zeros((batch.n_device_blocks, shape.block_bytes // 2), dtype=torch.bfloat16, device=DEV)
    out = torch.full((n, 8, 128), 7.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.PsError) as e:
        B.ps_step_static(ctx, batch, q, kv, kv, cache, out)
    assert e.value.code == B.PS_ENOMEM
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())              # nothing was enqueued
    B.ps_destroy(ctx)
