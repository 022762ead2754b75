"""ps_step_next_layer: the batch of a forward pass is planned and uploaded once (ps_step on the first
layer), the following layers run the same work lists over their own q, new K/V rows, cache and
output.  Every layer's output must equal the oracle's on that layer's tensors, and every layer's
cache, after its append, the oracle's cache bit for bit."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from paper_2512_12928_amd.kvlayout import from_device_layout, to_device_layout
from gpu_harness import DEV, check_close, dev_to_u16, oracle_cache, u16_to_dev

pytestmark = pytest.mark.gpu


def layer_tensors(b, ell, append):
    t = W.make_tensors(b, seed=b.seed + 77 * (ell + 1))
    full = oracle_cache(b, t)
    want = A.paged_attention(t.q, full, b.q_start, b.kv_len, b.bt_start, b.block_ids)
    start = oracle_cache(b, t, upto_prefix=True) if append else full
    k_new, v_new = t.new_rows(b) if append else (None, None)
    return dict(q=u16_to_dev(t.q), pool=u16_to_dev(to_device_layout(start.pool)), want=want, full=full.pool,
                k_new=None if k_new is None else u16_to_dev(k_new), v_new=None if v_new is None else u16_to_dev(v_new))


@pytest.mark.parametrize("append", [True, False])
@pytest.mark.parametrize("workload,scale,own_streams", [(1, 1.0, 0), (2, 0.08, 0), (2, 0.08, 1), (5, 0.05, 0)])
def test_layers_after_the_first_reuse_the_plan(workload, scale, own_streams, append):
    b = W.make_workload(workload) if workload == 1 else W.make_workload(workload, scale=scale)
    s = b.shape
    n_layers = 3
    layers = [layer_tensors(b, ell, append) for ell in range(n_layers)]
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, b.n_device_blocks, 0, out_dtype=B.PS_F32, own_streams=own_streams)
    nbytes = B.ps_workspace_bytes(ctx, b.n_req, b.n_tokens, len(b.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    outs = [torch.full((b.n_tokens, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.float32, device=DEV)
            for _ in layers]
    stream = torch.cuda.current_stream()
    for _ in range(2):   # two passes back to back: the second ps_step meets buffers the first pass's layers used
        for ell, L in enumerate(layers):
            if ell == 0:
                B.ps_step(ctx, b, L["q"], L["k_new"], L["v_new"], L["pool"], outs[ell], ws, nbytes, stream)
            else:
                B.ps_step_next_layer(ctx, L["q"], L["k_new"], L["v_new"], L["pool"], outs[ell], ws, nbytes, stream)
    torch.cuda.synchronize()
    for ell, L in enumerate(layers):
        check_close(outs[ell].cpu().numpy().astype(np.float64), L["want"], False)
        assert np.array_equal(from_device_layout(dev_to_u16(L["pool"]), s.n_kv_heads), L["full"])
    B.ps_destroy(ctx)


def test_next_layer_needs_a_batch():
    b = W.make_workload(1)
    s = b.shape
    L = layer_tensors(b, 0, True)
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, b.n_device_blocks, 0, out_dtype=B.PS_F32)
    nbytes = B.ps_workspace_bytes(ctx, b.n_req, b.n_tokens, len(b.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out = torch.zeros((b.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.float32, device=DEV)
    args = (L["q"], L["k_new"], L["v_new"], L["pool"], out, ws, nbytes)

    def refused(code, *a):
        with pytest.raises(B.PsError) as e:
            B.ps_step_next_layer(ctx, *a)
        assert e.value.code == code, str(e.value)

    refused(B.PS_ESTATE, *args)                                  # nothing planned yet
    B.ps_step(ctx, b, *args)
    B.ps_step_next_layer(ctx, *args)                             # now it runs
    B.ps_set_profiling(ctx, 1)                                   # and reports its phases like a ps_step
    B.ps_step_next_layer(ctx, *args)
    torch.cuda.synchronize()
    times = B.ps_get_step_times(ctx)
    assert times["attention_ms"] > 0 and times["append_ms"] > 0 and times["total_ms"] >= times["attention_ms"]
    assert times["upload_ms"] < 0.5 * times["total_ms"]          # nothing is uploaded
    B.ps_set_profiling(ctx, 0)
    refused(B.PS_EINVAL, L["q"], None, None, L["pool"], out, ws, nbytes)   # that ps_step had new K/V rows
    refused(B.PS_EINVAL, None, L["k_new"], L["v_new"], L["pool"], out, ws, nbytes)
    bad = W.make_workload(1)
    bad.kv_len = bad.kv_len.copy()
    bad.kv_len[0] += 100                                         # table length no longer matches
    with pytest.raises(B.PsError):
        B.ps_step(ctx, bad, *args)
    refused(B.PS_ESTATE, *args)                                  # a failed ps_step leaves no plan behind
    empty = W.MixedBatch(shape=s, n_device_blocks=b.n_device_blocks, q_start=np.zeros(1, np.int32), kv_len=np.zeros(0, np.int32),
                         bt_start=np.zeros(1, np.int32), block_ids=np.zeros(0, np.int32), prio=np.zeros(0, np.uint8))
    B.ps_step(ctx, b, *args)
    B.ps_step(ctx, empty, *args)
    refused(B.PS_ESTATE, *args)                                  # nor does an empty batch
    torch.cuda.synchronize()
    B.ps_destroy(ctx)


def test_layers_after_the_first_replay_as_a_hip_graph():
    """ps_step_next_layer is kernel launches only (no allocation, no copy, no event unless profiling or a
    ticket is asked for), so a caller can capture the layers after the first into a HIP graph.  Every replay,
    with eager work and synchronisation in between, must give what the eager calls give."""
    b = W.make_workload(2, scale=0.08)
    s = b.shape
    n_layers = 4
    layers = [layer_tensors(b, ell, True) for ell in range(n_layers)]
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, b.n_device_blocks, 0, out_dtype=B.PS_F32)
    nbytes = B.ps_workspace_bytes(ctx, b.n_req, b.n_tokens, len(b.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    outs = [torch.zeros((b.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.float32, device=DEV) for _ in layers]
    side = torch.cuda.Stream()

    def first_layer():
        L = layers[0]
        B.ps_step(ctx, b, L["q"], L["k_new"], L["v_new"], L["pool"], outs[0], ws, nbytes, side)

    def other_layers():
        for ell in range(1, n_layers):
            L = layers[ell]
            B.ps_step_next_layer(ctx, L["q"], L["k_new"], L["v_new"], L["pool"], outs[ell], ws, nbytes, side)

    first_layer()
    other_layers()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        other_layers()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        first_layer()                                            # eager, on the same stream
        side.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        torch.cuda.synchronize()
        for ell in range(n_layers):
            assert torch.equal(outs[ell], eager[ell]), (rep, ell)
            check_close(outs[ell].cpu().numpy().astype(np.float64), layers[ell]["want"], False)
    del graph
    B.ps_destroy(ctx)
