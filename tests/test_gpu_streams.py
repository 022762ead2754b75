"""Steps of one context issued on alternating streams (each with a workspace of its own): the context's two
device copies of the batch description are reused every other step, so a step must not overwrite a copy that
a step on the other stream may still be reading.  Normal use, nothing is raced on purpose: the outputs of six
steps over three different batches must equal those of the same steps on a single stream, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from gpu_harness import DEV, oracle_cache, u16_to_dev
from paper_2512_12928_amd.kvlayout import to_device_layout

pytestmark = pytest.mark.gpu


def test_steps_on_alternating_streams_equal_single_stream():
    batches = [W.make_workload(2, scale=s, seed=100 + i) for i, s in enumerate((0.25, 0.12, 0.2))]
    shape = batches[0].shape
    M = max(b.n_device_blocks for b in batches)
    tens = [W.make_tensors(b) for b in batches]
    caches, qs = [], []
    for b, t in zip(batches, tens):
        pool = oracle_cache(b, t).pool
        full = np.zeros((M,) + pool.shape[1:], dtype=np.uint16)
        full[:pool.shape[0]] = pool
        caches.append(u16_to_dev(to_device_layout(full)))
        qs.append(u16_to_dev(t.q))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]

    def run(alternate):
        ctx = B.ps_create(shape.n_q_heads, shape.n_kv_heads, M, 0, out_dtype=B.PS_F32)
        nbytes = max(B.ps_workspace_bytes(ctx, b.n_req, b.n_tokens, len(b.block_ids)) for b in batches)
        wss = [torch.empty(nbytes, dtype=torch.uint8, device=DEV) for _ in range(2)]
        outs = []
        torch.cuda.synchronize()
        for step in range(6):
            i = step % 3
            b = batches[i]
            out = torch.full((b.n_tokens, shape.n_q_heads, 128), float("nan"), dtype=torch.float32, device=DEV)
            k = step % 2 if alternate else 0
            B.ps_step(ctx, b, qs[i], None, None, caches[i], out, wss[k], nbytes, streams[k])
            outs.append(out)
        torch.cuda.synchronize()
        B.ps_destroy(ctx)
        return [o.cpu().numpy() for o in outs]

    single = run(False)
    both = run(True)
    for a, b in zip(single, both):
        assert np.isfinite(a).all() and np.array_equal(a, b)
