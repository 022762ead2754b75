"""Shared plumbing of the GPU parity tests: device buffers through torch, calls through the C ABI,
expected values from the oracle only."""
import numpy as np
import torch

from oracle import attention as A
from paper_2512_12928_amd import binding as B
from paper_2512_12928_amd import workloads as W
from paper_2512_12928_amd.kvlayout import from_device_layout, to_device_layout

DEV = "cuda:0"


def u16_to_dev(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device int16 tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def dev_to_u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def oracle_cache(batch: W.MixedBatch, tens: W.StepTensors, upto_prefix: bool = False, fill=W.BF16_NAN) -> A.PagedKV:
    s = batch.shape
    c = A.PagedKV(batch.n_device_blocks, s.n_kv_heads, s.block_tokens, s.head_dim, fill=fill)
    for r in range(batch.n_req):
        n = int(batch.kv_len[r]) - (batch.l_q(r) if upto_prefix else 0)
        c.append(batch.table(r), 0, tens.k[r][:n], tens.v[r][:n])
    return c


class Layer:
    def __init__(self, batch: W.MixedBatch, out_f32=True, decode_chunk=0, n_host_blocks=0, **kw):
        s = batch.shape
        self.shape = s
        self.M = batch.n_device_blocks
        self.out_f32 = out_f32
        self.ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, self.M, n_host_blocks, out_dtype=B.PS_F32 if out_f32 else B.PS_BF16,
                               decode_chunk=decode_chunk, **kw)
        self.ws = None
        self.ws_bytes = 0

    def close(self):
        B.ps_destroy(self.ctx)
        self.ctx = None

    def workspace(self, batch):
        need = B.ps_workspace_bytes(self.ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
        if need > self.ws_bytes:
            self.ws = torch.empty(need, dtype=torch.uint8, device=DEV)
            self.ws_bytes = need
        return self.ws

    def step(self, batch, q_dev, cache_dev, k_new=None, v_new=None, stream=None, wait_ticket=0):
        s = self.shape
        out = torch.full((batch.n_tokens, s.n_q_heads, s.head_dim), float("nan"),
                         dtype=torch.float32 if self.out_f32 else torch.bfloat16, device=DEV)
        ws = self.workspace(batch)
        B.ps_step(self.ctx, batch, q_dev, k_new, v_new, cache_dev, out, ws, self.ws_bytes, stream, wait_ticket)
        torch.cuda.synchronize()
        return out


def run_prefilled(batch, tens, **kw):
    """Cache already holds every token; returns (gpu_out float64 ndarray, layer)."""
    cache = oracle_cache(batch, tens)
    cache_dev = u16_to_dev(to_device_layout(cache.pool))
    lay = Layer(batch, **kw)
    out = lay.step(batch, u16_to_dev(tens.q), cache_dev)
    res = out.float().cpu().numpy().astype(np.float64)
    lay.close()
    return res, cache


def check_close(got: np.ndarray, want: np.ndarray, bf16_out: bool, tol=1e-2):
    assert np.isfinite(got).all(), "non-finite output"
    err = np.abs(got - want)
    bound = tol + (2.0 ** -8) * np.abs(want) if bf16_out else tol
    bad = err > bound
    assert not bad.any(), "max abs err %.4g at %s (want %.5g got %.5g)" % (
        err.max(), np.unravel_index(err.argmax(), err.shape), want.flat[err.argmax()], got.flat[err.argmax()])
    return float(err.max())
