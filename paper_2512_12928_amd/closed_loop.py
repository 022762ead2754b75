"""Driver of the closed loop of Sec. 4.3 ("Put it Together") over a multi-layer forward pass, as an engine would run
it: every round ps_form_batch orders the queue, sets the copy budget B_copy and the reload list; the blocks of the
list are reloaded layer by layer on a copy stream (ps_swap_in, one ticket per layer -- Appendix B's event per layer
chunk) while the attention layers run on the compute stream, each waiting only for its own layer's ticket; what the
budget left on the host is recomputed as prefill by the same batch; after the pass the round's offload list goes out
on a third stream and is reported to the scheduler once its tickets have completed (ps_sched_offloads_done).

Marshalling and stream order only: every decision is ps_form_batch's, every byte moved and every attention output is
the library's.  Used by tests/test_gpu_closed_loop.py (outputs of every layer against the oracle) and by bench.py
(the block-management arms of Sec. 5.3 side by side).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

import numpy as np

from . import binding as B

RELOAD_MODES = ("pipelined", "synchronous", "full_reload_first")


class ClosedLoop:
    def __init__(self, n_q_heads: int, n_kv_heads: int, n_device_blocks: int, n_host_blocks: int, n_layers: int,
                 sched_cfg: Dict, dev_free_order, host_free_order, rows: Callable, reload_mode: str = "pipelined",
                 out_dtype: int = B.PS_F32, device: str = "cuda:0"):
        """rows(rid, pos0, n, heads, what, layer) -> uint16 [n, heads, 128]: the q ("q"), k ("k") or v ("v") rows of
        request rid at positions pos0 .. pos0 + n - 1 in the given layer (a pure function, so that a recomputed token
        gets the rows it had the first time).  It may also return a bf16 tensor on the device (timing runs)."""
        import torch
        assert reload_mode in RELOAD_MODES
        self.torch, self.dev, self.L, self.mode, self.rows = torch, device, n_layers, reload_mode, rows
        self.Hq, self.Hkv, self.M, self.Mh = n_q_heads, n_kv_heads, n_device_blocks, n_host_blocks
        self.block_bytes = 2 * n_kv_heads * 16 * 128 * 2
        self.out_dtype = out_dtype
        self.sched = B.ps_sched_create(sched_cfg, np.asarray(dev_free_order, np.int32), np.asarray(host_free_order, np.int32))
        self.eta = int(sched_cfg["eta_ps"])
        self.ctx = B.ps_create(n_q_heads, n_kv_heads, n_device_blocks, n_host_blocks, out_dtype=out_dtype)
        self.caches = [torch.full((n_device_blocks, self.block_bytes // 2), float("nan"), dtype=torch.bfloat16, device=device)
                       for _ in range(n_layers)]
        self.hosts = [torch.zeros((n_host_blocks, self.block_bytes), dtype=torch.uint8).pin_memory() for _ in range(n_layers)]
        self.compute, self.side_in, self.side_out = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        self.ws_bytes = B.ps_workspace_bytes(self.ctx, 1024, 8192, n_device_blocks)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.offloads: List = []          # (round, [tickets of its layers]) still in flight, oldest first
        self.stats = dict(steps=0, evicted=0, blocks_reloaded=0, blocks_offloaded=0, tokens=0, prefill_tokens=0,
                          recomputed_tokens=0, pass_ms=0.0, dropped_in_flight=0)
        self.held: Dict[int, int] = {}    # rid -> tokens whose KV the engine has computed so far (to count recomputation)
        self.sched_cfg = dict(sched_cfg)
        self.last_pass_ms = 0.0
        self.token_times: Dict[int, List[int]] = {}   # rid -> delivery times of its tokens (ps on the run's clock), in order

    def close(self):
        for _, tks in self.offloads:
            for tk in tks:
                B.ps_ticket_wait(self.ctx, tk)
        self.torch.cuda.synchronize()
        B.ps_destroy(self.ctx)
        B.ps_sched_destroy(self.sched)

    def _up(self, parts):
        if isinstance(parts[0], self.torch.Tensor):
            return self.torch.cat(parts)
        return self.torch.from_numpy(np.ascontiguousarray(np.concatenate(parts)).view(np.int16)).to(self.dev)

    def _report_offloads(self):
        while self.offloads and all(B.ps_ticket_query(self.ctx, tk) == B.PS_OK for tk in self.offloads[0][1]):
            B.ps_sched_offloads_done(self.sched, self.offloads.pop(0)[0])

    def step(self, now_ps: int, on_layer: Optional[Callable] = None):
        """One scheduling round and its forward pass.  on_layer(layer, fb, out_tensor) is called after the pass for every
        layer.  Returns the round's ps_form_batch result (dict)."""
        torch = self.torch
        self._report_offloads()
        fb = B.ps_form_batch(self.sched, now_ps)
        st = self.stats
        st["steps"] += 1
        st["evicted"] += len(fb["evicted"])
        if fb["n_req"] == 0:
            return fb
        n_tok = int(fb["n_tokens"])
        st["tokens"] += n_tok
        ids = fb["req_ids"].tolist()
        lq = np.diff(fb["q_start"]).tolist()
        kv = fb["kv_len"].tolist()
        for rid, c, L in zip(ids, lq, kv):
            if c > 1:
                st["prefill_tokens"] += c
            st["recomputed_tokens"] += max(0, min(self.held.get(rid, 0), L) - (L - c))
            self.held[rid] = max(self.held.get(rid, 0), L)
        # this pass's rows, layer by layer (host work, outside the timed pass)
        q_l, k_l, v_l = [], [], []
        for ell in range(self.L):
            q_l.append(self._up([self.rows(r, L - c, c, self.Hq, "q", ell) for r, c, L in zip(ids, lq, kv)]))
            k_l.append(self._up([self.rows(r, L - c, c, self.Hkv, "k", ell) for r, c, L in zip(ids, lq, kv)]))
            v_l.append(self._up([self.rows(r, L - c, c, self.Hkv, "v", ell) for r, c, L in zip(ids, lq, kv)]))
        out_t = torch.float32 if self.out_dtype == B.PS_F32 else torch.bfloat16
        outs = [torch.empty((n_tok, self.Hq, 128), dtype=out_t, device=self.dev) for _ in range(self.L)]
        batch = B.make_batch(fb["q_start"], fb["kv_len"], fb["bt_start"], fb["block_ids"], fb["prio"])
        slots, blocks, budget = fb["swap_in_host_slots"], fb["swap_in_dev_blocks"], int(fb["copy_budget"])
        assert len(blocks) <= budget or len(blocks) == 0
        st["blocks_reloaded"] += len(blocks) * self.L

        def reload(ell):
            n, tk = B.ps_swap_in(self.ctx, slots, blocks, budget, self.hosts[ell], self.caches[ell], self.side_in)
            assert n == len(blocks)
            return tk

        def layer(ell, tk):
            if ell == 0:
                B.ps_step(self.ctx, batch, q_l[0], k_l[0], v_l[0], self.caches[0], outs[0], self.ws, self.ws_bytes, self.compute, tk)
            else:
                B.ps_step_next_layer(self.ctx, q_l[ell], k_l[ell], v_l[ell], self.caches[ell], outs[ell], self.ws, self.ws_bytes,
                                     self.compute, tk)

        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(self.compute)
        if self.mode == "synchronous":        # reload a layer, wait for it, compute it
            for ell in range(self.L):
                tk = reload(ell)
                if tk:
                    B.ps_ticket_wait(self.ctx, tk)
                layer(ell, 0)
        elif self.mode == "full_reload_first":  # everything over the link, then the pass
            tks = [reload(ell) for ell in range(self.L)]
            if tks[-1]:
                B.ps_ticket_wait(self.ctx, tks[-1])
            for ell in range(self.L):
                layer(ell, 0)
        else:                                  # layer l + 1 loads while layer l computes; each layer waits for its own ticket
            tk = reload(0)
            for ell in range(self.L):
                nxt = reload(ell + 1) if ell + 1 < self.L else 0
                layer(ell, tk)
                tk = nxt
        e1.record(self.compute)
        self.compute.synchronize()
        # the pass as an engine sees it: from the first reload's issue to the last layer's end (host waits included)
        self.last_pass_ms = e0.elapsed_time(e1)
        st["pass_ms"] += self.last_pass_ms
        if on_layer is not None:
            for ell in range(self.L):
                on_layer(ell, fb, outs[ell])
        # asynchronous offload of the round's newly completed blocks, every layer, outside the forward path
        if len(fb["swap_out_dev_blocks"]):
            tks = []
            for ell in range(self.L):
                n, tk = B.ps_swap_out(self.ctx, fb["swap_out_dev_blocks"], fb["swap_out_host_slots"], -1, self.caches[ell],
                                      self.hosts[ell], self.side_out)
                tks.append(tk)
            self.offloads.append((int(fb["round"]), tks))
            st["blocks_offloaded"] += len(fb["swap_out_dev_blocks"]) * self.L
        return fb

    def run(self, trace, max_steps: int, on_layer: Optional[Callable] = None, clock: str = "estimator") -> Dict:
        """clock "estimator": the virtual clock of ps_sched_simulate, which advances by T_pd(B) of every round;
        "measured": it advances by the GPU time the round's forward pass took (from the first reload's issue to the last
        layer's end), so that the batch former sees the time an engine would.  Tokens are delivered when their pass
        ends; score() applies Eq. 3 to the delivery times."""
        assert clock in ("estimator", "measured")
        pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
        nxt = now = 0
        while self.stats["steps"] < max_steps:
            while nxt < len(pending) and pending[nxt].arrival_ps <= now:
                p = pending[nxt]
                B.ps_sched_add_request(self.sched, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
                nxt += 1
            if B.ps_sched_counts(self.sched)[0] == 0:
                if nxt >= len(pending):
                    break
                now = pending[nxt].arrival_ps
                continue
            fb = self.step(now, on_layer)
            if fb["n_req"] == 0:
                now += self.eta
                continue
            now += int(self.last_pass_ms * 1e9) if clock == "measured" else int(fb["t_batch"])
            for rid in fb["emitted_req"].tolist():
                self.token_times.setdefault(int(rid), []).append(now)
        return dict(self.stats)

    def score(self, trace) -> Dict:
        """Eq. 3 over the requests that finished in run(): token-level deadline-aware gain against the gain with every
        token on time, and SLO attainment (ps_tdg_score does the arithmetic)."""
        gain = ideal = ok = done = 0
        for p in trace:
            tt = self.token_times.get(p.rid, [])
            if len(tt) < p.out_len:
                continue
            g, i, a = B.ps_tdg_score(self.sched_cfg, p.prio, p.out_len, np.asarray(tt, np.int64) - p.arrival_ps)
            gain, ideal, ok, done = gain + g, ideal + i, ok + a, done + 1
        return dict(finished=done, tdg_ratio=gain / ideal if ideal else 0.0, slo_attainment=ok / done if done else 0.0)
