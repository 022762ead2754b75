#!/usr/bin/env python3
"""Benchmark of the engine-step hot path on one MI355X.

A step is one pass of the hot path over one synthetic mixed batch (ps_step): host batch
description -> device and KV append (one launch), split-K decode attention and prefill-chunk
attention side by side (one launch), merge of the split-K partials (one launch).  The
headline workload is the largest single-GPU configuration, the Llama-70B-shaped layer (64 query / 8 KV
heads; 512 decode requests + 8192 prefill tokens in 4 chunks); the Qwen3-8B-shaped and the long-context
workloads are reported under "extra", each with its own roofline object.  Prints ONE JSON line: metric, value, unit, timing fields, a roofline object for the attention launch and
the oracle's speed on the same batch as cpu_baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the attention kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in runs of
# their own (scaled by a plain 1 GiB copy; summary in profiles/attention_kernel_hbm_traffic_pmc.md), by kernel and
# workload index.  Not measured in this run: counters need the profiler.
MEASURED_ATTENTION_TRAFFIC = {("attention_kernel", 2): 1.607e9, ("attention_kernel", 4): 3.382e9,
                              ("attention_kernel", 5): 4.690e9, ("fused_kernel", 4): 3.258e9, ("fused_kernel", 5): 4.598e9}
TRAFFIC_SOURCE = "profiles/attention_kernel_hbm_traffic_pmc.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; runs of their own)"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
NOMINAL_MHZ = 2400.0           # the shader clock the published matrix peak is quoted at


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=5, help="workload index 1..5 (5 = headline)")
    ap.add_argument("--decode-chunk", type=int, default=0)
    ap.add_argument("--mixed-launch", type=int, default=0,
                    help="cfg.mixed_launch: 0 the library picks, 1 decode and prefill work on disjoint compute units, "
                         "2 every workgroup carries both")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads / swap figures")
    ap.add_argument("--swap-only", action="store_true",
                    help="only the workload-3 swap figures (block copies next to attention steps), as one JSON object: "
                         "the command the swap kernel's profile in profiles/ is taken with")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (a known amount of HBM traffic) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2512_12928_amd import binding as B
    from paper_2512_12928_amd import workloads as W
    from paper_2512_12928_amd.kvlayout import request_kv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def device_inputs(batch, seed):
        return W.device_inputs(batch, seed, dev)

    def algorithmic(batch):
        """Bytes the attention launch has to move at least (decode: every cached K/V byte once, q, out,
        table; prefill: the K/V of every chunk's context once, q, out, table) and the prefill FLOPs."""
        s = batch.shape
        tok_bytes = s.n_kv_heads * s.head_dim * 2 * 2
        row_bytes = 2 * s.n_q_heads * s.head_dim * 2          # one q row in, one out row out

        def part(reqs):
            kv = int(batch.kv_len[reqs].astype(np.int64).sum()) * tok_bytes
            rows = int(sum(batch.l_q(int(r)) for r in reqs)) * row_bytes
            tab = int(sum(4 * -(-int(batch.kv_len[r]) // s.block_tokens) for r in reqs))
            return kv + rows + tab
        flops = 4 * s.head_dim * s.n_q_heads * batch.causal_pairs()
        return part(batch.decode_reqs), part(batch.prefill_reqs), flops

    def run(batch, steps, warmup, decode_chunk=0, profile_steps=20):
        s = batch.shape
        pool, q, kn, vn = device_inputs(batch, batch.seed)
        ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, 0, out_dtype=B.PS_BF16,
                          decode_chunk=decode_chunk, mixed_launch=args.mixed_launch)
        nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        out = torch.empty((batch.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
        cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
        stream = torch.cuda.current_stream()
        for _ in range(warmup):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # a forward pass plans and uploads the batch once: ps_step on the first layer, ps_step_next_layer on
        # the other 35 (here every "layer" works on the same tensors); reported beside the headline figure,
        # which rebuilds the batch description on every step
        n_layers = 36
        passes = max(1, steps // n_layers)
        t0 = time.perf_counter()
        for _ in range(passes):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
            for _ in range(n_layers - 1):
                B.ps_step_next_layer(ctx, q, kn, vn, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        dt_pass = (time.perf_counter() - t0) / (passes * n_layers)
        host_us = {}
        for name in ("ps_step", "ps_step_next_layer"):   # host time of a call (enqueue only), queue empty at the start;
            t0 = time.perf_counter()                     # three calls: the fifth ps_step in flight would wait for a staging slot
            for _ in range(3):
                if name == "ps_step":
                    B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
                else:
                    B.ps_step_next_layer(ctx, q, kn, vn, pool, out, ws, nbytes, stream)
            host_us[name] = (time.perf_counter() - t0) / 3 * 1e6
            torch.cuda.synchronize()
        # per-launch durations: HIP events recorded by the library on the launch stream, one set per step, read once
        # after the last step.  Mode 1: the timed region again, the same `steps` calls back to back, with the events
        # on (the library averages over the last 64 steps; the region's own ms_per_step is reported beside the
        # headline one).  Mode 2: the decode and the prefill work in launches of their own, `profile_steps` steps
        # back to back.
        phases = {}
        B.ps_set_profiling(ctx, 1)
        for _ in range(warmup):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        if warmup > 0:
            B.ps_get_step_times(ctx)                      # the warm-up steps are not part of the mean
        t0 = time.perf_counter()
        for _ in range(steps):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        dt_events = time.perf_counter() - t0
        phases[1] = B.ps_get_step_times(ctx)
        B.ps_set_profiling(ctx, 2)
        for _ in range(profile_steps):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        phases[2] = B.ps_get_step_times(ctx)
        B.ps_set_profiling(ctx, 0)
        res = dict(ms_per_step=dt / steps * 1e3, ms_per_step_with_events=dt_events / steps * 1e3, phases_ms=phases, ctx=ctx,
                   pool=pool, q=q, out=out, kn=kn, vn=vn, ms_per_layer_plan_reused=dt_pass * 1e3, host_us_per_call=host_us)
        return res

    def rooflines(batch, res):
        bytes_dec, bytes_pre, flops_pre = algorithmic(batch)
        run_, alone = res["phases_ms"][1], res["phases_ms"][2]
        att_s = run_["attention_ms"] * 1e-3
        dec_s, pre_s = alone["decode_ms"] * 1e-3, alone["prefill_ms"] * 1e-3
        att_gbs = (bytes_dec + bytes_pre) / att_s / 1e9 if att_s > 0 else 0.0
        att_tf = flops_pre / att_s / 1e12 if att_s > 0 else 0.0
        dec_gbs = bytes_dec / dec_s / 1e9 if dec_s > 0 else 0.0
        pre_tf = flops_pre / pre_s / 1e12 if pre_s > 0 else 0.0
        sh = batch.shape
        plan = B.ps_plan_launch(sh.n_q_heads, sh.n_kv_heads, batch.n_device_blocks, batch, mixed_launch=args.mixed_launch,
                                decode_chunk=args.decode_chunk)
        both = plan["decode_slots"] > 0 and plan["prefill_workgroups"] > 0
        return dict(kernel="fused_kernel" if both and plan["decode_workgroups"] == 0 else "attention_kernel",
                    attention_ms=run_["attention_ms"], ms_per_step_with_events=res["ms_per_step_with_events"],
                    attention_GBps=att_gbs, attention_hbm_frac=att_gbs / HBM_PEAK_GBS,
                    attention_TFLOPs=att_tf, attention_mfma_frac=att_tf / MFMA_BF16_PEAK_TFLOPS,
                    attention_bytes=bytes_dec + bytes_pre, prefill_flops=flops_pre,
                    append_ms=run_["append_ms"], merge_ms=run_["merge_ms"],
                    # the two kinds of work in launches of their own, each with the whole chip
                    decode_alone_ms=alone["decode_ms"], decode_alone_GBps=dec_gbs, decode_alone_frac=dec_gbs / HBM_PEAK_GBS,
                    prefill_alone_ms=alone["prefill_ms"], prefill_alone_TFLOPs=pre_tf,
                    prefill_alone_frac=pre_tf / MFMA_BF16_PEAK_TFLOPS,
                    # the shader clock the workgroups of each kind ran at (their own clock counters, read in the kernel):
                    # the published peaks are for 2400 MHz, the chip lowers the clock under load
                    shader_mhz=dict(mixed_decode=run_["decode_mhz"], mixed_prefill=run_["prefill_mhz"],
                                    decode_alone=alone["decode_mhz"], prefill_alone=alone["prefill_mhz"]),
                    prefill_alone_frac_of_peak_at_its_clock=(pre_tf / (MFMA_BF16_PEAK_TFLOPS * alone["prefill_mhz"] / NOMINAL_MHZ)
                                                             if alone["prefill_mhz"] > 0 else None))

    if args.swap_only:
        print(json.dumps({"swap": swap_bench(B, W, torch, np, dev)}))
        return 0

    if args.pmc_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    batch = W.make_workload(args.workload)
    res = run(batch, args.steps, args.warmup, args.decode_chunk)
    rl = rooflines(batch, res)
    rl["ms_per_layer_plan_reused"] = res["ms_per_layer_plan_reused"]
    rl["host_us_per_call"] = res["host_us_per_call"]
    tokens_per_s = batch.n_tokens / (res["ms_per_step"] * 1e-3)

    # ---- CPU baseline: the fp64 oracle, as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import attention as A
        from threadpoolctl import threadpool_info          # missing => fail loudly rather than report a guess
        pools = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        assert pools, "no BLAS thread pool found: cannot say how many cores the numpy oracle uses"
        cores = max(pools)
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                for ln in f:
                    if ln.startswith("model name"):
                        cpu_model = ln.split(":", 1)[1].strip()
                        break
        except OSError:
            pass
        s = batch.shape
        torch.cuda.synchronize()
        # sample: requests until about 32 M (query, key) pair-heads x Hq (10-30 s of fp64 numpy), decode
        # requests and prefill rows in the batch's own proportion of pairs
        budget = int(2.0e9 / s.n_q_heads)
        q_host = res["q"].view(torch.int16).cpu().numpy().view(np.uint16)
        pairs = 0
        t_cpu = 0.0
        n_dec = n_rows = 0
        total_pairs = batch.decode_kv_tokens() + batch.causal_pairs()
        frac = min(1.0, budget / total_pairs)
        order = []                                  # (request, rows): every chunk's leading rows, then decode requests
        for r in [int(x) for x in batch.prefill_reqs]:
            lq_r, p_r = batch.l_q(r), int(batch.kv_len[r]) - batch.l_q(r)
            rows_r = lq_r
            while rows_r > 1 and rows_r * p_r + rows_r * (rows_r + 1) // 2 > frac * (lq_r * p_r + lq_r * (lq_r + 1) // 2):
                rows_r -= max(1, rows_r // 16)
            order.append((r, rows_r))
        dec_budget = frac * batch.decode_kv_tokens()
        for r in [int(x) for x in batch.decode_reqs]:
            if dec_budget <= 0:
                break
            order.append((r, 1))
            dec_budget -= int(batch.kv_len[r])
        for r, rows in order:
            L, lq = int(batch.kv_len[r]), batch.l_q(r)
            p = L - lq
            tab = torch.from_numpy(batch.table(r).astype(np.int64)).to(dev)
            blocks = res["pool"][tab].view(torch.int16).cpu().numpy().view(np.uint16)
            k_bits, v_bits = request_kv(blocks, s.n_kv_heads, L)
            a = int(batch.q_start[r])
            # this step's own rows come from the inputs, not from what the append kernel wrote
            k_bits[p:] = res["kn"][a:a + lq].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            v_bits[p:] = res["vn"][a:a + lq].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            t1 = time.perf_counter()
            qf = A.bf16_to_f64(q_host[a:a + rows])
            kf, vf = A.bf16_to_f64(k_bits[:p + rows]), A.bf16_to_f64(v_bits[:p + rows])
            ref = A.dense_attention(qf, kf, vf)
            t_cpu += time.perf_counter() - t1
            pairs += rows * p + rows * (rows + 1) // 2
            n_dec += lq == 1
            n_rows += rows if lq > 1 else 0
            got = res["out"][a:a + rows].float().cpu().numpy().astype(np.float64)
            err = np.abs(got - ref)
            assert (err <= 1e-2 + 2.0 ** -8 * np.abs(ref)).all(), "bench sample disagrees with the oracle"
        est_step_s = t_cpu * total_pairs / max(pairs, 1)
        cpu = dict(value=batch.n_tokens / est_step_s, unit="tokens/s", cores=int(cores), kind="oracle",
                   cpu_model=cpu_model, nproc=os.cpu_count(), seconds=t_cpu,
                   sample="%d decode requests + %d prefill rows of %s (%.0f%% of its (query,key) pairs): %.1f s of "
                          "numpy fp64, every sampled output checked against the GPU's; scaled to the whole batch by pair "
                          "count" % (n_dec, n_rows, batch.name, 100.0 * pairs / (batch.decode_kv_tokens() + batch.causal_pairs()), t_cpu))

    extra = {}
    if not args.no_extra:
        extra["workload_%d" % args.workload] = rl
        B.ps_destroy(res.pop("ctx"))
        for k in ("pool", "q", "out", "kn", "vn"):
            res.pop(k, None)
        torch.cuda.empty_cache()
        for idx in (2, 4, 5):
            if idx == args.workload:
                continue
            bb = W.make_workload(idx)
            rr = run(bb, 20, 5, args.decode_chunk, profile_steps=10)
            e = rooflines(bb, rr)
            e["ms_per_step"] = rr["ms_per_step"]
            e["ms_per_layer_plan_reused"] = rr["ms_per_layer_plan_reused"]
            e["host_us_per_call"] = rr["host_us_per_call"]
            e["tokens_per_s"] = bb.n_tokens / (rr["ms_per_step"] * 1e-3)
            extra["workload_%d" % idx] = e
            B.ps_destroy(rr.pop("ctx"))
            del rr
            torch.cuda.empty_cache()
        extra["mixed_launch_layouts"] = layout_bench(B, W, torch, dev)
        extra["clock_under_load"] = clock_bench(B, W, torch, dev, args.workload)
        extra["swap"] = swap_bench(B, W, torch, np, dev)
        extra["reload_pipeline"] = reload_pipeline_bench(B, W, torch, np, dev)
        extra["closed_loop"] = closed_loop_bench(B, W, torch, np, dev, extra["swap"])
        extra["launch_bound_pass"] = graph_bench(B, W, torch, np, dev)
        extra["sched"] = sched_bench(B, W, np, extra["workload_2"]["ms_per_step"] if "ms_per_step" in extra.get("workload_2", {}) else res["ms_per_step"])

    roof = roof_of(rl, args.workload)
    for k, e in extra.items():
        if k.startswith("workload_") and k != "workload_%d" % args.workload:
            e["roofline"] = roof_of(e, int(k.split("_")[1]))
    line = {
        "metric": "mixed-batch paged-attn tokens/s per layer", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": batch.name, "n_decode": int(len(batch.decode_reqs)),
                   "n_prefill_tokens": int(batch.n_tokens - len(batch.decode_reqs)),
                   "decode_kv_tokens": batch.decode_kv_tokens(), "heads": "%dq/%dkv" % (batch.shape.n_q_heads, batch.shape.n_kv_heads)},
        "roofline": roof, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line))
    return 0


def roof_of(rl, workload):
    """The roofline object of the dominant kernel, the one attention launch of the mixed batch.  It does two kinds of
    work at once; the roof that binds it is the one that gives the later earliest end: all algorithmic bytes at the
    HBM peak, or all prefill FLOPs at the bf16 MFMA peak."""
    t_hbm = rl["attention_bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = rl["prefill_flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    how = dict(launch_us=rl["attention_ms"] * 1e3,
               launch_us_from="HIP events of the library on the launch stream around every launch of the timed steps run again "
                              "back to back with those events on (mean over the last 64 launches; ms_per_step of that region: "
                              "%.4f)" % rl["ms_per_step_with_events"])
    if t_hbm >= t_mfma:
        return dict(bound="hbm", kernel=rl["kernel"], achieved=rl["attention_GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=rl["attention_hbm_frac"], **how, traffic=MEASURED_ATTENTION_TRAFFIC.get((rl["kernel"], workload)),
                    traffic_source=TRAFFIC_SOURCE if (rl["kernel"], workload) in MEASURED_ATTENTION_TRAFFIC else None,
                    shader_mhz=rl["shader_mhz"],
                    other_roof=dict(bound="mfma", achieved=rl["attention_TFLOPs"], peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                                    frac=rl["attention_mfma_frac"]))
    return dict(bound="mfma", kernel=rl["kernel"], achieved=rl["attention_TFLOPs"], peak=MFMA_BF16_PEAK_TFLOPS,
                unit="TFLOP/s", frac=rl["attention_mfma_frac"], **how, traffic=MEASURED_ATTENTION_TRAFFIC.get((rl["kernel"], workload)),
                traffic_source=TRAFFIC_SOURCE if (rl["kernel"], workload) in MEASURED_ATTENTION_TRAFFIC else None,
                shader_mhz=rl["shader_mhz"],
                other_roof=dict(bound="hbm", achieved=rl["attention_GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                                frac=rl["attention_hbm_frac"]))


def layout_bench(B, W, torch, dev):
    """The attention launch of workloads 4 and 5 in both layouts, interleaved on one box: decode and prefill work on
    disjoint compute units (cfg.mixed_launch = 1) against workgroups that carry both (2); GPU time of the launch from
    the library's events, median of 5 rounds of 10 steps, and which of the two the library picks by itself."""
    out = {}
    for idx in (4, 5):
        batch = W.make_workload(idx)
        s = batch.shape
        pool, q, kn, vn = W.device_inputs(batch, batch.seed, dev)
        o = torch.empty((batch.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
        cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
        stream = torch.cuda.current_stream()
        ctxs, ws = {}, {}
        for mode in (1, 2):
            ctxs[mode] = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, 0, mixed_launch=mode)
            n = B.ps_workspace_bytes(ctxs[mode], batch.n_req, batch.n_tokens, len(batch.block_ids))
            ws[mode] = torch.empty(n, dtype=torch.uint8, device=dev)
            B.ps_set_profiling(ctxs[mode], 1)
            for _ in range(3):
                B.ps_step(ctxs[mode], cb, q, kn, vn, pool, o, ws[mode], ws[mode].numel(), stream)
        times = {1: [], 2: []}
        for _ in range(5):
            for mode in (1, 2):
                acc = 0.0
                for _ in range(10):
                    B.ps_step(ctxs[mode], cb, q, kn, vn, pool, o, ws[mode], ws[mode].numel(), stream)
                    acc += B.ps_get_step_times(ctxs[mode])["attention_ms"] / 10
                times[mode].append(acc)
        for mode in (1, 2):
            B.ps_destroy(ctxs[mode])
        picked = B.ps_plan_launch(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, batch)["decode_workgroups"] == 0
        out["workload_%d" % idx] = dict(attention_ms_disjoint_units=sorted(times[1])[2], attention_ms_both_in_every_workgroup=sorted(times[2])[2],
                                        library_picks="both_in_every_workgroup" if picked else "disjoint_units")
        del pool, q, kn, vn, o, ws
        torch.cuda.empty_cache()
    out["faults"] = B.ps_mixed_launch_faults()
    return out


def clock_bench(B, W, torch, dev, workload):
    """The same prefill launch (launched alone, profiling mode 2) on the workload's N(0,1) tensors and on all-zero
    tensors: same instructions, same addresses, other operand bits.  The time and the shader clock of both, as the
    kernel's own clock counters give it: the difference is the chip's power management, not the kernel's schedule."""
    batch = W.make_workload(workload)
    s = batch.shape
    pool, q, kn, vn = W.device_inputs(batch, batch.seed, dev)
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, 0)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    out = torch.empty((batch.n_tokens, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
    cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
    stream = torch.cuda.current_stream()
    flops = 4 * s.head_dim * s.n_q_heads * batch.causal_pairs()
    res = {}
    B.ps_set_profiling(ctx, 2)
    for name in ("normal_inputs", "zero_inputs"):
        if name == "zero_inputs":
            for t in (pool, q, kn, vn):
                t.zero_()
        for _ in range(3):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
        acc, n = {}, 10
        for _ in range(n):
            B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, stream)
            for k, v in B.ps_get_step_times(ctx).items():
                acc[k] = acc.get(k, 0.0) + v / n
        tf = flops / (acc["prefill_ms"] * 1e-3) / 1e12 if acc["prefill_ms"] > 0 else 0.0
        res[name] = dict(prefill_alone_ms=acc["prefill_ms"], prefill_mhz=acc["prefill_mhz"], prefill_TFLOPs=tf,
                         frac_of_peak=tf / MFMA_BF16_PEAK_TFLOPS, decode_alone_ms=acc["decode_ms"], decode_mhz=acc["decode_mhz"])
    B.ps_destroy(ctx)
    return res


def swap_bench(B, W, torch, np, dev):
    """Workload 3: per engine step, 512 blocks out and 512 in (32 MiB each way) on side streams, issued
    step by step next to the attention step as an engine would.  Reported against the host link as
    measured on this machine with large pinned copies (one direction, and both directions at once)."""
    import time as _t
    batch = W.make_workload(3)
    s = batch.shape
    Mh = 4096
    bb = s.block_bytes
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    pool = torch.empty((batch.n_device_blocks, bb // 2), dtype=torch.bfloat16, device=dev).normal_(generator=g)
    host = torch.empty((Mh, bb), dtype=torch.uint8).pin_memory()
    host.zero_()
    compute, side_out, side_in = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    res = {}
    # ---- measured host link: 256 MiB pinned copies, one way and both ways at once
    nbig = 1 << 28
    d1 = torch.empty(nbig, dtype=torch.uint8, device=dev)
    d2 = torch.empty(nbig, dtype=torch.uint8, device=dev)
    h1 = torch.empty(nbig, dtype=torch.uint8).pin_memory()
    h2 = torch.empty(nbig, dtype=torch.uint8).pin_memory()

    def link(do_out, do_in, reps=6, own_streams=True, nbytes=nbig):
        a1, a2, b1, b2 = h1[:nbytes], d1[:nbytes], d2[:nbytes], h2[:nbytes]
        torch.cuda.synchronize()
        t0 = _t.perf_counter()
        for _ in range(reps):
            if do_out:
                with torch.cuda.stream(side_out if own_streams else torch.cuda.current_stream()):
                    a1.copy_(a2, non_blocking=True)
            if do_in:
                with torch.cuda.stream(side_in if own_streams else torch.cuda.current_stream()):
                    b1.copy_(b2, non_blocking=True)
        torch.cuda.synchronize()
        return reps * nbytes / (_t.perf_counter() - t0) / 1e9

    link(True, True, 1)
    link(True, True, 1, False)
    # one direction at a time: best of the default stream and a side stream (they can land on
    # different copy engines); both directions at once: one stream each
    res["link_d2h_GBps"] = max(link(True, False), link(True, False, own_streams=False))
    res["link_h2d_GBps"] = max(link(False, True), link(False, True, own_streams=False))
    res["link_bidir_each_way_GBps"] = max(link(True, True) for _ in range(3))     # the best of three: this figure wanders from run to run
    # the same with copies of the size a step moves (32 MiB each way per copy): what the copy engines reach at that grain
    res["link_bidir_each_way_GBps_32MiB_copies"] = max(link(True, True, reps=48, nbytes=1 << 25) for _ in range(3))
    del d1, d2, h1, h2
    torch.cuda.empty_cache()

    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, Mh, swap_dma_runs=64)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    q = torch.randn((batch.n_tokens, s.n_q_heads, s.head_dim), generator=g, device=dev).to(torch.bfloat16)
    kn = torch.randn((batch.n_tokens, s.n_kv_heads, s.head_dim), generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
    step_bytes = 512 * bb

    def measure(host_run):
        """host_run 1: host slots scattered one by one (moved by a copy kernel that addresses host memory itself);
        32: host slots in 16 runs of 32 consecutive slots (moved by the copy engines, one DMA per run, through the
        context's staging buffers)."""
        rng = np.random.default_rng(33)
        used = batch.block_ids
        out_ids, out_slots = W.make_swap_lists(512, batch.n_device_blocks, Mh // 2, rng, exclude_device=used, host_run=host_run)
        free = np.setdiff1d(np.arange(batch.n_device_blocks, dtype=np.int32), np.concatenate([used, out_ids]))
        in_ids = rng.permutation(free)[:512].astype(np.int32)
        _, in_slots = W.make_swap_lists(512, batch.n_device_blocks, Mh // 2, rng, host_run=host_run)
        in_slots = (in_slots + Mh // 2).astype(np.int32)          # the other half of the host pool

        def run(n, do_attn, do_out, do_in):
            torch.cuda.synchronize()
            t0 = _t.perf_counter()
            for _ in range(n):
                if do_out:
                    B.ps_swap_out(ctx, out_ids, out_slots, -1, pool, host, side_out)
                if do_in:
                    B.ps_swap_in(ctx, in_slots, in_ids, -1, host, pool, side_in)
                if do_attn:
                    B.ps_step(ctx, cb, q, kn, kn, pool, out, ws, nbytes, compute)
            torch.cuda.synchronize()
            return (_t.perf_counter() - t0) / n

        run(5, True, True, True)
        n = 40

        def med(*mode):          # median of three runs of n steps
            return sorted(run(n, *mode) for _ in range(3))[1]

        r = {}
        t = med(True, False, False)
        r["attn_ms_swaps_off"] = t * 1e3
        r["swap_out_only_GBps"] = step_bytes / med(False, True, False) / 1e9
        r["swap_in_only_GBps"] = step_bytes / med(False, False, True) / 1e9
        r["swap_both_each_way_GBps"] = step_bytes / med(False, True, True) / 1e9
        t = med(True, True, True)
        r["overlap_both_each_way_GBps"] = step_bytes / t / 1e9
        r["overlap_both_step_ms"] = t * 1e3
        t = med(True, True, False)
        r["overlap_out_GBps"] = step_bytes / t / 1e9
        r["overlap_out_step_ms"] = t * 1e3
        t = med(True, False, True)
        r["overlap_in_GBps"] = step_bytes / t / 1e9
        r["overlap_in_step_ms"] = t * 1e3
        r["overlap_both_frac_of_bidir_link"] = r["overlap_both_each_way_GBps"] / res["link_bidir_each_way_GBps"]
        r["overlap_both_frac_of_bidir_link_32MiB_copies"] = r["overlap_both_each_way_GBps"] / res["link_bidir_each_way_GBps_32MiB_copies"]
        r["overlap_out_frac_of_link"] = r["overlap_out_GBps"] / res["link_d2h_GBps"]
        r["overlap_in_frac_of_link"] = r["overlap_in_GBps"] / res["link_h2d_GBps"]
        # what the link alone needs for this step's bytes: the floor of a step that swaps 32 MiB each way
        r["link_ms_for_both"] = step_bytes / (res["link_bidir_each_way_GBps"] * 1e9) * 1e3
        return r

    res.update(measure(1))
    res["host_slots_in_runs_of_32_by_copy_engines"] = measure(32)       # cfg.swap_dma_runs = 64 on this context
    B.ps_destroy(ctx)
    return res


def reload_pipeline_bench(B, W, torch, np, dev, n_layers=8):
    """Pipelined reload across layers (Sec. 4.3, Appendix B) on workload 3: the blocks of the batch's longest
    requests (512 blocks, 32 MiB per layer) are in pinned host memory when the forward pass over n_layers
    attention layers starts.  Three ways to run the pass: reload layer by layer and wait (synchronous), reload
    everything, then compute (full reload first), and the paper's pipeline: layer i+1's blocks are copied on a
    side stream while layer i computes, each layer waiting only for its own ticket; the last also under a copy
    budget sized so that a layer's copy takes no longer than its attention."""
    import time as _t
    batch = W.make_workload(3)
    s = batch.shape
    bb = s.block_bytes
    order = np.argsort(-batch.kv_len[batch.decode_reqs])
    ids = []
    for r in batch.decode_reqs[order]:
        ids.extend(batch.table(int(r)).tolist())
        if len(ids) >= 512:
            break
    dev_ids = np.array(ids[:512], dtype=np.int32)
    slots = np.random.default_rng(5).permutation(512).astype(np.int32)
    g = torch.Generator(device=dev)
    g.manual_seed(35)
    pools = [torch.empty((batch.n_device_blocks, bb // 2), dtype=torch.bfloat16, device=dev).normal_(generator=g)
             for _ in range(n_layers)]
    hosts = []
    for ell in range(n_layers):
        h = torch.empty((512, bb), dtype=torch.uint8).pin_memory()
        h.copy_(pools[ell].view(torch.uint8).view(batch.n_device_blocks, bb)[torch.from_numpy(dev_ids.astype(np.int64)).to(dev)][
            torch.from_numpy(np.argsort(slots).astype(np.int64)).to(dev)].cpu())
        hosts.append(h)
    q = torch.randn((batch.n_tokens, s.n_q_heads, s.head_dim), generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    ctx = B.ps_create(s.n_q_heads, s.n_kv_heads, batch.n_device_blocks, 512)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
    compute, side = torch.cuda.Stream(), torch.cuda.Stream()

    def layer(ell, tk=0):   # the pass plans its batch once: ps_step on the first layer, the rest reuse it
        if ell == 0:
            B.ps_step(ctx, cb, q, None, None, pools[ell], out, ws, nbytes, compute, tk)
        else:
            B.ps_step_next_layer(ctx, q, None, None, pools[ell], out, ws, nbytes, compute, tk)

    def one_pass(mode, budget=-1):
        if mode == "compute_only":
            for ell in range(n_layers):
                layer(ell)
        elif mode == "synchronous":
            for ell in range(n_layers):
                _, tk = B.ps_swap_in(ctx, slots, dev_ids, budget, hosts[ell], pools[ell], side)
                B.ps_ticket_wait(ctx, tk)
                layer(ell)
        elif mode == "full_reload_first":
            tks = [B.ps_swap_in(ctx, slots, dev_ids, budget, hosts[ell], pools[ell], side)[1] for ell in range(n_layers)]
            B.ps_ticket_wait(ctx, tks[-1])
            for ell in range(n_layers):
                layer(ell)
        else:  # pipelined
            tk = B.ps_swap_in(ctx, slots, dev_ids, budget, hosts[0], pools[0], side)[1]
            for ell in range(n_layers):
                nxt = B.ps_swap_in(ctx, slots, dev_ids, budget, hosts[ell + 1], pools[ell + 1], side)[1] if ell + 1 < n_layers else 0
                layer(ell, tk)
                tk = nxt

    def timed(mode, budget=-1, reps=10):
        one_pass(mode, budget)
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            t0 = _t.perf_counter()
            for _ in range(reps):
                one_pass(mode, budget)
            torch.cuda.synchronize()
            ts.append((_t.perf_counter() - t0) / reps * 1e3)
        return sorted(ts)[1]

    res = dict(n_layers=n_layers, blocks_per_layer=512, MiB_per_layer=512 * bb / 2 ** 20)
    res["compute_only_ms"] = timed("compute_only")
    res["synchronous_ms"] = timed("synchronous")
    res["full_reload_first_ms"] = timed("full_reload_first")
    res["pipelined_ms"] = timed("pipelined")
    # copy budget B_copy such that one layer's copy fits under one layer's attention (measured rates)
    layer_ms = res["compute_only_ms"] / n_layers
    copy_ms_per_block = (res["full_reload_first_ms"] - res["compute_only_ms"]) / n_layers / 512
    fit = max(1, min(512, int(layer_ms / copy_ms_per_block)))
    res["budget_blocks_that_fit"] = fit
    res["pipelined_budgeted_ms"] = timed("pipelined", fit)
    res["pipelined_budgeted_overhead_vs_compute_only"] = res["pipelined_budgeted_ms"] / res["compute_only_ms"] - 1.0
    B.ps_destroy(ctx)
    return res


def closed_loop_bench(B, W, torch, np, dev, swap, n_layers=4, steps=300):
    """The closed loop of Sec. 4.3 over an n_layers forward pass, driven by ps_form_batch on a trace that keeps the device
    pool under pressure (evictions, reloads): the scheduler's t_block is the block's bytes over the link rate measured in
    this run, its estimator constants the fit of profiles/estimator_fit_mi355x.md, both times n_layers.  Arms, side by
    side (Sec. 5.3, block-management ablation): the copy budget as ps_form_batch sets it with the reload pipelined layer
    by layer; the same with everything reloaded whatever it costs (t_block tiny), pipelined, layer-synchronous, and all
    up front; and no host copies at all (evicted requests are recomputed).  pass_ms is GPU time of the forward passes
    (from the first reload's issue to the last layer's end), summed over the rounds.  The run's clock is the measured one:
    every round advances it by the GPU time its pass took, and the tokens' delivery times on that clock are scored with
    Eq. 3 (SLOs scaled to this 4-layer attention-only pass: first token 20 ms, 0.5 ms per later token)."""
    from paper_2512_12928_amd.closed_loop import ClosedLoop
    Hq, Hkv, M, Mh = 32, 8, 1200, 3000
    bb = 2 * Hkv * 16 * 128 * 2
    L = n_layers
    MS, US = 10 ** 9, 10 ** 6
    link = min(swap["link_h2d_GBps"], swap["link_d2h_GBps"])
    t_block = int(bb / (link * 1e9) * 1e12) * L
    base = dict(n_classes=3, block_tokens=16, class_weight=[4, 2, 1], w_first=4, w_decode=1, ttft_slo_ps=20 * MS,
                tpot_slo_ps=MS // 2, a_p=3 * L, b_p=19 * L, c_p=5682 * L, a_d=554 * L, b_d=15784 * L, t_c=28 * US * L,
                eta_ps=2 * MS, tau_ps=30_000 * MS, gamma_num=9, gamma_den=10, beta_num=2, beta_den=1, rho_num=9, rho_den=10,
                t_block_ps=t_block, n_off_base=8)
    trace = W.make_trace(3, 400, rate_per_s=4000.0, seed=21, prompt_mean=700, prompt_max=3000, out_mean=24, out_max=96)
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    bank = {h: torch.randn((4096, h, 128), generator=g, device=dev).to(torch.bfloat16) for h in (Hq, Hkv)}

    def rows(rid, pos0, n, heads, what, layer):      # timing run: any rows will do
        return bank[heads][:n] if n <= 4096 else bank[heads].repeat((n + 4095) // 4096, 1, 1)[:n]

    arms = {"budgeted_pipelined": (base, "pipelined"),
            "copy_all_pipelined": (dict(base, t_block_ps=1), "pipelined"),
            "copy_all_layer_synchronous": (dict(base, t_block_ps=1), "synchronous"),
            "copy_all_full_reload_first": (dict(base, t_block_ps=1), "full_reload_first"),
            "recompute_no_host_copies": (dict(base, n_off_base=1 << 30), "pipelined")}
    res = dict(n_layers=L, device_blocks=M, host_slots=Mh, t_block_ps=t_block, rounds=steps)
    rng = np.random.default_rng(5)
    dev_order, host_order = rng.permutation(M), rng.permutation(Mh)
    for name, (cfg, mode) in arms.items():
        loop = ClosedLoop(Hq, Hkv, M, Mh, L, cfg, dev_order, host_order, rows, reload_mode=mode, out_dtype=B.PS_BF16, device=dev)
        st = loop.run(trace, steps, clock="measured")
        sc = loop.score(trace)
        loop.close()
        res[name] = dict(pass_ms=st["pass_ms"], ms_per_round=st["pass_ms"] / max(st["steps"], 1), tokens=st["tokens"],
                         evicted=st["evicted"], blocks_reloaded=st["blocks_reloaded"], blocks_offloaded=st["blocks_offloaded"],
                         recomputed_tokens=st["recomputed_tokens"],
                         tokens_per_pass_ms=st["tokens"] / st["pass_ms"] if st["pass_ms"] else 0.0,
                         finished=sc["finished"], tdg_ratio=sc["tdg_ratio"], slo_attainment=sc["slo_attainment"])
        del loop
        torch.cuda.empty_cache()
    return res


def graph_bench(B, W, torch, np, dev, n_layers=36):
    """A launch-bound case: 16 decode requests of about 1 k tokens (a kernel of a few microseconds per layer).
    One forward pass of n_layers layers, three ways: ps_step on every layer; ps_step on the first layer and
    ps_step_next_layer on the rest; the same with the rest captured once into a HIP graph and replayed."""
    import time as _t
    shape = W.LayerShape(32, 8)
    rng = np.random.default_rng(99)
    items = [(1, int(x)) for x in rng.integers(600, 1400, size=16)]
    batch = W.build_batch(shape, items, [1] * len(items), rng, name="16 decode requests", seed=99)
    g = torch.Generator(device=dev)
    g.manual_seed(99)
    pool = torch.empty((batch.n_device_blocks, shape.block_bytes // 2), dtype=torch.bfloat16, device=dev).normal_(generator=g)
    q = torch.randn((batch.n_tokens, shape.n_q_heads, shape.head_dim), generator=g, device=dev).to(torch.bfloat16)
    kn = torch.randn((batch.n_tokens, shape.n_kv_heads, shape.head_dim), generator=g, device=dev).to(torch.bfloat16)
    vn = torch.randn((batch.n_tokens, shape.n_kv_heads, shape.head_dim), generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    ctx = B.ps_create(shape.n_q_heads, shape.n_kv_heads, batch.n_device_blocks, 0)
    nbytes = B.ps_workspace_bytes(ctx, batch.n_req, batch.n_tokens, len(batch.block_ids))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    cb = B.make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, batch.prio)
    side = torch.cuda.Stream()

    def first():
        B.ps_step(ctx, cb, q, kn, vn, pool, out, ws, nbytes, side)

    def rest():
        for _ in range(n_layers - 1):
            B.ps_step_next_layer(ctx, q, kn, vn, pool, out, ws, nbytes, side)

    def timed(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        t0 = _t.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (_t.perf_counter() - t0) / (reps * n_layers) * 1e6

    res = dict(batch=batch.name, n_layers=n_layers)
    res["ps_step_every_layer_us_per_layer"] = timed(lambda: [first() for _ in range(n_layers)])
    res["plan_once_us_per_layer"] = timed(lambda: (first(), rest()))
    first()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rest()

    def replayed():
        first()
        with torch.cuda.stream(side):
            graph.replay()
    res["plan_once_graph_replay_us_per_layer"] = timed(replayed)
    del graph
    B.ps_destroy(ctx)
    return res


def sched_bench(B, W, np, step_ms):
    """Host time of ps_form_batch (SlideBatching + block management) on a steady synthetic trace whose
    batches resemble the headline workload (a few hundred decoding requests plus prefill chunks)."""
    import time as _t
    MS, US, NS, L = 10 ** 9, 10 ** 6, 10 ** 3, 36
    cfg = dict(n_classes=3, block_tokens=16, class_weight=[4, 2, 1], w_first=4, w_decode=1, ttft_slo_ps=2000 * MS,
               tpot_slo_ps=100 * MS, a_p=(13 * L) // 2, b_p=13 * L, c_p=50 * NS * L, a_d=730 * L, b_d=1 * US * L,
               t_c=2 * MS, eta_ps=10 * MS, tau_ps=30_000 * MS, gamma_num=9, gamma_den=10, beta_num=2, beta_den=1,
               rho_num=9, rho_den=10, t_block_ps=1200 * NS * L, n_off_base=8)
    trace = W.make_trace(2, 4000, rate_per_s=60.0, out_mean=256.0)
    rng = np.random.default_rng(1)
    M = 40_000
    s = B.ps_sched_create(cfg, rng.permutation(M).astype(np.int32), rng.permutation(2 * M).astype(np.int32))
    pending = sorted(trace, key=lambda x: (x.arrival_ps, x.rid))
    nxt, now, calls, t_sched, members, queued = 0, 0, 0, 0.0, 0, 0
    import ctypes as _C
    raw = B.ps_batch_out()
    while calls < 1500 and (nxt < len(pending) or B.ps_sched_counts(s)[0] > 0):
        while nxt < len(pending) and pending[nxt].arrival_ps <= now:
            p = pending[nxt]
            B.ps_sched_add_request(s, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len)
            nxt += 1
        if B.ps_sched_counts(s)[0] == 0:
            now = pending[nxt].arrival_ps
            continue
        t0 = _t.perf_counter()
        B.lib().ps_form_batch(s, now, _C.byref(raw))       # the C call alone, no copy-out
        dt = _t.perf_counter() - t0
        calls += 1
        if calls > 500:                      # steady state only
            t_sched += dt
            members += raw.batch.n_req
            queued += raw.n_order
        now += raw.t_batch_ps if raw.t_batch_ps > 0 else cfg["eta_ps"]
    B.ps_sched_destroy(s)
    n = max(calls - 500, 1)
    us = t_sched / n * 1e6
    return {"form_batch_us_per_call": us, "mean_batch_members": members / n, "mean_queue_len": queued / n,
            "frac_of_one_layer_step": us * 1e-3 / step_ms, "frac_of_36_layer_step": us * 1e-3 / (36 * step_ms)}


if __name__ == "__main__":
    sys.exit(main())
