"""ctypes binding of the C ABI in include/ps.h -- argument marshalling only.

Every function has the name and meaning of its C counterpart; all computation happens in
the HIP library.  Loading fails loudly if the library has not been built
(``python -m paper_2512_12928_amd.build``); there is no fallback path.

Tensors may be passed as torch tensors (their ``data_ptr()`` is used; the caller keeps them
alive and on the right device) or as integer addresses.  Batch arrays are numpy int32.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libproserve_mi355x.so")

PS_OK, PS_EINVAL, PS_ENOMEM, PS_EHIP, PS_ESTATE, PS_EBUSY = 0, -1, -2, -3, -4, -5
PS_BF16, PS_F32 = 0, 1

EXPORTS = [
    "ps_last_error", "ps_create", "ps_destroy", "ps_workspace_bytes", "ps_step", "ps_step_next_layer", "ps_set_profiling",
    "ps_get_step_times", "ps_plan_decode", "ps_plan_launch", "ps_swap_out", "ps_swap_in", "ps_ticket_query", "ps_ticket_wait",
    "ps_sched_create", "ps_sched_destroy", "ps_sched_add_request", "ps_form_batch", "ps_sched_counts",
    "ps_sched_offloads_done", "ps_tdg_score", "ps_sched_simulate", "ps_step_static", "ps_mixed_launch_faults",
]


class ps_layer_cfg(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_tokens", C.c_int32), ("n_device_blocks", C.c_int32), ("n_host_blocks", C.c_int32),
                ("softmax_scale", C.c_float), ("out_dtype", C.c_int32), ("decode_chunk", C.c_int32),
                ("swap_workgroups", C.c_int32), ("own_streams", C.c_int32), ("prefill_split_tiles", C.c_int32),
                ("decode_waves", C.c_int32), ("plan_stream_TBps", C.c_float), ("plan_tile_step_us", C.c_float),
                ("plan_merge_launch_steps", C.c_float), ("plan_merge_row_steps", C.c_float), ("plan_decode_share", C.c_float),
                ("plan_decode_knee_cus", C.c_int32), ("swap_dma_runs", C.c_int32), ("mixed_launch", C.c_int32)]


class ps_batch(C.Structure):
    _fields_ = [("n_req", C.c_int32), ("n_tokens", C.c_int32), ("q_start", C.POINTER(C.c_int32)),
                ("kv_len", C.POINTER(C.c_int32)), ("bt_start", C.POINTER(C.c_int32)),
                ("block_ids", C.POINTER(C.c_int32)), ("prio", C.POINTER(C.c_uint8))]


class ps_step_times(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("upload_ms", "append_ms", "decode_ms", "merge_ms", "prefill_ms", "total_ms",
                                             "attention_ms", "decode_mhz", "prefill_mhz")]


class ps_sched_cfg(C.Structure):
    _fields_ = [("n_classes", C.c_int32), ("block_tokens", C.c_int32), ("class_weight", C.c_int64 * 8),
                ("w_first", C.c_int64), ("w_decode", C.c_int64), ("ttft_slo_ps", C.c_int64),
                ("tpot_slo_ps", C.c_int64), ("a_p", C.c_int64), ("b_p", C.c_int64), ("c_p", C.c_int64),
                ("a_d", C.c_int64), ("b_d", C.c_int64), ("t_c", C.c_int64), ("eta_ps", C.c_int64),
                ("tau_ps", C.c_int64), ("gamma_num", C.c_int64), ("gamma_den", C.c_int64),
                ("beta_num", C.c_int64), ("beta_den", C.c_int64), ("rho_num", C.c_int64), ("rho_den", C.c_int64),
                ("t_block_ps", C.c_int64), ("n_off_base", C.c_int32), ("order_policy", C.c_int32)]


PS_ORDER_SLIDEBATCHING, PS_ORDER_FCFS = 0, 1


class ps_trace_req(C.Structure):
    _fields_ = [("rid", C.c_int64), ("arrival_ps", C.c_int64), ("prio", C.c_int32), ("prompt_len", C.c_int32),
                ("out_len", C.c_int32), ("reserved", C.c_int32)]


class ps_sim_result(C.Structure):
    _fields_ = [("gain", C.c_int64), ("ideal_gain", C.c_int64), ("slo_attained", C.c_int32), ("finished", C.c_int32),
                ("steps", C.c_int32), ("reserved", C.c_int32), ("end_ps", C.c_int64)]


class ps_batch_out(C.Structure):
    _fields_ = [("batch", ps_batch), ("req_ids", C.POINTER(C.c_int64)), ("t_budget_ps", C.c_int64),
                ("phi_ps", C.c_int64), ("t_batch_ps", C.c_int64), ("copy_budget", C.c_int64),
                ("n_order", C.c_int32), ("n_urgent", C.c_int32), ("order", C.POINTER(C.c_int64)),
                ("urgent", C.POINTER(C.c_int64)), ("n_swap_in", C.c_int32), ("n_swap_out", C.c_int32),
                ("swap_in_host_slots", C.POINTER(C.c_int32)), ("swap_in_dev_blocks", C.POINTER(C.c_int32)),
                ("swap_out_dev_blocks", C.POINTER(C.c_int32)), ("swap_out_host_slots", C.POINTER(C.c_int32)),
                ("n_evicted", C.c_int32), ("n_emitted", C.c_int32), ("evicted", C.POINTER(C.c_int64)),
                ("emitted_req", C.POINTER(C.c_int64)), ("emitted_index", C.POINTER(C.c_int32)),
                ("n_finished", C.c_int32), ("reserved", C.c_int32), ("finished", C.POINTER(C.c_int64)),
                ("round", C.c_int64)]


class PsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("ps error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """The loaded shared library; raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s not built: run `python -m paper_2512_12928_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.ps_last_error.restype = C.c_char_p
        L.ps_create.argtypes = [C.POINTER(ps_layer_cfg), C.POINTER(C.c_void_p)]
        L.ps_destroy.argtypes = [C.c_void_p]
        L.ps_destroy.restype = None
        L.ps_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.POINTER(C.c_size_t)]
        L.ps_step.argtypes = [C.c_void_p, C.POINTER(ps_batch)] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p, C.c_uint64]
        L.ps_step_static.argtypes = [C.c_void_p, C.POINTER(ps_batch)] + [C.c_void_p] * 5 + [C.c_void_p, C.c_uint64]
        L.ps_plan_launch.argtypes = [C.POINTER(ps_layer_cfg), C.POINTER(ps_batch), C.c_int32, C.POINTER(C.c_int32)]
        L.ps_mixed_launch_faults.argtypes = [C.POINTER(C.c_uint32)]
        L.ps_step_next_layer.argtypes = [C.c_void_p] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p, C.c_uint64]
        L.ps_set_profiling.argtypes = [C.c_void_p, C.c_int]
        L.ps_get_step_times.argtypes = [C.c_void_p, C.POINTER(ps_step_times)]
        swap_args = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_void_p,
                     C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]
        L.ps_swap_out.argtypes = swap_args
        L.ps_swap_in.argtypes = swap_args
        L.ps_ticket_query.argtypes = [C.c_void_p, C.c_uint64]
        L.ps_ticket_wait.argtypes = [C.c_void_p, C.c_uint64]
        L.ps_sched_create.argtypes = [C.POINTER(ps_sched_cfg), C.POINTER(C.c_int32), C.c_int32,
                                      C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p)]
        L.ps_sched_destroy.argtypes = [C.c_void_p]
        L.ps_sched_destroy.restype = None
        L.ps_sched_add_request.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.ps_form_batch.argtypes = [C.c_void_p, C.c_int64, C.POINTER(ps_batch_out)]
        L.ps_sched_counts.argtypes = [C.c_void_p] + [C.POINTER(C.c_int32)] * 3
        L.ps_sched_offloads_done.argtypes = [C.c_void_p, C.c_int64]
        L.ps_tdg_score.argtypes = [C.POINTER(ps_sched_cfg), C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.c_int32,
                                   C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.ps_sched_simulate.argtypes = [C.POINTER(ps_sched_cfg), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                        C.c_int32, C.POINTER(ps_trace_req), C.c_int32, C.c_int32, C.POINTER(C.c_int64),
                                        C.POINTER(C.c_int32), C.POINTER(ps_sim_result)]
        _lib = L
    return _lib


def ps_last_error() -> str:
    return lib().ps_last_error().decode()


def _check(rc: int, ok=(PS_OK,)) -> int:
    if rc not in ok:
        raise PsError(rc, ps_last_error())
    return rc


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return int(s.cuda_stream)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def ps_create(n_q_heads: int, n_kv_heads: int, n_device_blocks: int, n_host_blocks: int = 0,
              softmax_scale: float = 0.0, out_dtype: int = PS_BF16, decode_chunk: int = 0,
              swap_workgroups: int = 0, head_dim: int = 128, block_tokens: int = 16,
              own_streams: int = 0, prefill_split_tiles: int = 0, decode_waves: int = 0, **plan) -> int:
    """plan: the planner constants of ps_layer_cfg by name (plan_stream_TBps, ...), swap_dma_runs, mixed_launch;
    0 or absent = default."""
    cfg = ps_layer_cfg(n_q_heads, n_kv_heads, head_dim, block_tokens, n_device_blocks, n_host_blocks,
                       softmax_scale, out_dtype, decode_chunk, swap_workgroups, own_streams, prefill_split_tiles,
                       decode_waves)
    for k, v in plan.items():
        if not (k.startswith("plan_") or k in ("swap_dma_runs", "mixed_launch")):
            raise TypeError("unknown ps_layer_cfg field %r" % k)
        setattr(cfg, k, v)
    h = C.c_void_p()
    _check(lib().ps_create(C.byref(cfg), C.byref(h)))
    return h.value


def ps_destroy(ctx: int) -> None:
    lib().ps_destroy(ctx)


def ps_workspace_bytes(ctx: int, max_req: int, max_tokens: int, max_table_entries: int) -> int:
    out = C.c_size_t()
    _check(lib().ps_workspace_bytes(ctx, max_req, max_tokens, max_table_entries, C.byref(out)))
    return out.value


def make_batch(q_start, kv_len, bt_start, block_ids, prio=None):
    """Builds the C struct; returns (struct, keepalive) -- keep both until the call returns."""
    qs, kv, bs, ids = _i32(q_start), _i32(kv_len), _i32(bt_start), _i32(block_ids)
    pr = None if prio is None else np.ascontiguousarray(prio, dtype=np.uint8)
    b = ps_batch(len(kv), int(qs[-1]) if len(qs) else 0, _i32p(qs), _i32p(kv), _i32p(bs), _i32p(ids),
                 None if pr is None else pr.ctypes.data_as(C.POINTER(C.c_uint8)))
    return b, (qs, kv, bs, ids, pr)


def ps_step(ctx: int, batch, q, k_new, v_new, kv_cache, out, workspace, workspace_bytes: int,
            stream=None, wait_ticket: int = 0) -> None:
    """batch: a ps_batch struct, a (struct, keepalive) pair from make_batch, or an object with
    q_start / kv_len / bt_start / block_ids (/ prio) arrays."""
    keep = None
    if isinstance(batch, tuple):
        batch, keep = batch
    elif not isinstance(batch, ps_batch):
        batch, keep = make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids,
                                 getattr(batch, "prio", None))
    _check(lib().ps_step(ctx, C.byref(batch), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_cache), _ptr(out),
                         _ptr(workspace), workspace_bytes, _stream(stream), wait_ticket))
    del keep


PS_STATIC_SCRATCH_BYTES = 32 << 20


def ps_step_static(ctx: int, batch, q, k_new, v_new, kv_cache, out, stream=None, wait_ticket: int = 0) -> None:
    """ps_step without a workspace argument and without any allocation; batch as for ps_step."""
    keep = None
    if isinstance(batch, tuple):
        batch, keep = batch
    elif not isinstance(batch, ps_batch):
        batch, keep = make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids,
                                 getattr(batch, "prio", None))
    _check(lib().ps_step_static(ctx, C.byref(batch), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_cache), _ptr(out),
                                _stream(stream), wait_ticket))
    del keep


def ps_plan_launch(n_q_heads: int, n_kv_heads: int, n_device_blocks: int, batch, n_cus: int = 256, **cfg_kw) -> dict:
    """Host only.  batch: as for ps_step."""
    cfg = ps_layer_cfg()
    cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.block_tokens, cfg.n_device_blocks = n_q_heads, n_kv_heads, 128, 16, n_device_blocks
    for k, v in cfg_kw.items():
        setattr(cfg, k, v)
    keep = None
    if isinstance(batch, tuple):
        batch, keep = batch
    elif not isinstance(batch, ps_batch):
        batch, keep = make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, getattr(batch, "prio", None))
    out = (C.c_int32 * 6)()
    _check(lib().ps_plan_launch(C.byref(cfg), C.byref(batch), n_cus, out))
    del keep
    return dict(zip(("decode_waves", "decode_slots", "decode_workgroups", "prefill_workgroups", "prefill_split_tiles",
                     "partial_slots"), [int(x) for x in out]))


def ps_mixed_launch_faults() -> int:
    n = C.c_uint32()
    _check(lib().ps_mixed_launch_faults(C.byref(n)))
    return int(n.value)


def ps_step_next_layer(ctx: int, q, k_new, v_new, kv_cache, out, workspace, workspace_bytes: int,
                       stream=None, wait_ticket: int = 0) -> None:
    _check(lib().ps_step_next_layer(ctx, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_cache), _ptr(out),
                                    _ptr(workspace), workspace_bytes, _stream(stream), wait_ticket))


def ps_plan_decode(n_kv_heads: int, n_device_blocks: int, batch, waves: int, decode_chunk: int = 0):
    """Host only.  batch: as for ps_step.  Returns (segments int32 [n_seg, 5] = request, t0, t1, slot,
    part; n_slots)."""
    cfg = ps_layer_cfg()
    cfg.n_kv_heads, cfg.n_device_blocks, cfg.decode_chunk = n_kv_heads, n_device_blocks, decode_chunk
    keep = None
    if isinstance(batch, tuple):
        batch, keep = batch
    elif not isinstance(batch, ps_batch):
        batch, keep = make_batch(batch.q_start, batch.kv_len, batch.bt_start, batch.block_ids, getattr(batch, "prio", None))
    n_seg, n_slots = C.c_int32(), C.c_int32()
    rc = lib().ps_plan_decode(C.byref(cfg), C.byref(batch), waves, None, 0, C.byref(n_seg), C.byref(n_slots))
    if rc not in (PS_OK, PS_ENOMEM):
        _check(rc)
    seg = np.zeros((max(n_seg.value, 1), 5), dtype=np.int32)
    _check(lib().ps_plan_decode(C.byref(cfg), C.byref(batch), waves, _i32p(seg), n_seg.value, C.byref(n_seg),
                                C.byref(n_slots)))
    del keep
    return seg[:n_seg.value].copy(), n_slots.value


def ps_set_profiling(ctx: int, mode) -> None:
    _check(lib().ps_set_profiling(ctx, int(mode)))


def ps_get_step_times(ctx: int) -> dict:
    t = ps_step_times()
    _check(lib().ps_get_step_times(ctx, C.byref(t)))
    return {n: getattr(t, n) for n, _ in ps_step_times._fields_}


def _swap(fn, ctx, first_ids, second_ids, copy_budget, a, b, stream) -> Tuple[int, int]:
    x, y = _i32(first_ids), _i32(second_ids)
    if len(x) != len(y):
        raise ValueError("id lists differ in length")
    n_done, ticket = C.c_int32(), C.c_uint64()
    _check(fn(ctx, _i32p(x), _i32p(y), len(x), copy_budget, _ptr(a), _ptr(b), _stream(stream),
              C.byref(n_done), C.byref(ticket)))
    return n_done.value, ticket.value


def ps_swap_out(ctx: int, dev_block_ids, host_slot_ids, copy_budget: int, kv_cache, host_pool,
                side_stream=None) -> Tuple[int, int]:
    return _swap(lib().ps_swap_out, ctx, dev_block_ids, host_slot_ids, copy_budget, kv_cache, host_pool, side_stream)


def ps_swap_in(ctx: int, host_slot_ids, dev_block_ids, copy_budget: int, host_pool, kv_cache,
               side_stream=None) -> Tuple[int, int]:
    return _swap(lib().ps_swap_in, ctx, host_slot_ids, dev_block_ids, copy_budget, host_pool, kv_cache, side_stream)


def ps_ticket_query(ctx: int, ticket: int) -> int:
    """PS_OK when done, PS_EBUSY while in flight."""
    return _check(lib().ps_ticket_query(ctx, ticket), ok=(PS_OK, PS_EBUSY))


def ps_ticket_wait(ctx: int, ticket: int) -> None:
    _check(lib().ps_ticket_wait(ctx, ticket))


# ---------------------------------------------------------------------------- batch former
def _sched_cfg(cfg: dict) -> ps_sched_cfg:
    c = ps_sched_cfg()
    for k, v in cfg.items():
        if k == "class_weight":
            for i, w in enumerate(v):
                c.class_weight[i] = int(w)
        else:
            setattr(c, k, int(v))
    return c


def ps_tdg_score(cfg: dict, prio: int, out_len: int, token_times) -> Tuple[int, int, int]:
    """(gain, ideal gain, SLO attained) of one request; token_times relative to its arrival."""
    c = _sched_cfg(cfg)
    t = np.ascontiguousarray(token_times, dtype=np.int64)
    g, ideal, ok = C.c_int64(), C.c_int64(), C.c_int32()
    _check(lib().ps_tdg_score(C.byref(c), prio, out_len, t.ctypes.data_as(C.POINTER(C.c_int64)), len(t), C.byref(g),
                              C.byref(ideal), C.byref(ok)))
    return g.value, ideal.value, ok.value


def ps_sched_simulate(cfg: dict, dev_free_order, host_free_order, trace, max_steps: int) -> dict:
    """trace: objects with rid, arrival_ps, prio, prompt_len, out_len.  Returns the ps_sim_result fields plus
    token_times (one int64 array per request, in the order of `trace`)."""
    c = _sched_cfg(cfg)
    d, h = _i32(dev_free_order), _i32(host_free_order)
    tr = (ps_trace_req * max(len(trace), 1))()
    for i, p in enumerate(trace):
        tr[i] = ps_trace_req(p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len, 0)
    offs = np.zeros(len(trace) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([p.out_len for p in trace])
    times = np.zeros(max(int(offs[-1]), 1), dtype=np.int64)
    counts = np.zeros(max(len(trace), 1), dtype=np.int32)
    out = ps_sim_result()
    _check(lib().ps_sched_simulate(C.byref(c), _i32p(d), len(d), _i32p(h), len(h), tr, len(trace), max_steps,
                                   times.ctypes.data_as(C.POINTER(C.c_int64)), _i32p(counts), C.byref(out)))
    res = {n: getattr(out, n) for n, _ in ps_sim_result._fields_ if n != "reserved"}
    res["token_times"] = [times[offs[i]:offs[i] + counts[i]].copy() for i in range(len(trace))]
    return res


def ps_sched_create(cfg: dict, dev_free_order, host_free_order) -> int:
    """cfg: field name -> integer for ps_sched_cfg (class_weight as a list)."""
    c = _sched_cfg(cfg)
    d, h = _i32(dev_free_order), _i32(host_free_order)
    out = C.c_void_p()
    _check(lib().ps_sched_create(C.byref(c), _i32p(d), len(d), _i32p(h), len(h), C.byref(out)))
    return out.value


def ps_sched_destroy(s: int) -> None:
    lib().ps_sched_destroy(s)


def ps_sched_add_request(s: int, rid: int, arrival_ps: int, prio: int, prompt_len: int, out_len: int) -> None:
    _check(lib().ps_sched_add_request(s, rid, arrival_ps, prio, prompt_len, out_len))


def ps_sched_counts(s: int) -> Tuple[int, int, int]:
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().ps_sched_counts(s, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def ps_sched_offloads_done(s: int, upto_round: int) -> None:
    _check(lib().ps_sched_offloads_done(s, upto_round))


def ps_form_batch(s: int, now_ps: int) -> dict:
    """Runs one scheduling round and copies the result out of the scheduler's buffers."""
    o = ps_batch_out()
    _check(lib().ps_form_batch(s, now_ps, C.byref(o)))

    def arr(p, n, dt):
        return np.ctypeslib.as_array(p, shape=(n,)).astype(dt) if n > 0 else np.zeros(0, dtype=dt)

    n = o.batch.n_req
    nt = int(o.batch.bt_start[n]) if n > 0 else 0
    return dict(
        n_req=n, n_tokens=o.batch.n_tokens, q_start=arr(o.batch.q_start, n + 1, np.int32),
        kv_len=arr(o.batch.kv_len, n, np.int32), bt_start=arr(o.batch.bt_start, n + 1, np.int32),
        block_ids=arr(o.batch.block_ids, nt, np.int32), prio=arr(o.batch.prio, n, np.uint8),
        req_ids=arr(o.req_ids, n, np.int64), t_budget=o.t_budget_ps, phi=o.phi_ps, t_batch=o.t_batch_ps,
        copy_budget=o.copy_budget, order=arr(o.order, o.n_order, np.int64), urgent=arr(o.urgent, o.n_urgent, np.int64),
        swap_in_host_slots=arr(o.swap_in_host_slots, o.n_swap_in, np.int32),
        swap_in_dev_blocks=arr(o.swap_in_dev_blocks, o.n_swap_in, np.int32),
        swap_out_dev_blocks=arr(o.swap_out_dev_blocks, o.n_swap_out, np.int32),
        swap_out_host_slots=arr(o.swap_out_host_slots, o.n_swap_out, np.int32),
        evicted=arr(o.evicted, o.n_evicted, np.int64), emitted_req=arr(o.emitted_req, o.n_emitted, np.int64),
        emitted_index=arr(o.emitted_index, o.n_emitted, np.int32), finished=arr(o.finished, o.n_finished, np.int64),
        round=o.round)
