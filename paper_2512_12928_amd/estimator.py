"""Batch latency estimator of Sec. 4.1 (Eqs. 4-7), fitted to measured ps_step times on this machine.

    T(B) = sum over prefill requests (a_p l_q^2 + b_p l_q l_kv + c_p l_q)
         + sum over decode requests  (a_d l_kv + b_d)  +  t_c

is linear in (a_p, b_p, c_p, a_d, b_d, t_c), so the "training on offline profiling batches" the paper
describes is a least-squares problem on six batch features.  `python -m paper_2512_12928_amd.estimator`
draws seeded profiling batches, times ps_step on each (GPU needed), fits on one half and reports the mean
absolute percentage error on the other (the paper reports about 4.5 % for its whole-model estimator; here
only the attention layer is timed).  l_kv follows the scheduler's convention: cached prefix before this pass
for a prefill request, context including this token for a decode request.

Eq. 7 adds the requests' costs up.  One launch of this library is not quite additive: a batch whose prefill
work is a few long rows ends when the longest walk over the KV range ends, however little work there is in
total.  `fit_with_critical_path` therefore also fits the form

    T(B) = max( Eq. 7 ,  t_c + w * (64-token KV tiles the longest prefill row walks) )

(one more parameter, w).  Nor is a mixed launch the sum of its two kinds of work: decode waits for memory while prefill
computes, and part of the shorter of the two hides under the longer.  `fit_with_overlap` fits

    T(B) = t_c + max(P, D) + kappa * min(P, D),   P = max(prefill terms of Eq. 7, w * longest walk),  D = decode terms

(two more parameters, kappa and w; kappa = 1 and w = 0 give Eq. 7 back).  The batch former keeps the paper's additive form.
"""
from __future__ import annotations

import json
import sys
import time
from typing import List, Sequence, Tuple

import numpy as np

from . import workloads as W

PARAMS = ("a_p", "b_p", "c_p", "a_d", "b_d", "t_c")


def features(q_start: Sequence[int], kv_len: Sequence[int]) -> np.ndarray:
    """The six sums that multiply (a_p, b_p, c_p, a_d, b_d, t_c) in Eq. 7."""
    lq = np.diff(np.asarray(q_start, dtype=np.int64))
    kv = np.asarray(kv_len, dtype=np.int64)
    pre, dec = lq > 1, lq == 1
    prefix = kv[pre] - lq[pre]
    return np.array([float((lq[pre] ** 2).sum()), float((lq[pre] * prefix).sum()), float(lq[pre].sum()),
                     float(kv[dec].sum()), float(dec.sum()), 1.0])


def fit(X: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Least squares on relative error (each batch weighted by 1 / its time, the quantity MAPE measures),
    columns scaled for conditioning."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    Xw = X / y[:, None]
    scale = np.abs(Xw).max(axis=0)
    scale[scale == 0] = 1.0
    coef, *_ = np.linalg.lstsq(Xw / scale, np.ones_like(y), rcond=None)
    return coef / scale


def longest_walk(q_start: Sequence[int], kv_len: Sequence[int]) -> float:
    """64-token KV tiles the last query row of the longest prefill request walks (0 without prefill work)."""
    lq = np.diff(np.asarray(q_start, dtype=np.int64))
    kv = np.asarray(kv_len, dtype=np.int64)
    pre = lq > 1
    return float(-(-kv[pre].max() // 64)) if pre.any() else 0.0


def predict_max(coef: np.ndarray, w: float, X: np.ndarray, walk: np.ndarray) -> np.ndarray:
    coef = np.asarray(coef, dtype=np.float64)
    return np.maximum(np.asarray(X, dtype=np.float64) @ coef, coef[5] + w * np.asarray(walk, dtype=np.float64))


def fit_with_critical_path(X: np.ndarray, walk: np.ndarray, y: np.ndarray, rounds: int = 4):
    """Alternates between the additive coefficients (least squares on the batches the additive term explains)
    and w (a line search for the least mean relative error).  Returns (coef, w)."""
    X, walk, y = (np.asarray(a, dtype=np.float64) for a in (X, walk, y))
    coef, w = fit(X, y), 0.0
    for _ in range(rounds):
        grid = np.linspace(0.0, 4.0, 161)
        errs = [float(np.mean(np.abs(predict_max(coef, g, X, walk) - y) / y)) for g in grid]
        w = float(grid[int(np.argmin(errs))])
        additive = X @ coef >= coef[5] + w * walk
        if additive.sum() < 12:
            break
        coef = fit(X[additive], y[additive])
    return coef, w


def predict_overlap(coef: np.ndarray, kappa: float, w: float, X: np.ndarray, walk: np.ndarray) -> np.ndarray:
    X, walk, coef = (np.asarray(a, dtype=np.float64) for a in (X, walk, coef))
    P = np.maximum(X[:, :3] @ coef[:3], w * walk)
    D = X[:, 3:5] @ coef[3:5]
    return coef[5] + np.maximum(P, D) + kappa * np.minimum(P, D)


def fit_with_overlap(X: np.ndarray, walk: np.ndarray, y: np.ndarray, rounds: int = 8):
    """Grid over (kappa, w); for each pair the six coefficients by iterated least squares on relative error: with the
    larger kind of every batch fixed by the last iterate, the form is linear in them (the smaller kind's features
    weighted by kappa; a prefill part set by the critical path is a known term).  Returns (coef, kappa, w)."""
    X, walk, y = (np.asarray(a, dtype=np.float64) for a in (X, walk, y))
    best = None
    for kappa in np.linspace(0.2, 1.0, 17):
        for w in np.linspace(0.0, 1.2, 13):
            coef = fit(X, y)
            for _ in range(rounds):
                Pa, D = X[:, :3] @ coef[:3], X[:, 3:5] @ coef[3:5]
                crit = w * walk > Pa
                big_p = np.maximum(Pa, w * walk) >= D
                sp, sd = np.where(big_p, 1.0, kappa), np.where(big_p, kappa, 1.0)
                A = np.concatenate([X[:, :3] * (sp * ~crit)[:, None], X[:, 3:5] * sd[:, None], X[:, 5:6]], axis=1)
                rhs = y - sp * crit * w * walk
                Aw = A / y[:, None]
                scale = np.abs(Aw).max(axis=0)
                scale[scale == 0] = 1.0
                c, *_ = np.linalg.lstsq(Aw / scale, rhs / y, rcond=None)
                coef = c / scale
            err = float(np.mean(np.abs(predict_overlap(coef, kappa, w, X, walk) - y) / y))
            if best is None or err < best[0]:
                best = (err, coef, float(kappa), float(w))
    return best[1], best[2], best[3]


def predict(coef: np.ndarray, X: np.ndarray) -> np.ndarray:
    return np.asarray(X, dtype=np.float64) @ np.asarray(coef, dtype=np.float64)


def mape(coef: np.ndarray, X: np.ndarray, y: np.ndarray) -> float:
    y = np.asarray(y, dtype=np.float64)
    return float(np.mean(np.abs(predict(coef, X) - y) / y))


def profiling_batches(n: int, seed: int, shape: W.LayerShape, max_blocks: int) -> List[W.MixedBatch]:
    """Seeded synthetic profiling batches: 0-512 decode requests with lognormal contexts, 0-4 prefill chunks
    of 64-2048 tokens over prefixes of 0-8192 tokens, in random order; never empty."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        n_dec = int(rng.choice([0, 8, 32, 64, 128, 256, 384, 512]))
        n_pre = int(rng.integers(0, 5))
        if n_dec + n_pre == 0:
            continue
        mean = float(rng.choice([300, 800, 1500, 3000]))
        items: List[Tuple[int, int]] = []
        for _ in range(n_dec):
            L = int(np.clip(rng.lognormal(np.log(mean) - 0.32, 0.8), 16, 16384))
            items.append((1, L))
        for _ in range(n_pre):
            lq = int(rng.choice([64, 128, 256, 512, 1024, 2048]))
            items.append((lq, lq + int(rng.choice([0, 256, 1024, 2048, 4096, 8192]))))
        order = rng.permutation(len(items))
        items = [items[i] for i in order]
        need = sum(-(-L // shape.block_tokens) for _, L in items)
        if need > max_blocks:
            continue
        out.append(W.build_batch(shape, items, [1] * len(items), rng, n_device_blocks=max_blocks, seed=seed))
    return out


def measure(batches: Sequence[W.MixedBatch], shape: W.LayerShape, n_blocks: int, steps: int = 20) -> np.ndarray:
    """Wall time per ps_step in microseconds for each batch (inputs resident, cache already filled)."""
    import torch
    from . import binding as B
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    pool = torch.empty((n_blocks, shape.block_bytes // 2), dtype=torch.bfloat16, device=dev).normal_(generator=g)
    max_tok = max(b.n_tokens for b in batches)
    q = torch.randn((max_tok, shape.n_q_heads, shape.head_dim), generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    ctx = B.ps_create(shape.n_q_heads, shape.n_kv_heads, n_blocks, 0)
    nbytes = B.ps_workspace_bytes(ctx, max(b.n_req for b in batches), max_tok, max(len(b.block_ids) for b in batches))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    res = np.zeros(len(batches))
    for i, b in enumerate(batches):
        cb = B.make_batch(b.q_start, b.kv_len, b.bt_start, b.block_ids, b.prio)
        for _ in range(3):
            B.ps_step(ctx, cb, q, None, None, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.ps_step(ctx, cb, q, None, None, pool, out, ws, nbytes, stream)
        torch.cuda.synchronize()
        res[i] = (time.perf_counter() - t0) / steps * 1e6
    B.ps_destroy(ctx)
    return res


def main(argv=None) -> int:
    """python -m paper_2512_12928_amd.estimator [n_batches [file]]: the fit; with a file name the batches and their
    measured times are also written there (JSON) for fitting other forms without a GPU."""
    n = int(argv[0]) if argv else 240
    shape = W.LayerShape(32, 8)
    n_blocks = 60_000
    batches = profiling_batches(n, 2512_12928, shape, n_blocks)
    y = measure(batches, shape, n_blocks)
    X = np.stack([features(b.q_start, b.kv_len) for b in batches])
    walk = np.array([longest_walk(b.q_start, b.kv_len) for b in batches])
    if argv and len(argv) > 1:
        with open(argv[1], "w") as f:
            json.dump([dict(l_q=np.diff(b.q_start).tolist(), kv_len=np.asarray(b.kv_len).tolist(), us=float(t))
                       for b, t in zip(batches, y)], f)
    half = n // 2
    coef = fit(X[:half], y[:half])
    coef_m, w = fit_with_critical_path(X[:half], walk[:half], y[:half])
    rel_m = np.abs(predict_max(coef_m, w, X[half:], walk[half:]) - y[half:]) / y[half:]
    coef_o, kappa_o, w_o = fit_with_overlap(X[:half], walk[:half], y[:half])
    rel_o = np.abs(predict_overlap(coef_o, kappa_o, w_o, X[half:], walk[half:]) - y[half:]) / y[half:]
    kinds = np.array([("mixed" if (x[2] > 0 and x[4] > 0) else ("prefill" if x[2] > 0 else "decode")) for x in X[half:]])
    res = dict(n_train=half, n_eval=n - half, unit="us per ps_step (one attention layer, 32q/8kv)",
               params={k: float(v) for k, v in zip(PARAMS, coef)},
               mape_train=mape(coef, X[:half], y[:half]), mape_eval=mape(coef, X[half:], y[half:]),
               mape_eval_by_kind={k: mape(coef, X[half:][kinds == k], y[half:][kinds == k]) for k in np.unique(kinds)},
               with_critical_path=dict(params={k: float(v) for k, v in zip(PARAMS, coef_m)}, w_us_per_tile=w,
                                       mape_eval=float(rel_m.mean()),
                                       mape_eval_by_kind={k: float(rel_m[kinds == k].mean()) for k in np.unique(kinds)}),
               with_overlap=dict(params={k: float(v) for k, v in zip(PARAMS, coef_o)}, kappa=kappa_o, w_us_per_tile=w_o,
                                 mape_eval=float(rel_o.mean()),
                                 mape_eval_by_kind={k: float(rel_o[kinds == k].mean()) for k in np.unique(kinds)}),
               step_us_range=[float(y.min()), float(y.max())])
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
