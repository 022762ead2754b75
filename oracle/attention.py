"""Oracle A: causal softmax attention over a paged KV cache, in fp64.

TEST INFRASTRUCTURE ONLY.  The paper (Sec. 4.1, batch latency estimator; Sec. 4.3, block
management) fixes that a batch mixes prefill chunks of l_q tokens over a cached prefix
with single-token decode requests, and that the KV cache lives in fixed-size blocks
reached through per-request block lists.  It describes no kernel; the attention itself is
the textbook definition, written out here with a matmul as the only library step:

  request r, l_q query tokens, L = kv_len (includes these tokens), prefix p = L - l_q;
  query i (absolute position p+i), q-head h, kv-head g = h // G  (G = Hq/Hkv):
      s_j = <q_ih, k_jg> * scale        for j in [0, p+i]
      P_j = exp(s_j - max s) / sum_j exp(s_j - max s)
      o_ih = sum_j P_j v_jg
  token j lives in physical block  table[j // blk], slot j % blk.

The oracle's own paged pool is  pool[M, 2, Hkv, blk, d]  (index 0 = K, 1 = V) of bf16 bit
patterns; it is private to the oracle (the HIP library documents a different layout).
"""
from __future__ import annotations

import numpy as np


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64 (exact)."""
    b = np.asarray(bits)
    assert b.dtype == np.uint16
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def softmax_rows(s: np.ndarray, valid: np.ndarray) -> np.ndarray:
    """Row-wise softmax over the positions where ``valid`` is True; 0 elsewhere."""
    neg = np.where(valid, s, -np.inf)
    m = neg.max(axis=-1, keepdims=True)
    e = np.where(valid, np.exp(np.where(valid, s, 0.0) - m), 0.0)
    return e / e.sum(axis=-1, keepdims=True)


def dense_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None,
                    return_probs: bool = False):
    """q [l_q,Hq,d], k/v [L,Hkv,d] float64 -> o [l_q,Hq,d] float64.
    Query i sees keys 0 .. (L-l_q)+i."""
    l_q, Hq, d = q.shape
    L, Hkv, _ = k.shape
    assert L >= l_q and Hq % Hkv == 0
    G = Hq // Hkv
    p = L - l_q
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    valid = np.arange(L)[None, :] <= (p + np.arange(l_q))[:, None]
    o = np.empty((l_q, Hq, d), dtype=np.float64)
    probs = np.empty((l_q, Hq, L), dtype=np.float64) if return_probs else None
    for h in range(Hq):
        g = h // G
        s = (q[:, h, :] @ k[:, g, :].T) * scale
        P = softmax_rows(s, valid)
        o[:, h, :] = P @ v[:, g, :]
        if return_probs:
            probs[:, h, :] = P
    return (o, probs) if return_probs else o


class PagedKV:
    """The oracle's paged cache: fixed-size blocks reached through block tables."""

    def __init__(self, n_blocks: int, n_kv_heads: int, block_tokens: int, head_dim: int, fill=None):
        self.blk = block_tokens
        self.pool = np.zeros((n_blocks, 2, n_kv_heads, block_tokens, head_dim), dtype=np.uint16)
        if fill is not None:
            self.pool[...] = fill

    def append(self, table: np.ndarray, pos0: int, k_rows: np.ndarray, v_rows: np.ndarray) -> None:
        """Store rows for logical positions pos0 .. pos0+n-1 of the request owning ``table``."""
        j = pos0 + np.arange(k_rows.shape[0])
        b = np.asarray(table)[j // self.blk]
        # pool[b, 0, :, slot, :] with paired index arrays (b, slot): result axes [n, Hkv, d]
        self.pool[b, 0, :, j % self.blk, :] = k_rows
        self.pool[b, 1, :, j % self.blk, :] = v_rows

    def gather(self, table: np.ndarray, L: int):
        """Logical K, V [L,Hkv,d] (bf16 bits) of one request: token j from block table[j//blk], slot j%blk."""
        j = np.arange(L)
        b = np.asarray(table)[j // self.blk]
        return self.pool[b, 0, :, j % self.blk, :].copy(), self.pool[b, 1, :, j % self.blk, :].copy()


def paged_attention(q_bits: np.ndarray, cache: PagedKV, q_start, kv_len, bt_start, block_ids,
                    scale: float | None = None, requests=None) -> np.ndarray:
    """One attention layer over a mixed batch.  q_bits [n_tokens,Hq,d] bf16 bits; the
    cache must already hold every request's kv_len tokens.  Returns float64
    [n_tokens,Hq,d]; rows of requests not in ``requests`` (if given) are NaN."""
    n_tok, Hq, d = q_bits.shape
    out = np.full((n_tok, Hq, d), np.nan, dtype=np.float64)
    reqs = range(len(kv_len)) if requests is None else requests
    for r in reqs:
        a, b = int(q_start[r]), int(q_start[r + 1])
        table = block_ids[int(bt_start[r]):int(bt_start[r + 1])]
        kb, vb = cache.gather(table, int(kv_len[r]))
        out[a:b] = dense_attention(bf16_to_f64(q_bits[a:b]), bf16_to_f64(kb), bf16_to_f64(vb), scale)
    return out


def attention_rows(q_rows_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray,
                   n_visible: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Sampled-row form for full-size parity: row t of q_rows_bits [n,Hq,d] sees the first
    n_visible[t] tokens of k/v [L,Hkv,d].  Same definition, one row at a time."""
    n, Hq, d = q_rows_bits.shape
    k = bf16_to_f64(k_bits)
    v = bf16_to_f64(v_bits)
    out = np.empty((n, Hq, d), dtype=np.float64)
    for t in range(n):
        nv = int(n_visible[t])
        out[t] = dense_attention(bf16_to_f64(q_rows_bits[t:t + 1]), k[:nv], v[:nv], scale)[0]
    return out


# --- split-K merge identity (how partitioned softmax partials recombine) ------------------
def partial_softmax(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """One head, one query, one KV partition: returns (m, l, o~) with
    m = max s, l = sum exp(s-m), o~ = sum exp(s-m) v  (unnormalised)."""
    s = (k @ q) * scale
    m = s.max()
    e = np.exp(s - m)
    return m, e.sum(), e @ v


def merge_partials(parts):
    """Combine (m, l, o~) partials: m* = max m_i, l* = sum l_i e^{m_i-m*},
    o = sum o~_i e^{m_i-m*} / l*."""
    m_star = max(p[0] for p in parts)
    l_star = sum(p[1] * np.exp(p[0] - m_star) for p in parts)
    o = sum(p[2] * np.exp(p[0] - m_star) for p in parts)
    return o / l_star
