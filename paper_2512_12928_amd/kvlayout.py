"""The library's KV-cache layout (see include/ps.h) as numpy index permutations:
K  cache[b][0][g][x/8][t][x%8]  (groups of 8 dims, token-major inside a group),
V  cache[b][1][g][x][t]  (dim-major).

Converts between that device layout and the plain logical array pool[M, 2, Hkv, blk, d]
(0 = K, 1 = V; token-major for both), e.g. to import an existing cache or to read one back.
Pure index arithmetic on bit patterns; no method arithmetic."""
import numpy as np


def to_device_layout(pool: np.ndarray) -> np.ndarray:
    """logical pool [M,2,Hkv,blk,d] (bf16 bits) -> flat uint16 [M, 2*Hkv*blk*d] in device layout."""
    M, two, Hkv, blk, d = pool.shape
    out = np.empty((M, 2, Hkv, blk * d), dtype=np.uint16)
    out[:, 0] = pool[:, 0].reshape(M, Hkv, blk, d // 8, 8).transpose(0, 1, 3, 2, 4).reshape(M, Hkv, blk * d)
    out[:, 1] = pool[:, 1].transpose(0, 1, 3, 2).reshape(M, Hkv, blk * d)
    return out.reshape(M, -1)


def from_device_layout(flat: np.ndarray, Hkv: int, blk: int = 16, d: int = 128) -> np.ndarray:
    M = flat.shape[0]
    v = flat.reshape(M, 2, Hkv, blk * d)
    pool = np.empty((M, 2, Hkv, blk, d), dtype=np.uint16)
    pool[:, 0] = v[:, 0].reshape(M, Hkv, d // 8, blk, 8).transpose(0, 1, 3, 2, 4).reshape(M, Hkv, blk, d)
    pool[:, 1] = v[:, 1].reshape(M, Hkv, d, blk).transpose(0, 1, 3, 2)
    return pool


def request_kv(flat_blocks: np.ndarray, Hkv: int, kv_len: int, blk: int = 16, d: int = 128):
    """flat_blocks: the device-layout blocks of ONE request in logical order [nblk, 2*Hkv*blk*d].
    Returns logical K, V [kv_len, Hkv, d] (bf16 bits)."""
    pool = from_device_layout(flat_blocks, Hkv, blk, d)          # [nblk,2,Hkv,blk,d]
    k = pool[:, 0].transpose(0, 2, 1, 3).reshape(-1, Hkv, d)[:kv_len]
    v = pool[:, 1].transpose(0, 2, 1, 3).reshape(-1, Hkv, d)[:kv_len]
    return np.ascontiguousarray(k), np.ascontiguousarray(v)


def scatter_token_rows(pool, Hkv: int, blocks, slots, k_rows, v_rows, blk: int = 16, d: int = 128) -> None:
    """torch, in place: writes token rows k_rows / v_rows [n, Hkv, d] into slots[i] of blocks[i] of a
    device-layout pool tensor [M, 2*Hkv*blk*d] (any 16-bit dtype)."""
    M = pool.shape[0]
    kview = pool.view(M, 2, Hkv, d // 8, blk, 8)
    vview = pool.view(M, 2, Hkv, d, blk)
    n = blocks.shape[0]
    kview[blocks, 0, :, :, slots, :] = k_rows.reshape(n, Hkv, d // 8, 8)
    vview[blocks, 1, :, :, slots] = v_rows
