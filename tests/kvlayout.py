"""Test-side view of the library's documented KV-cache layout (include/ps.h):
K token-major  cache[b][0][g][t][x],  V dim-major  cache[b][1][g][x][t].
Pure index permutation between that layout and the oracle's private pool[M,2,Hkv,blk,d]."""
import numpy as np


def to_device_layout(pool: np.ndarray) -> np.ndarray:
    """oracle pool [M,2,Hkv,blk,d] (bf16 bits) -> flat uint16 [M, 2*Hkv*blk*d] in library layout."""
    M, two, Hkv, blk, d = pool.shape
    out = np.empty((M, 2, Hkv, blk * d), dtype=np.uint16)
    out[:, 0] = pool[:, 0].reshape(M, Hkv, blk * d)
    out[:, 1] = pool[:, 1].transpose(0, 1, 3, 2).reshape(M, Hkv, blk * d)
    return out.reshape(M, -1)


def from_device_layout(flat: np.ndarray, Hkv: int, blk: int = 16, d: int = 128) -> np.ndarray:
    M = flat.shape[0]
    v = flat.reshape(M, 2, Hkv, blk * d)
    pool = np.empty((M, 2, Hkv, blk, d), dtype=np.uint16)
    pool[:, 0] = v[:, 0].reshape(M, Hkv, blk, d)
    pool[:, 1] = v[:, 1].reshape(M, Hkv, d, blk).transpose(0, 1, 3, 2)
    return pool
