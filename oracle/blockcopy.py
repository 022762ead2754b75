"""Oracle C: KV block offload / reload as plain block copies.

TEST INFRASTRUCTURE ONLY.  Sec. 4.3 ("Asynchronous Offloading", "Pipelined Reloading",
"Adaptive Copy-Budget Control") moves whole KV blocks between the device pool and host
memory, at most a budgeted number per step, consumed in queue order.  The result has a
plain definition: the first min(n, budget) listed blocks are copied byte for byte and
nothing else changes.

Pools are 2-D uint8 arrays [n_blocks, block_bytes].
"""
from __future__ import annotations

import numpy as np


def n_moved(n: int, copy_budget: int) -> int:
    """A negative budget means unlimited."""
    return n if copy_budget < 0 else min(n, copy_budget)


def swap_out(dev_pool: np.ndarray, host_pool: np.ndarray, dev_ids, host_slots, copy_budget: int = -1) -> int:
    """host[host_slots[k]] <- dev[dev_ids[k]] for the first min(n, budget) entries, in order."""
    m = n_moved(len(dev_ids), copy_budget)
    for k in range(m):
        host_pool[int(host_slots[k])] = dev_pool[int(dev_ids[k])]
    return m


def swap_in(host_pool: np.ndarray, dev_pool: np.ndarray, host_slots, dev_ids, copy_budget: int = -1) -> int:
    """dev[dev_ids[k]] <- host[host_slots[k]] for the first min(n, budget) entries, in order."""
    m = n_moved(len(dev_ids), copy_budget)
    for k in range(m):
        dev_pool[int(dev_ids[k])] = host_pool[int(host_slots[k])]
    return m
