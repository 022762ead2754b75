"""Pins for oracle C (KV block offload/reload as plain copies).  CPU only."""
import numpy as np

from oracle import blockcopy as C


def pools(seed=0, nd=12, nh=9, bb=64):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, (nd, bb), dtype=np.uint8), rng.integers(0, 256, (nh, bb), dtype=np.uint8)


def test_round_trip_identity_to_other_blocks():
    dev, host = pools()
    dev0 = dev.copy()
    assert C.swap_out(dev, host, [3, 7, 1], [2, 0, 8]) == 3
    assert C.swap_in(host, dev, [2, 0, 8], [5, 6, 9]) == 3
    assert np.array_equal(dev[[5, 6, 9]], dev0[[3, 7, 1]])
    untouched = [i for i in range(12) if i not in (5, 6, 9)]
    assert np.array_equal(dev[untouched], dev0[untouched])


def test_budget_moves_exactly_the_first_k_in_order():
    for budget, want in [(0, 0), (2, 2), (3, 3), (10, 3), (-1, 3)]:
        dev, host = pools(1)
        host0 = host.copy()
        n = C.swap_out(dev, host, [4, 5, 6], [1, 2, 3], budget)
        assert n == want
        for k in range(3):
            src = dev[4 + k] if k < want else host0[1 + k]
            assert np.array_equal(host[1 + k], src)
        rest = [0, 4, 5, 6, 7, 8]
        assert np.array_equal(host[rest], host0[rest])


def test_swap_in_budget_and_untouched_bytes():
    dev, host = pools(2)
    dev0 = dev.copy()
    assert C.swap_in(host, dev, [8, 7, 6, 5], [0, 11, 3, 4], 2) == 2
    assert np.array_equal(dev[0], host[8]) and np.array_equal(dev[11], host[7])
    rest = [i for i in range(12) if i not in (0, 11)]
    assert np.array_equal(dev[rest], dev0[rest])


def test_empty_list_is_a_successful_noop():
    dev, host = pools(3)
    d0, h0 = dev.copy(), host.copy()
    assert C.swap_out(dev, host, [], []) == 0 and C.swap_in(host, dev, [], []) == 0
    assert np.array_equal(dev, d0) and np.array_equal(host, h0)
