"""Trace mode of the preemption-heavy configuration (40 000-block pool, Qwen3-8B shapes, classes 1:2:4): the seeded
search finds an arrival rate at which about 30 % of the low-priority requests present are preempted per 100 rounds, and
reports the fraction it realised.  Host only; every decision is ps_form_batch's."""
import numpy as np

from paper_2512_12928_amd import preemption_trace as PT
from paper_2512_12928_amd import workloads as W


def test_search_lands_in_the_band_and_is_seeded():
    r = PT.tune_rate()
    print("rate %.1f requests/s: %.1f %% of the low-priority requests preempted per 100 rounds; probes %s"
          % (r["rate_per_s"], 100 * r["fraction"], r["probes"]))
    assert r["in_band"] and 0.25 <= r["fraction"] <= 0.35
    assert r["last"]["rounds"] == 1000 and r["last"]["evictions"] > 1000
    assert PT.tune_rate() == r                                   # same seed, same answer


def test_no_pressure_no_preemption():
    tr = W.make_trace(3, 300, rate_per_s=5.0, seed=1)
    r = PT.preempted_fraction(PT.default_cfg(), tr, 300)
    assert r["evictions"] == 0 and r["fraction"] == 0.0 and r["rounds"] == 300
