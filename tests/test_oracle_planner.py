"""Pins for the oracle's weight-cache simulator (Section 4.2) and cost model (Section 4.1):
the paper's worked cache example, hand-worked equations, limiting cases and scaling laws."""
import math
import os

import numpy as np
import pytest

from oracle import activeflow_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lfu_fixture():
    head, steps = {}, []
    for line in open(os.path.join(GOLDEN, "lfu_cache_worked.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if ";" in line:
            need, hits, loaded, ev, after = [[int(v) for v in p.split()] for p in line.split(";")]
            steps.append((need, hits[0], loaded[0], ev, after))
        else:
            k, *v = line.split()
            head[k] = [int(x) for x in v]
    return head, steps


def test_lfu_paper_worked_example():
    head, steps = _lfu_fixture()
    c = O.LfuCache(head["channels"][0], head["capacity"][0], head["initial"])
    ratios = []
    for need, hits, loaded, ev, after in steps:
        h, l, e = c.step(need)
        assert (h, l, sorted(e), sorted(c.cached)) == (hits, loaded, ev, after)
        ratios.append(h / len(need))
    assert ratios == [0.25, 0.75]
    assert (c.tokens, c.needed, c.hits, c.evictions) == (2, 8, 4, 4)


def test_lfu_limits_and_invariants():
    g = np.random.default_rng(0)
    n = 64
    streams = [np.sort(g.choice(n, size=24, replace=False)) for _ in range(40)]
    # no cache: never a hit; cache as large as the tensor: every channel misses exactly once
    c0, call = O.LfuCache(n, 0), O.LfuCache(n, n)
    seen, first_touches = set(), 0
    for s in streams:
        assert c0.step(s)[0] == 0
        new = [j for j in s if j not in seen]
        h, l, e = call.step(s)
        assert l == len(new) and e == []
        seen.update(int(j) for j in s)
    # any capacity: size bound, hits counted against the content before the step, counters = usage
    c = O.LfuCache(n, 20, initial=range(20))
    use = np.zeros(n, int)
    for s in streams:
        before = set(c.cached)
        h, l, e = c.step(s)
        use[s] += 1
        assert h == len(before & set(int(j) for j in s)) and h + l == len(s)
        assert len(c.cached) <= 20 and all(v in before for v in e)
        assert not (set(e) & set(int(j) for j in s))               # a needed channel never leaves
    assert c.count == use.tolist()


def test_lfu_learns_a_hot_set():
    """A fixed hot set that fits the cache is fully cached after it has been seen once, whatever
    cold channels pass by; the hit ratio then stays at the hot fraction or above."""
    g = np.random.default_rng(1)
    n, cap = 256, 64
    hot = np.arange(10, 10 + 48)
    c = O.LfuCache(n, cap, initial=range(190, 190 + cap))
    for t in range(30):
        cold = g.choice(np.setdiff1d(np.arange(n), hot), size=16, replace=False)
        h, l, _ = c.step(np.concatenate([hot, cold]))
        if t >= 1:
            assert set(hot.tolist()) <= c.cached and h >= len(hot)


def _cost_fixture():
    args, exp = {}, {}
    for line in open(os.path.join(GOLDEN, "cost_model_worked.txt")):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] == "expect":
            exp[p[1]] = float(p[2])
        else:
            args[p[0]] = float(p[1])
    return args, exp


def test_cost_model_hand_worked():
    args, exp = _cost_fixture()
    got = O.cost_model(**args)
    for k, v in exp.items():
        assert math.isclose(got[k], v, rel_tol=1e-12), k


def test_cost_model_limits_and_scaling():
    args, _ = _cost_fixture()
    base = O.cost_model(**args)
    # a perfect cache leaves only the two compute terms
    c = O.cost_model(**{**args, "hr": 1.0})
    assert c["T_load"] == c["T_onload"] == c["T_preload"] == 0.0
    assert math.isclose(c["T_decode"], 2 * c["T_comp"])
    # fully similar layers need no on-demand loads
    assert O.cost_model(**{**args, "si": 1.0})["T_onload"] == 0.0
    # all bandwidths x2 -> all times / 2, memory unchanged
    c = O.cost_model(**{**args, "bw_mem": 2 * args["bw_mem"], "bw_flash_small": 2 * args["bw_flash_small"],
                        "bw_flash_large": 2 * args["bw_flash_large"]})
    for k in ("T_load", "T_comp", "T_onload", "T_preload", "T_overlap", "T_decode"):
        assert math.isclose(c[k], base[k] / 2, rel_tol=1e-12)
    assert c["M"] == base["M"]
    # the group's memory and compute time are linear in N; on-demand loading does not depend on N
    c = O.cost_model(**{**args, "N": 8})
    assert math.isclose(c["M_cl"], 2 * base["M_cl"]) and math.isclose(c["T_comp"], 2 * base["T_comp"])
    assert c["T_onload"] == base["T_onload"]
    # the overlap term switches from preload-bound to compute-bound
    slow = O.cost_model(**{**args, "bw_mem": 100e6})
    assert math.isclose(slow["T_overlap"], slow["T_onload"] + slow["T_comp"]) and slow["T_preload"] < slow["T_comp"]


def test_plan_search_rules():
    kw = dict(M_kv=0.2e9, si=0.8, bw_mem=2000e9, bw_flash_small=1e9, bw_flash_large=4e9)
    hr = lambda frac: min(1.0, max(0.0, frac)) ** 0.5
    # the budget sets the sparsity; a budget at or above the model needs none
    sp, N, M_cache, c, visited = O.plan_search(M_max=4e9, S_m=8e9, S_l=0.25e9, hr_of_fraction=hr, **kw)
    assert math.isclose(sp, 0.5) and N >= 1 and c["M"] <= 4e9 * (1 + 1e-12)
    assert math.isclose(c["M"], 4e9)                                   # the cache takes what is left
    assert O.plan_search(M_max=9e9, S_m=8e9, S_l=0.25e9, hr_of_fraction=hr, **kw)[0] == 0.0
    # every visited N satisfies the budget, N grows by one, and the result is the best visited
    assert [v[0] for v in visited] == list(range(1, len(visited) + 1))
    assert all(v[3]["M"] <= 4e9 * (1 + 1e-12) for v in visited)
    assert c["T_decode"] == min(v[3]["T_decode"] for v in visited)
    # stop rule 1: preload hidden behind compute -> the search ends at that N
    fast = O.plan_search(M_max=4e9, S_m=8e9, S_l=0.25e9, hr_of_fraction=lambda f: 0.999,
                         M_kv=0.2e9, si=0.8, bw_mem=1e9, bw_flash_small=1e9, bw_flash_large=4e9)
    assert len(fast[4]) == 1 and fast[4][0][3]["T_preload"] <= fast[4][0][3]["T_comp"]
    # stop rule 2: budget exhausted -> no N whose group does not fit
    last = visited[-1]
    assert last[3]["M_cl"] + 0.2e9 <= 4e9
    # stop rule 3: a large min_gain ends the search after the second candidate
    short = O.plan_search(M_max=4e9, S_m=8e9, S_l=0.25e9, hr_of_fraction=hr, min_gain=1e9, **kw)
    assert len(short[4]) == 2
