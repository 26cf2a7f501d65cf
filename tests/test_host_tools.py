"""Host-side tools of the library (no GPU): the weight-cache simulator and the cost model,
compared with the oracle on the same inputs.  Integer results must be identical; the cost model
is the same double arithmetic on both sides and is compared to 1e-12."""
import math

import numpy as np
import pytest

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B


def test_lfu_paper_example_through_the_abi():
    c = B.LfuCache(8, 4, [0, 2, 3, 5])
    assert c.step([0, 1, 4, 6]) == (1, 3, [2, 3, 5]) and c.cached() == [0, 1, 4, 6]
    assert c.step([0, 4, 6, 7]) == (3, 1, [1]) and c.cached() == [0, 4, 6, 7]
    assert c.stats() == {"tokens": 2, "needed": 8, "hits": 4, "evictions": 4}


@pytest.mark.parametrize("n,cap,k,seed", [(64, 16, 20, 0), (64, 0, 9, 1), (64, 64, 30, 2), (512, 200, 256, 3),
                                          (1024, 256, 512, 4), (100, 99, 50, 5), (33, 5, 33, 6)])
def test_lfu_matches_oracle_on_random_and_structured_streams(n, cap, k, seed):
    g = np.random.default_rng(seed)
    init = sorted(g.choice(n, size=g.integers(0, cap + 1), replace=False).tolist()) if cap else []
    a, b = B.LfuCache(n, cap, init), O.LfuCache(n, cap, init)
    # skewed popularity (a hot set exists), as activation magnitudes have per-channel scales
    p = g.pareto(1.5, size=n) + 0.05
    p /= p.sum()
    for t in range(40):
        kk = k if t % 7 else max(1, k // 3)
        idx = np.sort(g.choice(n, size=kk, replace=False, p=p))
        ha, la, ea = a.step(idx.tolist())
        hb, lb, eb = b.step(idx)
        assert (ha, la, ea) == (hb, lb, eb), t
        assert a.cached() == sorted(b.cached)
    s = a.stats()
    assert (s["tokens"], s["needed"], s["hits"], s["evictions"]) == (b.tokens, b.needed, b.hits, b.evictions)


def test_lfu_on_the_synthetic_activation_stream():
    """Index sets as the hot path emits them (top-k of the synthetic activations)."""
    n = 1024
    scales = S.channel_scales(0, n, "lfu")
    a, b = B.LfuCache(n, n // 2, list(range(n // 2))), O.LfuCache(n, n // 2, range(n // 2))
    for tok in range(16):
        idx = O.select_topk(S.activation(0, scales, "lfu", tok), n // 2)
        assert a.step(idx.tolist()) == b.step(idx)
    assert a.stats()["hits"] == b.hits and a.stats()["hits"] / a.stats()["needed"] > 0.5


def test_lfu_argument_errors():
    with pytest.raises(B.AfError):
        B.LfuCache(8, 2, [0, 1, 2])                  # more initial channels than slots
    with pytest.raises(B.AfError):
        B.LfuCache(8, 4, [0, 0])                     # duplicate
    c = B.LfuCache(8, 4)
    with pytest.raises(B.AfError):
        c.step([3, 1])                               # not ascending
    with pytest.raises(B.AfError):
        c.step([8])                                  # out of range
    assert c.step([]) == (0, 0, [])


def test_cost_model_matches_oracle():
    g = np.random.default_rng(0)
    for _ in range(50):
        kw = dict(sp=g.uniform(0, 0.95), hr=g.uniform(0, 1), si=g.uniform(0, 1), bw_mem=g.uniform(1e9, 8e12),
                  bw_flash_small=g.uniform(1e8, 1e10), bw_flash_large=g.uniform(1e9, 6e10),
                  S_l=g.uniform(1e8, 2e9), N=float(g.integers(1, 9)), M_cache=g.uniform(0, 1e10), M_kv=g.uniform(0, 1e9))
        got, ref = B.cost_eval(**kw), O.cost_model(**kw)
        for k in ref:
            assert math.isclose(got[k], ref[k], rel_tol=1e-12, abs_tol=0.0), k
    with pytest.raises(B.AfError):
        B.cost_eval(sp=0.5, hr=0.5, si=0.5, bw_mem=0.0, bw_flash_small=1.0, bw_flash_large=1.0, S_l=1.0, N=1.0,
                    M_cache=0.0, M_kv=0.0)


def test_plan_search_matches_oracle():
    pts = [(0.0, 0.0), (0.1, 0.45), (0.25, 0.7), (0.5, 0.82), (1.0, 1.0)]
    hr = lambda f: float(np.interp(f, [p[0] for p in pts], [p[1] for p in pts]))
    g = np.random.default_rng(1)
    for _ in range(40):
        S_l = g.uniform(1e8, 8e8)
        S_m = S_l * g.integers(8, 81)
        kw = dict(M_max=S_m * g.uniform(0.15, 1.2), S_m=S_m, S_l=S_l, M_kv=S_l * g.uniform(0, 2), si=g.uniform(0.5, 0.95),
                  bw_mem=g.choice([50e9, 8e12]), bw_flash_small=g.uniform(5e8, 2e10), bw_flash_large=g.uniform(2e9, 6e10))
        mg = float(g.choice([0.0, 1e-4, 1e-2]))
        got = B.plan_search(hr_points=pts, n_max=32, min_gain=mg, **kw)
        sp, N, M_cache, c, visited = O.plan_search(hr_of_fraction=hr, n_max=32, min_gain=mg, **kw)
        assert math.isclose(got["sp"], sp, rel_tol=1e-12, abs_tol=1e-15)
        assert got["N"] == N and got["visited"] == len(visited)
        if N:
            assert math.isclose(got["M_cache"], M_cache, rel_tol=1e-9, abs_tol=1e-3)
            for k in c:
                assert math.isclose(got["cost"][k], c[k], rel_tol=1e-9), k
