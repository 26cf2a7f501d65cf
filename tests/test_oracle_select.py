"""Pins for the oracle's selection functions (Section 2.1 Top-K sparsity; Section 6
threshold form).  None of these re-types the oracle's formula: they check invariants,
brute force, closed forms and hand-worked fixtures."""
import itertools
import os

import numpy as np
import pytest

from oracle import activeflow_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _mag(x):
    """Magnitude as a Python float (inf/nan free inputs only)."""
    return [abs(float(v)) for v in np.asarray(x, dtype=np.float16)]


def _pairwise_rule_holds(x, S):
    """Every chosen channel beats every dropped one: bigger |x|, or equal and lower index."""
    m = _mag(x)
    S = set(int(i) for i in S)
    for i in S:
        for j in range(len(m)):
            if j in S:
                continue
            if not (m[i] > m[j] or (m[i] == m[j] and i < j)):
                return False
    return True


def test_golden_worked_examples():
    rows = 0
    for line in open(os.path.join(GOLDEN, "topk_worked.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, xs, exp = [p.strip() for p in line.split(";")]
        x = np.array([float(v) for v in xs.split()], dtype=np.float16)
        expected = [int(v) for v in exp.split()]
        assert O.select_topk(x, int(k)).tolist() == expected
        rows += 1
    assert rows == 8


@pytest.mark.parametrize("seed", range(6))
def test_pairwise_invariant_with_many_ties(seed):
    g = np.random.default_rng(seed)
    n = int(g.integers(1, 513))
    # few distinct magnitudes -> ties at the k-th value are the common case
    x = (g.integers(-6, 7, size=n) * 0.25).astype(np.float16)
    for k in {0, 1, n // 3, n // 2, n - 1, n}:
        if not 0 <= k <= n:
            continue
        S = O.select_topk(x, k)
        assert S.dtype == np.int32 and len(S) == k
        assert np.all(np.diff(S) > 0)
        assert _pairwise_rule_holds(x, S)


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_small(seed):
    g = np.random.default_rng(100 + seed)
    n = int(g.integers(2, 11))
    x = (g.integers(-3, 4, size=n) * 0.5).astype(np.float16)
    m = _mag(x)
    for k in range(n + 1):
        valid = [c for c in itertools.combinations(range(n), k) if _pairwise_rule_holds(x, c)]
        assert len(valid) == 1                      # the rule defines a unique set
        S = O.select_topk(x, k)
        assert tuple(S.tolist()) == valid[0]
        best = max(sum(m[i] for i in c) for c in itertools.combinations(range(n), k))
        assert sum(m[i] for i in S) == best         # and it keeps the most magnitude


def test_distinct_magnitudes_closed_form():
    g = np.random.default_rng(7)
    n, k = 1000, 377
    ranks = g.permutation(n)                         # rank r -> magnitude (r+1)/16, all distinct
    sign = g.choice([-1.0, 1.0], size=n)
    x = ((ranks + 1) / 16.0 * sign).astype(np.float16)
    expected = np.sort(np.nonzero(ranks >= n - k)[0])
    assert O.select_topk(x, k).tolist() == expected.tolist()


def test_degenerate_inputs():
    n = 37
    ones = np.full(n, -1.5, dtype=np.float16)
    for k in (0, 1, 17, n):
        assert O.select_topk(ones, k).tolist() == list(range(k))
    z = np.array([0.0, -0.0, 0.0, -0.0], dtype=np.float16)
    assert O.select_topk(z, 2).tolist() == [0, 1]
    pm = np.array([1, -1, 2, -2, 3, -3], dtype=np.float16)
    assert O.select_topk(pm, 3).tolist() == [2, 4, 5]
    with pytest.raises(ValueError):
        O.select_topk(ones, n + 1)
    with pytest.raises(ValueError):
        O.select_topk(ones, -1)
    assert O.select_topk(np.zeros(0, dtype=np.float16), 0).tolist() == []


def test_subnormals_inf_nan_order():
    tiny = np.float16(6e-8)          # smallest fp16 subnormal
    x = np.array([0.0, tiny, -2 * tiny, 6.1e-5, np.inf, -np.inf, 65504.0, np.nan], dtype=np.float16)
    # order by magnitude key: nan > inf (idx 4 before 5) > 65504 > 6.1e-5 > 2*tiny > tiny > 0
    full = [7, 4, 5, 6, 3, 2, 1, 0]
    for k in range(len(full) + 1):
        assert O.select_topk(x, k).tolist() == sorted(full[:k])


def test_radix_digit_boundaries():
    """Magnitude keys that differ only in the low 7 bits or only in the high 8 bits."""
    keys = np.array([0x3C00, 0x3C7F, 0x3C80, 0x3BFF, 0x3C01, 0x3D00, 0x3C80, 0x0080, 0x007F],
                    dtype=np.uint16)
    x = keys.view(np.float16).copy()
    x[::2] = -x[::2]
    want = sorted(range(len(keys)), key=lambda j: (-int(keys[j]), j))
    for k in range(len(keys) + 1):
        assert O.select_topk(x, k).tolist() == sorted(want[:k])


def test_magnitude_key_is_monotone_in_abs():
    allbits = np.arange(0x7C01, dtype=np.uint16)          # every finite non-negative fp16 and +inf
    vals = allbits.view(np.float16).astype(np.float64)
    assert np.all(np.diff(vals) > 0)                      # bit order == value order
    neg = (allbits | np.uint16(0x8000)).view(np.float16)
    assert np.array_equal(O.magnitude_key(neg), allbits)


def test_keep_count():
    # Eq. 9: active share is (1 - sp)
    assert O.keep_count(4096, 50) == 2048
    assert O.keep_count(4096, 30) == 2868 and O.keep_count(4096, 70) == 1229
    assert O.keep_count(11008, 30) == 7706 and O.keep_count(11008, 70) == 3303
    assert O.keep_count(5120, 30) == 3584 and O.keep_count(13824, 70) == 4148
    assert O.keep_count(10, 0) == 10 and O.keep_count(10, 100) == 0


# ---------------------------------------------------------------- threshold form
def test_threshold_extremes_and_strictness():
    g = np.random.default_rng(3)
    x = g.standard_normal(300).astype(np.float16)
    assert O.select_threshold(x, -1.0).tolist() == list(range(300))
    assert O.select_threshold(x, np.inf).tolist() == []
    y = np.array([0.5, -0.5, 0.25, 1.0, -0.0], dtype=np.float16)
    assert O.select_threshold(y, 0.5).tolist() == [3]          # "above" is strict
    assert O.select_threshold(y, 0.0).tolist() == [0, 1, 2, 3]
    assert O.select_threshold(y, 0.4999).tolist() == [0, 1, 3]


def test_threshold_matches_topk_when_no_ties():
    g = np.random.default_rng(11)
    n = 777
    x = ((g.permutation(n) + 1) / 8.0 * g.choice([-1.0, 1.0], size=n)).astype(np.float16)
    mags = np.sort(np.abs(x.astype(np.float64)))[::-1]
    for k in (1, 100, 388, n - 1):
        t = mags[k]                                           # the (k+1)-th largest magnitude
        assert O.select_threshold(x, t).tolist() == O.select_topk(x, k).tolist()


def test_threshold_brute_force():
    g = np.random.default_rng(5)
    x = (g.integers(-8, 9, size=64) / 4.0).astype(np.float16)
    for t in (0.0, 0.25, 0.3, 1.0, 1.99, 2.0):
        exp = [j for j in range(64) if abs(float(x[j])) > t]
        assert O.select_threshold(x, t).tolist() == exp
