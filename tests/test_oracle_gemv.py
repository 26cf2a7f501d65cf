"""Pins for the oracle's sparse GEMV (Section 4, operation C), 4-bit weights (Section 6,
Section 7.1), the small-batch union and the overlap metric (Section 3).  Expected values
come from exact integer arithmetic, scalar loops, closed forms or hand-worked fixtures,
never from the oracle's own matmul."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import activeflow_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _scalar_gemv(W, x, idx):
    """Triple-loop definition with exactly rounded sums (math.fsum)."""
    W = np.asarray(W, dtype=np.float16)
    keep = set(int(j) for j in idx)
    return [math.fsum(float(W[o, j]) * float(x[j]) for j in range(W.shape[1]) if j in keep)
            for o in range(W.shape[0])]


def _exact_gemv(W, x, idx):
    """Rational arithmetic: no rounding anywhere."""
    keep = set(int(j) for j in idx)
    return [sum((Fraction(float(W[o, j])) * Fraction(float(x[j])) for j in range(W.shape[1]) if j in keep),
                Fraction(0)) for o in range(W.shape[0])]


def test_all_masks_brute_force():
    g = np.random.default_rng(0)
    out, n = 7, 9
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    x = g.laplace(size=n).astype(np.float16)
    for bits in range(1 << n):
        idx = [j for j in range(n) if bits >> j & 1]
        got = O.sparse_gemv(W, x, np.array(idx, dtype=np.int32))
        exp = _scalar_gemv(W, x, idx)
        assert np.allclose(got, exp, rtol=1e-13, atol=1e-18)


def test_exact_rational_reference():
    g = np.random.default_rng(1)
    out, n = 5, 40
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    x = (g.laplace(size=n) * 3).astype(np.float16)
    idx = np.sort(g.choice(n, size=17, replace=False)).astype(np.int32)
    got = O.sparse_gemv(W, x, idx)
    exact = _exact_gemv(W, x, idx)
    scale = sum(abs(float(W[0, j]) * float(x[j])) for j in range(n))
    for o in range(out):
        assert abs(Fraction(float(got[o])) - exact[o]) <= Fraction(scale) * Fraction(1, 2 ** 45)


def test_integer_inputs_are_exact():
    g = np.random.default_rng(2)
    out, n = 33, 65                                       # non-square: a transposed operand cannot pass
    W = g.integers(-8, 9, size=(out, n)).astype(np.float16)
    x = g.integers(-8, 9, size=n).astype(np.float16)
    idx = np.sort(g.choice(n, size=30, replace=False)).astype(np.int32)
    exp = [sum(int(W[o, j]) * int(x[j]) for j in idx) for o in range(out)]
    assert O.sparse_gemv(W, x, idx).tolist() == [float(v) for v in exp]


def test_sparsity_zero_is_dense_and_empty_is_zero():
    g = np.random.default_rng(3)
    out, n = 12, 20
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    x = g.laplace(size=n).astype(np.float16)
    dense = _scalar_gemv(W, x, range(n))
    assert np.allclose(O.sparse_gemv(W, x, np.arange(n, dtype=np.int32)), dense, rtol=1e-13)
    assert np.all(O.sparse_gemv(W, x, np.zeros(0, dtype=np.int32)) == 0)


def test_one_hot_identity_ones_additivity():
    g = np.random.default_rng(4)
    out, n = 10, 16
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    x = g.laplace(size=n).astype(np.float16)
    for j in (0, 5, n - 1):
        y = O.sparse_gemv(W, x, np.array([j], dtype=np.int32))
        assert np.array_equal(y, W[:, j].astype(np.float64) * float(x[j]))
    idx = np.array([1, 4, 6, 9, 15], dtype=np.int32)
    eye = np.eye(n, dtype=np.float16)
    m = np.zeros(n); m[idx] = 1
    assert np.array_equal(O.sparse_gemv(eye, x, idx), x.astype(np.float64) * m)
    ones = np.ones((3, n), dtype=np.float16)
    s = math.fsum(float(x[j]) for j in idx)
    assert np.allclose(O.sparse_gemv(ones, x, idx), [s] * 3, rtol=1e-14)
    a, b = idx[:2], idx[2:]
    assert np.allclose(O.sparse_gemv(W, x, a) + O.sparse_gemv(W, x, b), O.sparse_gemv(W, x, idx), rtol=1e-13, atol=1e-18)


# ----------------------------------------------------------------------- 4-bit
def test_q4_golden_group():
    rows = [l for l in open(os.path.join(GOLDEN, "q4_worked.txt")) if l.strip() and not l.startswith("#")]
    w64 = np.array([float(v) for v in rows[0].split()])
    q_exp = np.array([int(v) for v in rows[1].split()])
    W = (w64 / 64.0).astype(np.float16).reshape(1, 32)
    assert np.array_equal(W[0].astype(np.float64) * 64.0, w64)          # the fixture is fp16-exact
    nib, s = O.quantize_q4_g32(W)
    assert s.shape == (1, 1) and float(s[0, 0]) == 1.0 / 64.0
    assert np.array_equal(nib[0].astype(int) - 8, q_exp)
    assert np.array_equal(O.dequant_q4_g32(nib, s)[0], q_exp / 64.0)


def test_q4_error_bound_and_range():
    g = np.random.default_rng(5)
    out, n = 24, 96
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    nib, s = O.quantize_q4_g32(W)
    assert nib.dtype == np.uint8 and nib.min() >= 1 and nib.max() <= 15
    assert s.shape == (n // 32, out) and s.dtype == np.float16
    deq = O.dequant_q4_g32(nib, s)
    sfull = np.repeat(s.astype(np.float64).T, 32, axis=1)
    # rounding to the nearest step costs at most half a step; the scale's own fp16 rounding
    # (relative 2^-11) can push the largest element just past 7 steps before the clamp
    assert np.all(np.abs(W.astype(np.float64) - deq) <= 0.5 * sfull * (1 + 1e-6) + 7 * sfull * 2.0 ** -11)
    # each group's largest element maps to +-7
    a = np.abs(W.astype(np.float64)).reshape(out, n // 32, 32)
    q = (nib.astype(int) - 8).reshape(out, n // 32, 32)
    assert np.all(np.abs(np.take_along_axis(q, a.argmax(axis=2)[..., None], axis=2)) == 7)


def test_q4_special_groups():
    W = np.zeros((2, 64), dtype=np.float16)
    W[1, 40] = -0.75                                      # a single extreme in one group
    nib, s = O.quantize_q4_g32(W)
    assert np.all(nib[0] == 8) and np.all(s[:, 0] == 0)
    assert float(s[0, 1]) == 0 and nib[1, 40] == 1 and np.all(np.delete(nib[1], 40) == 8)
    assert float(s[1, 1]) == float(np.float16(np.float32(0.75) / np.float32(7)))
    deq = O.dequant_q4_g32(nib, s)
    assert abs(deq[1, 40] + 0.75) <= 0.75 * 2.0 ** -10 and np.count_nonzero(deq) == 1


def test_q4_pack_layout_and_roundtrip():
    g = np.random.default_rng(6)
    out, n = 16, 32
    nib = g.integers(1, 16, size=(out, n)).astype(np.uint8)
    p = O.pack_q4(nib)
    assert p.shape == (n, out // 2)
    for j in (0, 7, 31):
        for i in (0, 3, 7):
            assert p[j, i] == int(nib[2 * i, j]) | (int(nib[2 * i + 1, j]) << 4)
    assert np.array_equal(O.unpack_q4(p, out), nib)


def test_q4_gemv_against_scalar_loop():
    g = np.random.default_rng(7)
    out, n = 6, 64
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    x = g.laplace(size=n).astype(np.float16)
    nib, s = O.quantize_q4_g32(W)
    idx = np.sort(g.choice(n, size=29, replace=False)).astype(np.int32)
    exp = [math.fsum((int(nib[o, j]) - 8) * float(s[j // 32, o]) * float(x[j]) for j in idx) for o in range(out)]
    assert np.allclose(O.sparse_gemv_q4(nib, s, x, idx), exp, rtol=1e-12, atol=1e-18)


# ------------------------------------------------- 4-bit, channel-local groups
def test_q4_cl_golden_group():
    """The hand-worked group of the fixture, laid along the output dim of one input channel."""
    rows = [l for l in open(os.path.join(GOLDEN, "q4_worked.txt")) if l.strip() and not l.startswith("#")]
    w64 = np.array([float(v) for v in rows[0].split()])
    q_exp = np.array([int(v) for v in rows[1].split()])
    W = (w64 / 64.0).astype(np.float16).reshape(32, 1)                   # [out = 32][in = 1]
    nib, s = O.quantize_q4_cl(W)
    assert s.shape == (1, 1) and float(s[0, 0]) == 1.0 / 64.0
    assert np.array_equal(nib[:, 0].astype(int) - 8, q_exp)
    assert np.array_equal(O.dequant_q4_cl(nib, s)[:, 0], q_exp / 64.0)


def test_q4_cl_is_g32_of_the_transpose():
    """Grouping 32 output columns of channel j is grouping 32 'input channels' of the
    transposed matrix: the two quantisers must agree through that relabelling."""
    g = np.random.default_rng(15)
    out, n = 64, 24
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    nib_cl, s_cl = O.quantize_q4_cl(W)
    nib_t, s_t = O.quantize_q4_g32(np.ascontiguousarray(W.T))           # [in][out] as if out-major
    assert np.array_equal(nib_cl, nib_t.T)
    assert np.array_equal(s_cl, s_t.T)                                   # [in][out/32] vs [out/32][in]
    assert np.array_equal(O.dequant_q4_cl(nib_cl, s_cl), O.dequant_q4_g32(nib_t, s_t).T)


def test_q4_cl_error_bound_and_gemv_scalar_loop():
    g = np.random.default_rng(16)
    out, n = 96, 40
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    nib, s = O.quantize_q4_cl(W)
    assert nib.min() >= 1 and nib.max() <= 15 and s.shape == (n, out // 32) and s.dtype == np.float16
    deq = O.dequant_q4_cl(nib, s)
    sfull = np.repeat(s.astype(np.float64), 32, axis=1).T
    assert np.all(np.abs(W.astype(np.float64) - deq) <= 0.5 * sfull * (1 + 1e-6) + 7 * sfull * 2.0 ** -11)
    x = g.laplace(size=n).astype(np.float16)
    idx = np.sort(g.choice(n, size=17, replace=False)).astype(np.int32)
    exp = [math.fsum((int(nib[o, j]) - 8) * float(s[j, o // 32]) * float(x[j]) for j in idx) for o in range(out)]
    assert np.allclose(O.sparse_gemv_q4_cl(nib, s, x, idx), exp, rtol=1e-12, atol=1e-18)
    # a channel's scales depend on that channel alone (what makes its bytes self-contained)
    W2 = W.copy(); W2[:, 5] *= np.float16(3.0)
    nib2, s2 = O.quantize_q4_cl(W2)
    keep = np.arange(n) != 5
    assert np.array_equal(s2[keep], s[keep]) and np.array_equal(nib2[:, keep], nib[:, keep])


# ----------------------------------------------------------------------- union
def test_union_small_batch():
    g = np.random.default_rng(8)
    out, n, B, k = 5, 24, 3, 9
    W = (g.standard_normal((out, n)) * 0.02).astype(np.float16)
    X = g.laplace(size=(B, n)).astype(np.float16)
    idx_b = [np.sort(g.choice(n, size=k, replace=False)).astype(np.int32) for _ in range(B)]
    U = O.union_indices(idx_b)
    assert U.tolist() == sorted(set().union(*[set(i.tolist()) for i in idx_b]))
    Y = O.union_gemv(W, X, idx_b)
    for b in range(B):
        assert np.allclose(Y[b], _scalar_gemv(W, X[b], idx_b[b]), rtol=1e-13, atol=1e-18)
    # identical tokens: the union is one token's set
    assert O.union_indices([idx_b[0]] * 4).tolist() == idx_b[0].tolist()
    assert O.union_indices([]).tolist() == []
    # B = 1 is the single-token product
    assert np.array_equal(O.union_gemv(W, X[:1], idx_b[:1])[0], O.sparse_gemv(W, X[0], idx_b[0]))


# --------------------------------------------------------------------- overlap
def test_overlap_metric():
    a = np.array([1, 3, 5, 7], dtype=np.int32)
    assert O.overlap(a, a) == 1.0
    assert O.overlap(a, np.array([0, 2, 4, 6])) == 0.0
    assert O.overlap(a, np.array([1, 2, 3, 4])) == 0.5
    assert O.overlap(a, np.zeros(0, dtype=np.int32)) == 1.0
    # independent random k-subsets of n overlap k/n on average (hypergeometric mean)
    g = np.random.default_rng(9)
    n, k, trials = 400, 100, 300
    m = np.mean([O.overlap(g.choice(n, k, replace=False), g.choice(n, k, replace=False)) for _ in range(trials)])
    sd = math.sqrt(k / n * (1 - k / n) * (n - k) / (n - 1) / k / trials)
    assert abs(m - k / n) < 5 * sd


def test_rel_err_measure():
    ref = np.array([1.0, -2.0, 0.0, 4.0])
    assert O.rel_err(ref, ref) == 0.0
    got = ref + np.array([1e-3, 0, 0, 0])
    assert abs(O.rel_err(got, ref) - 1e-3) < 1e-12
    # an element at zero is judged against 1 % of the vector's rms
    rms = math.sqrt((1 + 4 + 16) / 4)
    got = ref + np.array([0, 0, 1e-4, 0])
    assert abs(O.rel_err(got, ref) - 1e-4 / (0.01 * rms)) < 1e-9
