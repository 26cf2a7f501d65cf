"""Pins for the oracle's threshold calibration (Section 6: one preloaded activation
threshold per sparsity level).  Checked against the counting definition by brute force,
against a closed-form quantile, against the top-k rule it stands for, and on held-out
draws of the synthetic activation recipe."""
import math

import numpy as np
import pytest

import synth_inputs as S
from oracle import activeflow_oracle as O


def _pool(samples):
    return [abs(float(v)) for s in samples for v in np.asarray(s, dtype=np.float16)]


@pytest.mark.parametrize("seed", range(5))
def test_counting_definition_brute_force(seed):
    """t is a pooled magnitude with at most m values above it and more than m at or above
    it: counted with Python floats, no sort."""
    g = np.random.default_rng(seed)
    samples = [(g.integers(-20, 21, size=int(g.integers(1, 40))) * 0.125).astype(np.float16)
               for _ in range(int(g.integers(1, 6)))]
    pool = _pool(samples)
    N = len(pool)
    for sp in (0, 10, 37, 50, 90, 99, 100):
        m = N - (sp * N) // 100
        t = O.calibrate_threshold(samples, sp)
        if m >= N:
            assert t == -1.0
            continue
        assert t in pool
        above = sum(v > t for v in pool)
        at_or_above = sum(v >= t for v in pool)
        assert above <= m < at_or_above


def test_matches_topk_on_the_pooled_sample_without_ties():
    g = np.random.default_rng(11)
    # distinct magnitudes: a permutation of 1..N scaled into fp16's exact range
    N = 600
    vals = (g.permutation(N) + 1).astype(np.float16) * g.choice([-1.0, 1.0], size=N).astype(np.float16)
    samples = [vals[:100], vals[100:350], vals[350:]]
    for sp in (25, 50, 80):
        t = O.calibrate_threshold(samples, sp)
        m = O.keep_count(N, sp)
        assert O.select_threshold(vals, t).tolist() == O.select_topk(vals, m).tolist()


def test_closed_form_quantile_of_an_exponential():
    """|x| ~ Exp(1): P(|x| > t) = exp(-t), so the threshold for keep fraction q is -ln q.
    Sample quantile error: sd = sqrt(q(1-q)/N) / pdf(t) = sqrt((1-q)/(qN))."""
    g = np.random.default_rng(5)
    N = 400_000
    x = g.exponential(1.0, size=N) * g.choice([-1.0, 1.0], size=N)
    samples = np.array_split(x.astype(np.float16), 50)
    for sp in (30, 50, 70, 90):
        q = 1.0 - sp / 100.0
        t = O.calibrate_threshold(samples, sp)
        sd = math.sqrt((1 - q) / (q * N))
        fp16_step = 2.0 ** (math.floor(math.log2(-math.log(q))) - 10)
        assert abs(t - (-math.log(q))) < 5 * sd + fp16_step


def test_edges():
    x = np.array([0.0, -0.0, 1.0, -2.0, 3.0], dtype=np.float16)
    assert O.calibrate_threshold([x], 0) == -1.0                   # keep everything, zeros too
    assert len(O.select_threshold(x, O.calibrate_threshold([x], 0))) == 5
    t = O.calibrate_threshold([x], 100)                             # keep nothing
    assert t == 3.0 and len(O.select_threshold(x, t)) == 0
    assert O.calibrate_threshold([], 50) == -1.0
    # NaN never enters the pool; Inf is a magnitude like any other
    y = np.array([np.nan, np.inf, 1.0, 2.0], dtype=np.float16)
    assert O.calibrate_threshold([y], 34) == 1.0                    # N = 3, m = 2 -> third largest
    # ties at the boundary: the strict rule keeps fewer than m
    z = np.array([1.0, 1.0, 1.0, 2.0], dtype=np.float16)
    t = O.calibrate_threshold([z], 50)                              # m = 2 -> third largest = 1
    assert t == 1.0 and O.select_threshold(z, t).tolist() == [3]


@pytest.mark.parametrize("sp", [30, 50, 70])
def test_held_out_keep_rate_on_the_synthetic_recipe(sp):
    """Calibrated on 64 tokens of the synthetic activation stream, the threshold keeps the
    target fraction of held-out tokens' channels within sampling error.  Channels are not
    identically distributed (per-channel scales), so the per-token count is a sum of
    independent Bernoullis: its variance is at most n q (1 - q)."""
    n = 4096
    scales = S.channel_scales(0, n, "calib-pin")
    cal = [S.activation(0, scales, "calib-pin", tok) for tok in range(64)]
    t = O.calibrate_threshold(cal, sp)
    q = 1.0 - sp / 100.0
    held = [S.activation(0, scales, "calib-pin", tok) for tok in range(1000, 1064)]
    kept = sum(len(O.select_threshold(x, t)) for x in held)
    total = n * len(held)
    # both the calibration quantile and the held-out count fluctuate: two binomial terms
    sd = math.sqrt(2 * q * (1 - q) / total)
    assert abs(kept / total - q) < 5 * sd + 1e-3
