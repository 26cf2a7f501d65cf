"""GPU parity: threshold calibration (af_calib_*) against the oracle.  A calibrated
threshold is an fp16 magnitude chosen by counting, so the comparison is exact."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import activeflow_oracle as O
from gpu_util import ctx, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu

LEVELS = [0, 1, 30, 50, 70, 90, 99, 100]


def _calibrate(ctx, samples, levels):
    hist = ctx.calib_hist()
    for s in samples:
        if len(s):
            ctx.calib_accumulate(to_dev(np.asarray(s, dtype=np.float16)), hist)
    t = ctx.calib_thresholds(hist, levels)
    ctx.synchronize()
    return to_host(t), to_host(hist)


def test_synthetic_stream_all_levels(ctx):
    n = 4096
    scales = S.channel_scales(0, n, "calib")
    samples = [S.activation(0, scales, "calib", tok) for tok in range(24)]
    got, hist = _calibrate(ctx, samples, LEVELS)
    assert int(hist.astype(np.int64).sum()) == n * len(samples)
    for l, sp in enumerate(LEVELS):
        assert float(got[l]) == O.calibrate_threshold(samples, sp), sp


@pytest.mark.parametrize("seed", range(4))
def test_ragged_vectors_with_ties_and_specials(ctx, seed):
    g = np.random.default_rng(seed)
    samples = []
    for _ in range(int(g.integers(1, 7))):
        n = int(g.integers(1, 3000))
        x = (g.integers(-9, 10, size=n) * 0.25).astype(np.float16)          # heavy ties
        x[g.integers(0, n, size=max(1, n // 50))] = np.float16(np.nan)      # never pooled
        x[g.integers(0, n)] = np.float16(np.inf)
        x[g.integers(0, n)] = np.float16(-6e-8)                             # subnormal
        samples.append(x)
    got, _ = _calibrate(ctx, samples, LEVELS)
    for l, sp in enumerate(LEVELS):
        assert float(got[l]) == O.calibrate_threshold(samples, sp), (seed, sp)


def test_empty_pool_and_single_value(ctx):
    got, hist = _calibrate(ctx, [np.zeros(0, np.float16)], [0, 50, 100])
    assert hist.sum() == 0 and got.tolist() == [-1.0, -1.0, -1.0]
    got, _ = _calibrate(ctx, [np.array([-3.0], np.float16)], [0, 50, 100])
    assert got.tolist() == [O.calibrate_threshold([np.array([-3.0], np.float16)], sp) for sp in (0, 50, 100)]


def test_maximum_length_vector(ctx):
    x = S.activation(3, S.channel_scales(3, 32768, "calib-max"), "calib-max", 0)
    got, _ = _calibrate(ctx, [x], [50, 70])
    assert [float(v) for v in got] == [O.calibrate_threshold([x], sp) for sp in (50, 70)]


def test_calibrated_threshold_selects_like_the_oracle_says(ctx):
    """The threshold found on the GPU, fed to the GPU's threshold selection, keeps what the
    oracle keeps with the oracle's threshold."""
    n = 11008
    scales = S.channel_scales(1, n, "calib2")
    samples = [S.activation(1, scales, "calib2", tok) for tok in range(8)]
    got, _ = _calibrate(ctx, samples, [50])
    held = S.activation(1, scales, "calib2", 99)
    idx, cnt = ctx.select_threshold(to_dev(held), float(got[0]))
    ctx.synchronize()
    c = int(to_host(cnt)[0])
    ref = O.select_threshold(held, O.calibrate_threshold(samples, 50))
    assert np.array_equal(to_host(idx)[:c], ref)
    assert abs(c / n - 0.5) < 0.05


def test_layer_taps_feed_the_four_histograms(ctx):
    from paper_2504_08378_amd import binding as B, model as M
    shape = S.MODEL_SHAPES["tiny_gqa"]
    w = S.layer_weights(0, shape, 0)
    lay = M.DeviceLayer(ctx, shape, w)
    kv_len, cap = 5, 8
    K, V = S.kv_cache(0, shape.n_kv_heads, cap, shape.head_dim, kv_len, shape.name, 0)
    st = M.DeviceStack(ctx, shape, [lay], [(K, V)], cap)
    widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
    ks = tuple(O.keep_count(n, 50) for n in widths)
    hists = [ctx.calib_hist() for _ in range(4)]
    xs = [[] for _ in range(4)]
    scales = S.channel_scales(0, shape.d_model, shape.name)
    for tok in range(3):
        h = to_dev(S.activation(0, scales, "hidden", tok))
        st.layer(0, h, st.hidden_out, kv_len, kv_len, M.select_cfg(B.AF_SEL_TOPK, ks))
        ctx.calib_accumulate_layer(st.cfg, hists)
        ctx.synchronize()
        for p, tap in enumerate((0, 2, 4, 6)):
            xs[p].append(to_host(ctx.layer_tap(tap, widths[p])))
    for p in range(4):
        t = ctx.calib_thresholds(hists[p], [30, 50, 70])
        ctx.synchronize()
        # expected from the very vectors the layer produced (fetched through the taps)
        assert [float(v) for v in to_host(t)] == [O.calibrate_threshold(xs[p], sp) for sp in (30, 50, 70)]
