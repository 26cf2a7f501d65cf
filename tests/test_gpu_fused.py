"""GPU parity: af_select_gemv_f16 (producer + selection + gathered GEMV in one launch)
against the oracle's separate steps.  The selection input of each case is computed by the
oracle's own arithmetic on the same fp16 bits, so index sets are compared bit-for-bit where
the producer is the identity; behind a norm / SwiGLU producer the GPU's own x is used to
check the set from the definition and the oracle's set may differ only at the k-th magnitude."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B
from gpu_util import ctx, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _wx(out, n, seed):
    W = S.weight_matrix(seed, out, n, "fused", out, n)
    x = S.activation(seed, S.channel_scales(seed, n, "fused"), "fused", 0)
    return W, x


def _run(ctx, Wt, src, n, **kw):
    xo = torch.zeros(n, dtype=torch.float16, device="cuda")
    io = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    co = torch.zeros(1, dtype=torch.int32, device="cuda")
    y = ctx.select_gemv_f16(Wt, src, x_out=xo, idx_out=io, count_out=co, **kw)
    ctx.synchronize()
    c = int(to_host(co)[0])
    return to_host(y), to_host(xo), to_host(io)[:c], c


@pytest.mark.parametrize("out,n,k", [(136, 64, 32), (520, 1000, 377), (4096, 4096, 2048),
                                     (1032, 11008, 5504), (2056, 5120, 1536), (264, 28672, 14336)])
def test_identity_producer_topk_is_bit_exact(ctx, out, n, k):
    W, x = _wx(out, n, out + n)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    y, _, idx, c = _run(ctx, Wt, to_dev(x), n, sel_mode=B.AF_SEL_TOPK, k=k, y_kind=B.AF_F32)
    ref_idx = O.select_topk(x, k)
    assert c == k and np.array_equal(idx, ref_idx)
    assert O.rel_err(y, O.sparse_gemv(W, x, ref_idx)) <= 1e-4


def test_threshold_dense_and_empty(ctx):
    W, x = _wx(520, 2048, 5)
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x)
    mags = np.sort(np.abs(x.astype(np.float64)))
    for t in (-1.0, 0.0, float(mags[1024]), 0.37, 3.0, 1e9, float("inf")):
        y, _, idx, c = _run(ctx, Wt, xd, 2048, sel_mode=B.AF_SEL_THRESHOLD, t=t, y_kind=B.AF_F32)
        ref_idx = O.select_threshold(x, t)
        assert c == len(ref_idx) and np.array_equal(idx, ref_idx), t
        assert O.rel_err(y, O.sparse_gemv(W, x, ref_idx)) <= 1e-4, t
    y = ctx.select_gemv_f16(Wt, xd, sel_mode=B.AF_SEL_DENSE, y_kind=B.AF_F32)
    ctx.synchronize()
    assert O.rel_err(to_host(y), O.sparse_gemv(W, x, np.arange(2048))) <= 1e-4
    res = S.activation(5, S.channel_scales(5, 520, "r"), "r", 0)
    y, _, idx, c = _run(ctx, Wt, xd, 2048, sel_mode=B.AF_SEL_TOPK, k=0, residual=to_dev(res))
    assert c == 0 and np.array_equal(y, res)
    # special values: NaN ranks highest for top-k and never passes a threshold
    z = x.copy(); z[7] = np.nan; z[9] = np.inf; z[11] = -np.inf
    _, _, idx, c = _run(ctx, Wt, to_dev(z), 2048, sel_mode=B.AF_SEL_TOPK, k=3)
    assert idx.tolist() == [7, 9, 11]
    _, _, idx, c = _run(ctx, Wt, to_dev(z), 2048, sel_mode=B.AF_SEL_THRESHOLD, t=1e4)
    assert idx.tolist() == O.select_threshold(z, 1e4).tolist() == [9, 11]


def _topk_property(x16, idx, k):
    key = (np.asarray(x16).view(np.uint16) & 0x7FFF).astype(np.int64)
    assert len(idx) == k and np.all(np.diff(idx) > 0)
    sel = np.zeros(len(key), bool); sel[idx] = True
    if k == 0 or k == len(key):
        return
    lo, hi = key[sel].min(), key[~sel].max()
    assert lo >= hi
    if lo == hi:
        assert np.nonzero(sel & (key == lo))[0].max() < np.nonzero(~sel & (key == lo))[0].min()


@pytest.mark.parametrize("n,out", [(256, 264), (4096, 12288), (5120, 1032)])
def test_rmsnorm_producer(ctx, n, out):
    W, h = _wx(out, n, n + 1)
    g = S.norm_gain(3, n, "fused")
    x_ref = O.round_f16(O.rmsnorm(h, g, 1e-5))
    k = n // 2
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    y, x_gpu, idx, c = _run(ctx, Wt, to_dev(h), n, producer=B.AF_PRO_RMSNORM, gain=to_dev(g),
                            eps=1e-5, sel_mode=B.AF_SEL_TOPK, k=k, y_kind=B.AF_F32)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    _topk_property(x_gpu, idx, k)
    ref_idx = O.select_topk(x_ref, k)
    if np.array_equal(x_gpu.view(np.uint16), x_ref.view(np.uint16)):
        assert np.array_equal(idx, ref_idx)
    # the GEMV itself, judged on the GPU's own x and set
    assert O.rel_err(y, O.sparse_gemv(W, x_gpu, idx)) <= 1e-4


def test_silumul_producer(ctx):
    n, out = 11008, 520
    W, _ = _wx(out, n, 77)
    sc = S.channel_scales(77, 2 * n, "gu")
    gu = (S.activation(77, sc, "gu", 0).astype(np.float32) * 0.3).astype(np.float16)
    x_ref = O.round_f16(O.silu(gu[:n]) * gu[n:].astype(np.float64))
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    k = O.keep_count(n, 50)
    y, x_gpu, idx, c = _run(ctx, Wt, to_dev(gu), n, producer=B.AF_PRO_SILUMUL,
                            sel_mode=B.AF_SEL_TOPK, k=k, y_kind=B.AF_F32)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    _topk_property(x_gpu, idx, k)
    assert O.rel_err(y, O.sparse_gemv(W, x_gpu, idx)) <= 1e-4


def test_argument_errors(ctx):
    W, x = _wx(64, 64, 1)
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x)
    for kw, code in ((dict(producer=9), -1), (dict(sel_mode=5), -1), (dict(k=65), -1),
                     (dict(producer=B.AF_PRO_RMSNORM), -2), (dict(sel_mode=B.AF_SEL_THRESHOLD, t=float("nan")), -1)):
        with pytest.raises(B.AfError) as e:
            ctx.select_gemv_f16(Wt, xd, **kw)
        assert e.value.status == code, kw


# ---- threshold selection per channel range (no index list asked for) ---------------------
def _run_noidx(ctx, Wt, src, n, **kw):
    xo = torch.zeros(n, dtype=torch.float16, device="cuda")
    y = ctx.select_gemv_f16(Wt, src, x_out=xo, sel_mode=B.AF_SEL_THRESHOLD, y_kind=B.AF_F32, **kw)
    ctx.synchronize()
    return to_host(y), to_host(xo)


@pytest.mark.parametrize("out,n", [(136, 64), (520, 1000), (4096, 4096), (1032, 11008),
                                   (2056, 5120), (264, 28672), (22016, 4096), (8, 32768)])
def test_range_threshold_identity_producer(ctx, out, n):
    W, x = _wx(out, n, out + n)
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x)
    mags = np.sort(np.abs(x.astype(np.float64)))
    for t in (-1.0, 0.0, float(mags[n // 2]), float(mags[(7 * n) // 10]), 1e9):
        y, xo = _run_noidx(ctx, Wt, xd, n, t=t)
        assert np.array_equal(xo.view(np.uint16), x.view(np.uint16))
        ref_idx = O.select_threshold(x, t)
        assert O.rel_err(y, O.sparse_gemv(W, x, ref_idx)) <= 1e-4, (t, len(ref_idx))


def test_range_threshold_special_values_and_residual(ctx):
    n, out = 2048, 520
    W, x = _wx(out, n, 5)
    z = x.copy(); z[7] = np.nan; z[9] = np.inf; z[11] = -np.inf; z[2040] = np.nan
    W2 = W.copy(); W2[:, [9, 11]] = 0     # keep the reference finite: Inf channels meet zero weights
    Wt = ctx.pack_inmajor_f16(to_dev(W2))
    # NaN never passes; Inf passes any finite threshold (and multiplies a zero weight -> NaN in
    # IEEE arithmetic, on both sides), so compare on a vector with the Infs removed as well
    z2 = z.copy(); z2[[9, 11]] = 0
    y, _ = _run_noidx(ctx, Wt, to_dev(z2), n, t=0.5)
    ref_idx = O.select_threshold(z2, 0.5)
    assert 7 not in ref_idx and 2040 not in ref_idx
    # the oracle multiplies the masked vector out densely (NaN * 0 = NaN), so its input is the
    # same vector with the unselected NaN channels cleared
    z3 = z2.copy(); z3[[7, 2040]] = 0
    assert O.rel_err(y, O.sparse_gemv(W2, z3, ref_idx)) <= 1e-4
    res = S.activation(5, S.channel_scales(5, out, "r"), "r", 0)
    y = ctx.select_gemv_f16(Wt, to_dev(x), sel_mode=B.AF_SEL_THRESHOLD, t=1e9, residual=to_dev(res))
    ctx.synchronize()
    assert np.array_equal(to_host(y), res)            # nothing passes: y is the residual


@pytest.mark.parametrize("n,out", [(256, 264), (4096, 12288), (5120, 1032), (8192, 10240)])
def test_range_threshold_rmsnorm_producer(ctx, n, out):
    W, h = _wx(out, n, n + 1)
    g = S.norm_gain(3, n, "fused")
    x_ref = O.round_f16(O.rmsnorm(h, g, 1e-5))
    t = float(np.sort(np.abs(x_ref.astype(np.float64)))[n // 2])
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    y, x_gpu = _run_noidx(ctx, Wt, to_dev(h), n, producer=B.AF_PRO_RMSNORM, gain=to_dev(g), eps=1e-5, t=t)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    # same bits as the list-building form of the kernel
    _, x_list, idx, c = _run(ctx, Wt, to_dev(h), n, producer=B.AF_PRO_RMSNORM, gain=to_dev(g),
                             eps=1e-5, sel_mode=B.AF_SEL_THRESHOLD, t=t, y_kind=B.AF_F32)
    assert np.array_equal(x_gpu.view(np.uint16), x_list.view(np.uint16))
    # the GEMV, judged on the GPU's own x: the set follows from the definition
    own = O.select_threshold(x_gpu, t)
    assert np.array_equal(idx, own)
    assert O.rel_err(y, O.sparse_gemv(W, x_gpu, own)) <= 1e-4
    assert abs(len(own) / n - 0.5) < 0.02


def test_range_threshold_silumul_producer(ctx):
    n, out = 11008, 520
    W, _ = _wx(out, n, 77)
    sc = S.channel_scales(77, 2 * n, "gu")
    gu = (S.activation(77, sc, "gu", 0).astype(np.float32) * 0.3).astype(np.float16)
    x_ref = O.round_f16(O.silu(gu[:n]) * gu[n:].astype(np.float64))
    t = float(np.sort(np.abs(x_ref.astype(np.float64)))[n // 2])
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    y, x_gpu = _run_noidx(ctx, Wt, to_dev(gu), n, producer=B.AF_PRO_SILUMUL, t=t)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    own = O.select_threshold(x_gpu, t)
    assert O.rel_err(y, O.sparse_gemv(W, x_gpu, own)) <= 1e-4


@pytest.mark.parametrize("name,out,n,producer", [("gateup", 22016, 4096, "rmsnorm"), ("down", 4096, 11008, "silumul"),
                                                 ("o", 4096, 4096, "none")])
def test_7b_shapes_fused_forms_sampled(ctx, name, out, n, producer):
    """The benchmark's full-size operators in the launch shapes the bench times: the fused top-k
    form and the fused threshold form (no index list), sampled output columns against the oracle
    on the x the GPU produced (the selection is then checked from the definition)."""
    W = S.weight_matrix(0, out, n, "7b-fused", name, threads=8)
    kw = {}
    if producer == "rmsnorm":
        src = S.activation(0, S.channel_scales(0, n, "7b-fused", name), "7b-fused", name)
        g = S.norm_gain(0, n, "7b-fused", name)
        kw = dict(producer=B.AF_PRO_RMSNORM, gain=to_dev(g), eps=1e-5)
        x_ref = O.round_f16(O.rmsnorm(src, g, 1e-5))
    elif producer == "silumul":
        sc = S.channel_scales(0, 2 * n, "7b-fused", name)
        src = (S.activation(0, sc, "7b-fused", name).astype(np.float32) * 0.3).astype(np.float16)
        kw = dict(producer=B.AF_PRO_SILUMUL)
        x_ref = O.round_f16(O.silu(src[:n]) * src[n:].astype(np.float64))
    else:
        src = S.activation(0, S.channel_scales(0, n, "7b-fused", name), "7b-fused", name)
        x_ref = src
    Wt = ctx.pack_inmajor_f16(to_dev(W)); sd = to_dev(src)
    rows = np.random.default_rng(1).choice(out, size=64, replace=False)
    k = O.keep_count(n, 50)
    # top-k, fused
    y, x_gpu, idx, c = _run(ctx, Wt, sd, n, sel_mode=B.AF_SEL_TOPK, k=k, y_kind=B.AF_F32, **kw)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    _topk_property(x_gpu, idx, k)
    ref = O.sparse_gemv(W[rows], x_gpu, idx)
    assert np.max(np.abs(y[rows] - ref)) <= 1e-4 * np.sqrt(np.mean(ref ** 2))
    # threshold, fused, no index list: the set follows from the definition on the GPU's x
    t = float(np.sort(np.abs(x_gpu.astype(np.float64)))[n // 2])
    y, x2 = _run_noidx(ctx, Wt, sd, n, t=t, **kw)
    assert np.array_equal(x2.view(np.uint16), x_gpu.view(np.uint16))
    own = O.select_threshold(x_gpu, t)
    ref = O.sparse_gemv(W[rows], x_gpu, own)
    assert np.max(np.abs(y[rows] - ref)) <= 1e-4 * np.sqrt(np.mean(ref ** 2))


def _random_cases(count, seed=2024):
    """Seeded mix of operator shapes that reaches every launch-shape branch (narrow / medium / wide
    tiles, one split and many), ragged sizes, every producer and both selection kinds."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        out = 8 * int(rng.integers(1, [40, 800, 1600, 3600][i % 4]))
        n = 8 * int(rng.integers(1, min(2048, max(8, (3 << 20) // out))))   # the fused form takes in % 8 == 0
        pro = ("none", "rmsnorm", "silumul")[int(rng.integers(0, 3))]
        keep = float(rng.choice([0.05, 0.3, 0.5, 0.8, 1.0]))
        cases.append((out, n, pro, keep, int(rng.integers(0, 3))))
    return cases


@pytest.mark.parametrize("out,n,pro,keep,form", _random_cases(28))
def test_random_shapes_every_form(ctx, out, n, pro, keep, form):
    """form 0: top-k with list, 1: threshold with list, 2: threshold by channel range."""
    seed = out * 131 + n
    W = S.weight_matrix(seed, out, n, "rand", out, n)
    kw = {}
    if pro == "rmsnorm":
        src = S.activation(seed, S.channel_scales(seed, n, "rand"), "rand", 0)
        g = S.norm_gain(seed, n, "rand")
        kw = dict(producer=B.AF_PRO_RMSNORM, gain=to_dev(g), eps=1e-5)
        x_ref = O.round_f16(O.rmsnorm(src, g, 1e-5))
    elif pro == "silumul":
        src = (S.activation(seed, S.channel_scales(seed, 2 * n, "rand"), "rand", 1).astype(np.float32)
               * 0.3).astype(np.float16)
        kw = dict(producer=B.AF_PRO_SILUMUL)
        x_ref = O.round_f16(O.silu(src[:n]) * src[n:].astype(np.float64))
    else:
        src = S.activation(seed, S.channel_scales(seed, n, "rand"), "rand", 0)
        x_ref = src
    Wt = ctx.pack_inmajor_f16(to_dev(W)); sd = to_dev(src)
    k = min(n, max(1, int(round(keep * n))))
    if form == 0:
        y, x_gpu, idx, c = _run(ctx, Wt, sd, n, sel_mode=B.AF_SEL_TOPK, k=k, y_kind=B.AF_F32, **kw)
        _topk_property(x_gpu, idx, k)
    else:
        mags = np.sort(np.abs(x_ref.astype(np.float64)))
        t = float(mags[n - k]) if k < n else 0.0
        if form == 1:
            y, x_gpu, idx, c = _run(ctx, Wt, sd, n, sel_mode=B.AF_SEL_THRESHOLD, t=t, y_kind=B.AF_F32, **kw)
            assert np.array_equal(idx, O.select_threshold(x_gpu, t))
        else:
            y, x_gpu = _run_noidx(ctx, Wt, sd, n, t=t, **kw)
            idx = O.select_threshold(x_gpu, t)
    assert O.rel_err(x_gpu, x_ref) <= TOL
    if pro == "none":
        assert np.array_equal(x_gpu.view(np.uint16), x_ref.view(np.uint16))
    assert O.rel_err(y, O.sparse_gemv(W, x_gpu, idx)) <= 1e-4
