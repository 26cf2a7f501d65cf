"""GPU parity: af_sparse_gemv_f16 / af_pack_inmajor_f16 / af_sparse_gemv_union_f16 against the
oracle (outputs within 2e-3 by the oracle's rel_err measure; layouts and unions bit-exact)."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B
from gpu_util import ctx, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu
TOL = 2e-3   # spec bound: fp32 accumulation, fp16 weights, fp16 output rounding 2^-11


def _case(out, n, seed):
    W = S.weight_matrix(seed, out, n, "gemv", out, n)
    x = S.activation(seed, S.channel_scales(seed, n, "gemv"), "gemv", 0)
    return W, x


def _run(ctx, W, x, idx, y_kind=B.AF_F16, residual=None, ld=None, nidx_dev=None, nidx=None):
    Wd = to_dev(W)
    Wt = ctx.pack_inmajor_f16(Wd, ld=ld)
    y = ctx.sparse_gemv_f16(Wt, to_dev(x), None if idx is None else to_dev(idx), y_kind=y_kind,
                            residual=None if residual is None else to_dev(residual),
                            out=W.shape[0], nidx_dev=nidx_dev, nidx=nidx)
    ctx.synchronize()
    return to_host(y)


def test_pack_is_a_transpose(ctx):
    W, _ = _case(1032, 1000, 1)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    ctx.synchronize()
    assert np.array_equal(to_host(Wt), W.T)
    # fused side by side with a leading dimension
    A, _ = _case(40, 72, 2); Bm, _ = _case(24, 72, 3)
    buf = torch.zeros((72, 64), dtype=torch.float16, device="cuda")
    ctx.pack_inmajor_f16(to_dev(A), buf, col0=0); ctx.pack_inmajor_f16(to_dev(Bm), buf, col0=40)
    ctx.synchronize()
    assert np.array_equal(to_host(buf), np.concatenate([A, Bm]).T)


def test_config0(ctx):
    W, x = _case(2048, 2048, 0)
    idx = O.select_topk(x, 1024)
    for kind in (B.AF_F16, B.AF_F32):
        y = _run(ctx, W, x, idx, y_kind=kind)
        assert O.rel_err(y, O.sparse_gemv(W, x, idx)) <= (TOL if kind == B.AF_F16 else 1e-4)


@pytest.mark.parametrize("out,n,k", [(8, 1, 1), (8, 33, 17), (136, 100, 50), (520, 777, 300),
                                     (1032, 1000, 999), (4096, 1024, 512), (4104, 2048, 614),
                                     (12288, 512, 256), (22016, 256, 77), (1024, 8192, 4096)])
def test_shapes_with_ragged_tiles(ctx, out, n, k):
    W, x = _case(out, n, out + n)
    idx = O.select_topk(x, k)
    y = _run(ctx, W, x, idx)
    assert O.rel_err(y, O.sparse_gemv(W, x, idx)) <= TOL


def test_dense_empty_residual_and_device_count(ctx):
    W, x = _case(520, 640, 5)
    res = S.activation(5, S.channel_scales(5, 520, "res"), "res", 0)
    allidx = np.arange(640, dtype=np.int32)
    ref_dense = O.sparse_gemv(W, x, allidx)
    assert O.rel_err(_run(ctx, W, x, None), ref_dense) <= TOL             # idx == NULL
    assert O.rel_err(_run(ctx, W, x, allidx), ref_dense) <= TOL           # sparsity 0
    empty = np.zeros(0, dtype=np.int32)
    y0 = _run(ctx, W, x, np.zeros(1, np.int32), nidx=0)
    assert np.all(y0 == 0)
    yr = _run(ctx, W, x, np.zeros(1, np.int32), nidx=0, residual=res)
    assert np.array_equal(yr, res)
    idx = O.select_topk(x, 320)
    y = _run(ctx, W, x, idx, residual=res)
    assert O.rel_err(y, O.sparse_gemv(W, x, idx) + res.astype(np.float64)) <= TOL
    # the count can live on the device (threshold selection): only the first 200 entries count
    cnt = to_dev(np.array([200], dtype=np.int32))
    y = _run(ctx, W, x, idx, nidx_dev=cnt)
    assert O.rel_err(y, O.sparse_gemv(W, x, idx[:200])) <= TOL
    # leading dimension wider than out
    y = _run(ctx, W, x, idx, ld=528)
    assert O.rel_err(y, O.sparse_gemv(W, x, idx)) <= TOL
    del empty


def test_one_hot_and_determinism(ctx):
    W, x = _case(264, 96, 6)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    xd = to_dev(x)
    for j in (0, 50, 95):
        y = ctx.sparse_gemv_f16(Wt, xd, to_dev(np.array([j], np.int32)), y_kind=B.AF_F32)
        ctx.synchronize()
        assert np.array_equal(to_host(y), (W[:, j].astype(np.float32) * np.float32(x[j])))
    W, x = _case(4096, 4096, 7)
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x); idx = to_dev(O.select_topk(x, 2048))
    first = None
    for _ in range(20):
        y = ctx.sparse_gemv_f16(Wt, xd, idx, y_kind=B.AF_F32)
        ctx.synchronize()
        h = to_host(y).copy()
        if first is None:
            first = h
        assert np.array_equal(first, h)


@pytest.mark.parametrize("name,out,n", [("qkv", 12288, 4096), ("o", 4096, 4096),
                                        ("gateup", 22016, 4096), ("down", 4096, 11008)])
def test_7b_shapes_sampled_outputs(ctx, name, out, n):
    """Full-size operator of the benchmark workload: sampled output columns against the
    oracle, plus the additivity property over a split of the index list for all columns."""
    W = S.weight_matrix(0, out, n, "7b-op", name, threads=8)
    x = S.activation(0, S.channel_scales(0, n, "7b-op", name), "7b-op", name)
    idx = O.select_topk(x, O.keep_count(n, 50))
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x)
    y = ctx.sparse_gemv_f16(Wt, xd, to_dev(idx), y_kind=B.AF_F32)
    ctx.synchronize()
    y = to_host(y)
    rows = np.random.default_rng(0).choice(out, size=96, replace=False)
    ref = O.sparse_gemv(W[rows], x, idx)
    scale = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(y[rows] - ref)) <= 1e-4 * scale
    ya = ctx.sparse_gemv_f16(Wt, xd, to_dev(idx[: len(idx) // 3]), y_kind=B.AF_F32)
    yb = ctx.sparse_gemv_f16(Wt, xd, to_dev(idx[len(idx) // 3:]), y_kind=B.AF_F32)
    ctx.synchronize()
    assert np.max(np.abs(to_host(ya) + to_host(yb) - y)) <= 1e-4 * scale


def test_argument_errors(ctx):
    W, x = _case(16, 32, 8)
    Wt = ctx.pack_inmajor_f16(to_dev(W)); xd = to_dev(x)
    idx = to_dev(np.arange(4, dtype=np.int32))
    with pytest.raises(B.AfError) as e:
        ctx.sparse_gemv_f16(Wt, xd, idx, out=12)          # out % 8
    assert e.value.status == -3
    with pytest.raises(B.AfError) as e:
        ctx.sparse_gemv_f16(Wt, xd, idx, nidx=33)         # more indices than channels
    assert e.value.status == -1
    with pytest.raises(B.AfError) as e:
        ctx.sparse_gemv_f16(Wt, xd, idx, y_kind=7)
    assert e.value.status == -1


# --------------------------------------------------------------------------- union
@pytest.mark.parametrize("Bt", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("out,n", [(264, 200), (2056, 1024), (8192, 512)])
def test_union_small_batch(ctx, Bt, out, n):
    W = S.weight_matrix(9, out, n, "union", out, n)
    sc = S.channel_scales(9, n, "union")
    X = np.stack([S.activation(9, sc, "union", b) for b in range(Bt)])
    k = n // 2
    idx_b = np.stack([O.select_topk(X[b], k) for b in range(Bt)])
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    Y, U, un = ctx.sparse_gemv_union_f16(Wt, to_dev(X), to_dev(idx_b), y_kind=B.AF_F32)
    ctx.synchronize()
    Uo = O.union_indices(list(idx_b))
    assert int(to_host(un)[0]) == len(Uo)
    assert np.array_equal(to_host(U)[: len(Uo)], Uo)
    ref = O.union_gemv(W, X, list(idx_b))
    Yh = to_host(Y)
    for b in range(Bt):
        assert O.rel_err(Yh[b], ref[b]) <= 1e-4
    Y16, _, _ = ctx.sparse_gemv_union_f16(Wt, to_dev(X), to_dev(idx_b))
    ctx.synchronize()
    for b in range(Bt):
        assert O.rel_err(to_host(Y16)[b], ref[b]) <= TOL


def test_union_identical_tokens_and_b1_equals_single(ctx):
    out, n = 520, 384
    W = S.weight_matrix(10, out, n, "union2")
    x = S.activation(10, S.channel_scales(10, n, "union2"), "union2", 0)
    idx = O.select_topk(x, 192)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    X = np.stack([x] * 4); idx_b = np.stack([idx] * 4)
    Y, U, un = ctx.sparse_gemv_union_f16(Wt, to_dev(X), to_dev(idx_b), y_kind=B.AF_F32)
    ctx.synchronize()
    assert int(to_host(un)[0]) == 192 and np.array_equal(to_host(U)[:192], idx)
    Yh = to_host(Y)
    assert all(np.array_equal(Yh[0], Yh[b]) for b in range(4))
    assert O.rel_err(Yh[0], O.sparse_gemv(W, x, idx)) <= 1e-4


@pytest.mark.parametrize("name,out,n,Bt", [("down", 8192, 28672, 8), ("gateup", 57344, 8192, 4)])
def test_union_70b_shapes_sampled(ctx, name, out, n, Bt):
    """Widest input (28672) and widest output (57344) of the 70B-shape layer: the union is
    compared bit-for-bit, sampled output columns against the oracle for every token."""
    W = S.weight_matrix(0, out, n, "70b-union", name, threads=8)
    sc = S.channel_scales(0, n, "70b-union", name)
    X = np.stack([S.activation(0, sc, "70b-union", name, b) for b in range(Bt)])
    k = O.keep_count(n, 50)
    idx_b = np.stack([O.select_topk(X[b], k) for b in range(Bt)])
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    Y, U, un = ctx.sparse_gemv_union_f16(Wt, to_dev(X), to_dev(idx_b), y_kind=B.AF_F32)
    ctx.synchronize()
    Uo = O.union_indices(list(idx_b))
    assert int(to_host(un)[0]) == len(Uo) and np.array_equal(to_host(U)[: len(Uo)], Uo)
    assert k < len(Uo) < n                      # shared channel scales: tokens overlap but differ
    rows = np.random.default_rng(1).choice(out, size=48, replace=False)
    ref = O.union_gemv(W[rows], X, list(idx_b))
    Yh = to_host(Y)
    for b in range(Bt):
        assert np.max(np.abs(Yh[b][rows] - ref[b])) <= 1e-4 * np.sqrt(np.mean(ref[b] ** 2)), b
    # per-token selection on the GPU gives the same sets the union was built from
    for b in (0, Bt - 1):
        got = ctx.select_topk(to_dev(X[b]), k)
        ctx.synchronize()
        assert np.array_equal(to_host(got), idx_b[b])


def test_index_precondition_is_reported_not_followed(ctx):
    """An index list that breaks its precondition never makes a kernel read outside the
    caller's buffers: an entry out of range adds nothing and sets AF_DEVERR_IDX; with
    AF_OPT_VALIDATE an unsorted or repeated list is reported as well."""
    W, x = _case(136, 100, 11)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    good = O.select_topk(x, 40)
    assert ctx.last_device_error() == 0
    bad = good.copy(); bad[7] = 100; bad[9] = -3            # out of range on both sides
    y = ctx.sparse_gemv_f16(Wt, to_dev(x), to_dev(bad)); ctx.synchronize()
    assert ctx.last_device_error() == B.AF_DEVERR_IDX
    kept = np.delete(good, [7, 9])
    assert O.rel_err(to_host(y), O.sparse_gemv(W, x, kept)) <= TOL
    assert ctx.last_device_error() == 0                      # the read above cleared the word
    # sorted-and-unique is only checked in validate mode
    rep = good.copy(); rep[5] = rep[4]
    ctx.sparse_gemv_f16(Wt, to_dev(x), to_dev(rep)); ctx.synchronize()
    assert ctx.last_device_error() == 0
    ctx.set_option(B.AF_OPT_VALIDATE, 1)
    try:
        ctx.sparse_gemv_f16(Wt, to_dev(x), to_dev(rep)); ctx.synchronize()
        assert ctx.last_device_error() == B.AF_DEVERR_IDX
        ctx.sparse_gemv_f16(Wt, to_dev(x), to_dev(good)); ctx.synchronize()
        assert ctx.last_device_error() == 0
        # union: a row of the batch with an entry out of range
        X = np.stack([x, x[::-1].copy()])
        idx_b = np.stack([good, O.select_topk(X[1], 40)]).astype(np.int32)
        idx_b[1, 3] = 4000
        ctx.sparse_gemv_union_f16(Wt, to_dev(X), to_dev(idx_b)); ctx.synchronize()
        assert ctx.last_device_error() == B.AF_DEVERR_IDX
    finally:
        ctx.set_option(B.AF_OPT_VALIDATE, 0)


def _random_gemv_cases(count, seed=99):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        out = 8 * int(rng.integers(1, [40, 800, 1600, 3600][i % 4]))
        n = int(rng.integers(1, min(16384, max(64, (24 << 20) // out))))
        cases.append((out, n, max(1, int(n * float(rng.choice([0.02, 0.3, 0.5, 0.8, 1.0]))))))
    return cases


@pytest.mark.parametrize("out,n,k", _random_gemv_cases(20))
def test_random_shapes_and_random_sets(ctx, out, n, k):
    """Seeded shapes across the launch-shape branches with index sets drawn at random (any subset
    is a valid argument, not only a top-k set)."""
    W, x = _case(out, n, out * 3 + n)
    idx = np.sort(np.random.default_rng(out + n).choice(n, size=k, replace=False)).astype(np.int32)
    Wt = ctx.pack_inmajor_f16(to_dev(W))
    y = ctx.sparse_gemv_f16(Wt, to_dev(x), to_dev(idx), y_kind=B.AF_F32)
    ctx.synchronize()
    assert O.rel_err(to_host(y), O.sparse_gemv(W, x, idx)) <= 1e-4
