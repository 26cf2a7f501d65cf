"""GPU parity: af_pack_q4_g32 (bit-exact against the oracle's quantiser) and
af_sparse_gemv_q4 (within 2e-3 of the oracle on the dequantised weights)."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B
from gpu_util import ctx, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _case(out, n, seed):
    W = S.weight_matrix(seed, out, n, "q4", out, n)
    x = S.activation(seed, S.channel_scales(seed, n, "q4"), "q4", 0)
    return W, x


@pytest.mark.parametrize("out,n", [(8, 32), (136, 96), (1032, 640), (4096, 2048)])
def test_pack_matches_oracle_quantiser_bit_for_bit(ctx, out, n):
    W, _ = _case(out, n, 1)
    if out >= 136:   # special groups: all zero, a lone extreme, fp16 subnormals
        W[3, 32:64] = 0
        W[5, 0:32] = 0; W[5, 7] = -0.75
        W[6, 32:64] = np.float16(6e-8)
    packed, scales = ctx.pack_q4_g32(to_dev(W))
    ctx.synchronize()
    nib, s = O.quantize_q4_g32(W)
    assert np.array_equal(to_host(scales).view(np.uint16), s.view(np.uint16))
    assert np.array_equal(to_host(packed), O.pack_q4(nib))


@pytest.mark.parametrize("out,n,k", [(8, 32, 9), (136, 96, 48), (520, 768, 300), (1032, 640, 640),
                                     (4096, 2048, 1024), (12288, 1024, 307), (22016, 256, 128)])
def test_q4_gemv(ctx, out, n, k):
    W, x = _case(out, n, out + n)
    nib, s = O.quantize_q4_g32(W)
    idx = O.select_topk(x, k)
    packed, scales = ctx.pack_q4_g32(to_dev(W))
    for kind, tol in ((B.AF_F32, 1e-4), (B.AF_F16, TOL)):
        y = ctx.sparse_gemv_q4(packed, scales, to_dev(x), to_dev(idx), y_kind=kind)
        ctx.synchronize()
        assert O.rel_err(to_host(y), O.sparse_gemv_q4(nib, s, x, idx)) <= tol, kind


def test_q4_dense_empty_residual(ctx):
    W, x = _case(264, 320, 3)
    nib, s = O.quantize_q4_g32(W)
    res = S.activation(3, S.channel_scales(3, 264, "q4res"), "q4res", 0)
    packed, scales = ctx.pack_q4_g32(to_dev(W))
    xd = to_dev(x)
    y = ctx.sparse_gemv_q4(packed, scales, xd, None)
    ctx.synchronize()
    assert O.rel_err(to_host(y), O.sparse_gemv_q4(nib, s, x, np.arange(320))) <= TOL
    y = ctx.sparse_gemv_q4(packed, scales, xd, to_dev(np.zeros(1, np.int32)), nidx=0, residual=to_dev(res))
    ctx.synchronize()
    assert np.array_equal(to_host(y), res)
    idx = O.select_topk(x, 111)
    y = ctx.sparse_gemv_q4(packed, scales, xd, to_dev(idx), residual=to_dev(res))
    ctx.synchronize()
    assert O.rel_err(to_host(y), O.sparse_gemv_q4(nib, s, x, idx) + res.astype(np.float64)) <= TOL
    with pytest.raises(B.AfError):
        ctx.sparse_gemv_q4(packed[:40], scales[:1], xd[:40], None)      # in % 32 != 0


def test_q4_7b_down_shape_sampled(ctx):
    out, n = 4096, 11008
    W = S.weight_matrix(0, out, n, "7b-q4", "down", threads=8)
    x = S.activation(0, S.channel_scales(0, n, "7b-q4"), "7b-q4", 0)
    packed, scales = ctx.pack_q4_g32(to_dev(W))
    for sp in (50, 70):
        idx = O.select_topk(x, O.keep_count(n, sp))
        y = ctx.sparse_gemv_q4(packed, scales, to_dev(x), to_dev(idx), y_kind=B.AF_F32)
        ctx.synchronize()
        rows = np.random.default_rng(sp).choice(out, size=64, replace=False)
        nib, s = O.quantize_q4_g32(W[rows])
        ref = O.sparse_gemv_q4(nib, s, x, idx)
        assert np.max(np.abs(to_host(y)[rows] - ref)) <= 1e-4 * np.sqrt(np.mean(ref ** 2))
