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


# ---- channel-local groups (scales inside a channel's row) ---------------------------------
@pytest.mark.parametrize("out,n", [(32, 8), (160, 96), (1056, 640), (4096, 2048)])
def test_cl_pack_matches_oracle_quantiser_bit_for_bit(ctx, out, n):
    W, _ = _case(out, n, 2)
    if out >= 160:
        W[32:64, 3] = 0
        W[0:32, 5] = 0; W[7, 5] = -0.75
        W[32:64, 6] = np.float16(6e-8)
    packed, scales = ctx.pack_q4_cl(to_dev(W))
    ctx.synchronize()
    nib, s = O.quantize_q4_cl(W)
    assert np.array_equal(to_host(scales).view(np.uint16), s.view(np.uint16))
    assert np.array_equal(to_host(packed), O.pack_q4(nib))


def test_cl_pack_fused_columns(ctx):
    """Two operators side by side (as q|k|v and gate|up are stored): each keeps its own groups."""
    Wa, _ = _case(64, 96, 3); Wb, _ = _case(96, 96, 4)
    import torch
    packed = torch.zeros((96, 80), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((96, 5), dtype=torch.float16, device="cuda")
    ctx.pack_q4_cl(to_dev(Wa), packed, scales, col0=0)
    ctx.pack_q4_cl(to_dev(Wb), packed, scales, col0=64)
    ctx.synchronize()
    na, sa = O.quantize_q4_cl(Wa); nb, sb = O.quantize_q4_cl(Wb)
    assert np.array_equal(to_host(packed), np.concatenate([O.pack_q4(na), O.pack_q4(nb)], axis=1))
    assert np.array_equal(to_host(scales).view(np.uint16), np.concatenate([sa, sb], axis=1).view(np.uint16))


@pytest.mark.parametrize("out,n,k", [(32, 8, 3), (160, 96, 48), (544, 768, 300), (1056, 640, 640),
                                     (4096, 2048, 1024), (12288, 1024, 307), (22016, 256, 128),
                                     (4096, 11008, 5511)])
def test_cl_gemv(ctx, out, n, k):
    W, x = _case(out, n, out + n + 1)
    nib, s = O.quantize_q4_cl(W)
    idx = O.select_topk(x, k)
    packed, scales = ctx.pack_q4_cl(to_dev(W))
    ref = O.sparse_gemv_q4_cl(nib, s, x, idx)
    for kind, tol in ((B.AF_F32, 1e-4), (B.AF_F16, TOL)):
        y = ctx.sparse_gemv_q4_cl(packed, scales, to_dev(x), to_dev(idx), y_kind=kind)
        ctx.synchronize()
        assert O.rel_err(to_host(y), ref) <= tol, kind
    res = S.activation(3, S.channel_scales(3, out, "q4res"), "q4res", 0)
    y = ctx.sparse_gemv_q4_cl(packed, scales, to_dev(x), None, residual=to_dev(res))
    ctx.synchronize()
    assert O.rel_err(to_host(y), O.sparse_gemv_q4_cl(nib, s, x, np.arange(n)) + res.astype(np.float64)) <= TOL
    with pytest.raises(B.AfError):
        ctx.sparse_gemv_q4_cl(packed, scales, to_dev(x), None, out=out - 8)      # out % 32 != 0


@pytest.mark.parametrize("out,n,col0,ld", [(8, 32, 0, 8), (136, 96, 0, 136), (520, 640, 8, 544)])
def test_unpack_is_the_inverse_of_pack_on_the_device(ctx, out, n, col0, ld):
    """af_unpack_q4_g32 reads the packed bytes and scales the way the GEMV kernel does: the
    integers it returns are the oracle quantiser's, the products are exact in fp32.  A nibble
    order or a scale index that differed from the documented layout would fail here."""
    import torch
    W, _ = _case(out, n, 7)
    W[1, :32] = 0                                       # a group whose scale is zero
    packed = torch.zeros((n, ld // 2), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((n // 32, ld), dtype=torch.float16, device="cuda")
    ctx.pack_q4_g32(to_dev(W), packed, scales, col0=col0)
    q, w = ctx.unpack_q4_g32(packed, scales, out, col0=col0)
    ctx.synchronize()
    nib, s = O.quantize_q4_g32(W)
    assert np.array_equal(to_host(q).astype(np.int64), nib.astype(np.int64) - 8)
    assert np.array_equal(to_host(w).astype(np.float64), O.dequant_q4_g32(nib, s))


def _random_q4_cases(count, seed=77):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        out = 32 * int(rng.integers(1, [10, 200, 400, 900][i % 4]))
        n = 32 * int(rng.integers(1, min(512, max(2, (3 << 20) // (4 * out)))))
        cases.append((out, n, max(1, int(n * float(rng.choice([0.05, 0.3, 0.5, 0.8, 1.0])))), i % 2))
    return cases


@pytest.mark.parametrize("out,n,k,cl", _random_q4_cases(16))
def test_q4_random_shapes_both_layouts(ctx, out, n, k, cl):
    """Seeded shapes across the launch-shape branches, in the row-major-group layout (cl = 0) and
    the column-block layout (cl = 1)."""
    W, x = _case(out, n, out * 7 + n)
    idx = O.select_topk(x, k)
    if cl:
        nib, s = O.quantize_q4_cl(W)
        packed, scales = ctx.pack_q4_cl(to_dev(W))
        y = ctx.sparse_gemv_q4_cl(packed, scales, to_dev(x), to_dev(idx), y_kind=B.AF_F32)
        ref = O.sparse_gemv_q4_cl(nib, s, x, idx)
    else:
        nib, s = O.quantize_q4_g32(W)
        packed, scales = ctx.pack_q4_g32(to_dev(W))
        y = ctx.sparse_gemv_q4(packed, scales, to_dev(x), to_dev(idx), y_kind=B.AF_F32)
        ref = O.sparse_gemv_q4(nib, s, x, idx)
    ctx.synchronize()
    assert O.rel_err(to_host(y), ref) <= 1e-4
