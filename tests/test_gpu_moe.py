"""GPU parity: af_decode_moe_layer against the oracle's mixture-of-experts block.

The router decides integers from fp32 logits; the oracle's logits are fp64.  The expert
choice is compared where the oracle's margin between the last chosen and the first rejected
logit is far above fp32 rounding (always the case for the seeded inputs used here; asserted),
the index sets as in the dense layer tests."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B
from paper_2504_08378_amd import model as M
from gpu_util import ctx, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu
TOL = 2e-3
KV_LEN, KV_CAP = 37, 48


def _setup(shape_name, seed):
    shape = S.MODEL_SHAPES[shape_name]
    w = S.moe_layer_weights(seed, shape, 0)
    K, V = S.kv_cache(seed, shape.n_kv_heads, KV_CAP, shape.head_dim, KV_LEN, shape.name, 0)
    h = S.activation(seed, S.channel_scales(seed, shape.d_model, shape.name), "hidden", 0)
    cfg = O.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn)
    widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
    return shape, cfg, w, K, V, h, widths


def _margin_ok(tr):
    z = np.sort(tr.logits)[::-1]
    top = len(tr.experts)
    gaps = np.abs(np.diff(z[: top + 1]))
    return gaps.min() > 1e-4 * max(1.0, np.abs(z).max())


def _sets_close(got, ref, x_ref):
    if np.array_equal(got, ref):
        return True
    key = (np.asarray(x_ref).view(np.uint16) & 0x7FFF).astype(np.int64)
    thr = key[ref].min()
    diff = np.setxor1d(got, ref)
    return len(got) == len(ref) and np.all(np.abs(key[diff] - thr) <= 2)


def _quantised(w, kind):
    """The oracle's view of the weights for a 4-bit kind: every matrix but the router quantised
    by the oracle's own quantiser (the device packer's bits are checked in test_gpu_q4)."""
    if kind == B.AF_W_F16:
        return w, False
    q = O.quantize_q4_cl if kind == B.AF_W_Q4CL else O.quantize_q4_g32
    out = {}
    for k, v in w.items():
        if k == "Wr" or not k.startswith("W"):
            out[k] = v
        elif isinstance(v, list):
            out[k] = [q(m) for m in v]
        else:
            out[k] = q(v)
    return out, ("cl" if kind == B.AF_W_Q4CL else True)


@pytest.mark.parametrize("sp,kind", [(50, B.AF_W_F16), (70, B.AF_W_F16), (50, B.AF_W_Q4G32), (50, B.AF_W_Q4CL)])
def test_moe_layer_topk(ctx, sp, kind):
    shape, cfg, w, K, V, h, widths = _setup("tiny_moe", 11)
    ks = tuple(O.keep_count(n, sp) for n in widths)
    wq, q4 = _quantised(w, kind)
    tr = O.decode_moe_layer(cfg, wq, h, K.copy(), V.copy(), KV_LEN, KV_LEN, O.SelectCfg(O.SEL_TOPK, ks),
                            weights_q4=q4)
    assert _margin_ok(tr)
    lay = M.DeviceMoeLayer(ctx, shape, w, weight_kind=kind)
    Kd, Vd = to_dev(K), to_dev(V)
    hin = to_dev(h); hout = torch.zeros_like(hin)
    lay.run(hin, hout, Kd, Vd, KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_TOPK, ks))
    ctx.synchronize()
    assert to_host(lay.experts).tolist() == tr.experts.tolist()
    assert np.allclose(to_host(lay.weights), tr.weights, rtol=1e-4)
    assert np.allclose(to_host(lay.logits), tr.logits, rtol=1e-3, atol=1e-3)
    d, f = shape.d_model, shape.d_ffn
    assert O.rel_err(to_host(ctx.layer_tap(3, d)), tr.h_mid, 1.0) <= TOL
    same = True
    for p in range(3):
        got = to_host(lay.idx[p])[: ks[p]]
        assert _sets_close(got, tr.idx[p], tr.x[p]), p
        same &= np.array_equal(got, tr.idx[p])
    gu = to_host(ctx.layer_tap(5, 4 * f)); xd = to_host(ctx.layer_tap(6, 2 * f))
    for s in range(2):
        got = to_host(lay.idx[3 + s])[: ks[3]]
        assert _sets_close(got, tr.idx_down[s], tr.x_down[s]), s
        same &= np.array_equal(got, tr.idx_down[s])
        assert O.rel_err(gu[s * 2 * f: (s + 1) * 2 * f], tr.gateup[s * 2 * f: (s + 1) * 2 * f], 1.0) <= (TOL if same else 5e-2)
        assert O.rel_err(xd[s * f: (s + 1) * f], tr.x_down[s], 1.0) <= (TOL if same else 5e-2)
    assert np.array_equal(to_host(Kd)[:, KV_LEN], tr.k_new)
    assert O.rel_err(to_host(hout), tr.hidden, 1.0) <= (TOL if same else 5e-2)


def test_moe_layer_dense_threshold_and_skip_sets(ctx):
    shape, cfg, w, K, V, h, widths = _setup("tiny_moe", 12)
    lay = M.DeviceMoeLayer(ctx, shape, w)
    hin = to_dev(h); hout = torch.zeros_like(hin)
    dense = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), KV_LEN, KV_LEN, O.SelectCfg(O.SEL_DENSE))
    assert _margin_ok(dense)
    lay.run(hin, hout, to_dev(K), to_dev(V), KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_DENSE))
    ctx.synchronize()
    assert to_host(lay.experts).tolist() == dense.experts.tolist()
    assert O.rel_err(to_host(hout), dense.hidden, 1.0) <= TOL
    # thresholds in gaps of the magnitudes along the threshold-mode chain (point 3 serves both slots:
    # its threshold sits in a gap of the pooled magnitudes of the two slots)
    ts = [0.0] * 4
    for p in range(4):
        tr = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), KV_LEN, KV_LEN, O.SelectCfg(O.SEL_THRESHOLD, t=tuple(ts)))
        x = tr.x[p] if p < 3 else np.concatenate(tr.x_down)
        m = np.sort(np.abs(x.astype(np.float64)))
        lo = len(m) // 3
        j = lo + int(np.argmax(np.diff(m)[lo: 2 * len(m) // 3]))
        ts[p] = float(np.float32((m[j] + m[j + 1]) / 2))
    tr = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), KV_LEN, KV_LEN, O.SelectCfg(O.SEL_THRESHOLD, t=tuple(ts)))
    assert _margin_ok(tr)
    for flags in (0, B.AF_SEL_SKIP_SETS):
        for p in range(5):
            lay.count[p].fill_(-7)
        lay.run(hin, hout, to_dev(K), to_dev(V), KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_THRESHOLD, t=ts, flags=flags))
        ctx.synchronize()
        assert to_host(lay.experts).tolist() == tr.experts.tolist()
        same = True
        if flags == 0:
            for p in range(3):
                same &= np.array_equal(to_host(lay.idx[p])[: int(lay.count[p].item())], tr.idx[p])
            for s in range(2):
                same &= np.array_equal(to_host(lay.idx[3 + s])[: int(lay.count[3 + s].item())], tr.idx_down[s])
        else:
            assert all(int(lay.count[p].item()) == -7 for p in range(5))
        assert O.rel_err(to_host(hout), tr.hidden, 1.0) <= (TOL if same else 5e-2), flags


def test_moe_argument_errors(ctx):
    shape, cfg, w, K, V, h, widths = _setup("tiny_moe", 11)
    lay = M.DeviceMoeLayer(ctx, shape, w)
    hin = to_dev(h); hout = torch.zeros_like(hin)
    Kd, Vd = to_dev(K), to_dev(V)
    ks = tuple(O.keep_count(n, 50) for n in widths)
    with pytest.raises(B.AfError):
        lay.run(hin, hout, Kd, Vd, KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_TOPK, ks, reuse_mask=1))
    bad = B.MoeCfg(lay.cfg.base, 99, 2)
    with pytest.raises(B.AfError):
        ctx.decode_moe_layer(bad, lay.weights_struct(), hin, hout, Kd, Vd, KV_LEN, KV_CAP, KV_LEN,
                             M.select_cfg(B.AF_SEL_TOPK, ks), lay.sets_struct(), lay.route_struct())
    with pytest.raises(B.AfError):
        ctx.decode_moe_layer(lay.cfg, lay.weights_struct(), hin, hout, Kd, Vd, KV_LEN, KV_CAP, KV_LEN,
                             M.select_cfg(B.AF_SEL_TOPK, ks), lay.sets_struct(), B.MoeRoute())


@pytest.mark.parametrize("cols,n,E,slots", [(136, 64, 3, 2), (2752, 512, 4, 2), (520, 1000, 5, 3),
                                            (28672, 256, 2, 2), (4096, 1376, 4, 1)])
def test_expert_indexed_gemv(ctx, cols, n, E, slots):
    """af_select_gemv_experts_f16: slot s of the output multiplies by the matrix of expert
    sel[s]; widths that are not a multiple of the tile leave ragged slot edges."""
    g = np.random.default_rng(cols + n)
    Ws = [S.weight_matrix(cols + n, cols, n, "experts", e) for e in range(E)]
    x = S.activation(cols, S.channel_scales(cols, n, "experts"), "experts", 0)
    Wt_all = torch.empty((E, n, cols), dtype=torch.float16, device="cuda")
    for e in range(E):
        ctx.pack_inmajor_f16(to_dev(Ws[e]), Wt_all[e])
    ctx.synchronize()
    sel = g.choice(E, size=slots, replace=False).astype(np.int32)
    k = n // 2
    idx = O.select_topk(x, k)
    io = torch.zeros(n, dtype=torch.int32, device="cuda"); co = torch.zeros(1, dtype=torch.int32, device="cuda")
    y = ctx.select_gemv_experts_f16(Wt_all, to_dev(sel), slots, to_dev(x), sel_mode=B.AF_SEL_TOPK, k=k,
                                    idx_out=io, count_out=co, y_kind=B.AF_F32)
    ctx.synchronize()
    assert np.array_equal(to_host(io)[:k], idx)
    ref = np.concatenate([O.sparse_gemv(Ws[e], x, idx) for e in sel])
    assert O.rel_err(to_host(y), ref) <= 1e-4
    # scaled product added to a residual, threshold form without an index list
    res = S.activation(7, S.channel_scales(7, cols * slots, "experts-res"), "experts-res", 0)
    scale = np.array([0.375], np.float32)
    t = float(np.sort(np.abs(x.astype(np.float64)))[n // 2])
    y = ctx.select_gemv_experts_f16(Wt_all, to_dev(sel), slots, to_dev(x), sel_mode=B.AF_SEL_THRESHOLD, t=t,
                                    residual=to_dev(res), y_scale=to_dev(scale))
    ctx.synchronize()
    idx_t = O.select_threshold(x, t)
    ref = res.astype(np.float64) + 0.375 * np.concatenate([O.sparse_gemv(Ws[e], x, idx_t) for e in sel])
    assert O.rel_err(to_host(y), ref) <= TOL


@pytest.mark.parametrize("top", [1, 3])
def test_moe_other_top_counts(ctx, top):
    """One expert per token, and three of four: slot handling beyond the usual top-2."""
    shape, cfg, w, K, V, h, widths = _setup("tiny_moe", 13)
    ks = tuple(O.keep_count(n, 50) for n in widths)
    tr = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), KV_LEN, KV_LEN, O.SelectCfg(O.SEL_TOPK, ks), top=top)
    assert _margin_ok(tr)
    lay = M.DeviceMoeLayer(ctx, shape, w, top=top)
    hin = to_dev(h); hout = torch.zeros_like(hin)
    lay.run(hin, hout, to_dev(K), to_dev(V), KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_TOPK, ks))
    ctx.synchronize()
    assert to_host(lay.experts).tolist() == tr.experts.tolist()
    assert np.allclose(to_host(lay.weights), tr.weights, rtol=1e-4)
    same = all(np.array_equal(to_host(lay.idx[p])[: ks[p]], tr.idx[p]) for p in range(3))
    same &= all(np.array_equal(to_host(lay.idx[3 + s])[: ks[3]], tr.idx_down[s]) for s in range(top))
    assert O.rel_err(to_host(hout), tr.hidden, 1.0) <= (TOL if same else 5e-2)


def test_router_as_its_own_launch_gives_the_same_layer(ctx):
    """The router runs inside the gate|up launch by default; the stand-alone router kernel (used
    when that launch cannot take it) must lead to the same experts and the same layer output."""
    shape, cfg, w, K, V, h, widths = _setup("tiny_moe", 11)
    ks = tuple(O.keep_count(n, 50) for n in widths)
    lay = M.DeviceMoeLayer(ctx, shape, w)
    hin = to_dev(h)
    outs = []
    for separate in (False, True):
        ctx.set_option(B.AF_OPT_MOE_ROUTER_KERNEL, 1 if separate else 0)
        hout = torch.zeros_like(hin)
        lay.run(hin, hout, to_dev(K), to_dev(V), KV_LEN, KV_CAP, KV_LEN, M.select_cfg(B.AF_SEL_TOPK, ks))
        ctx.synchronize()
        ctx.set_option(B.AF_OPT_MOE_ROUTER_KERNEL, 0)
        outs.append((to_host(lay.experts).copy(), to_host(lay.weights).copy(), to_host(lay.logits).copy(),
                     to_host(hout).copy()))
    assert outs[0][0].tolist() == outs[1][0].tolist()
    assert np.allclose(outs[0][1], outs[1][1], rtol=1e-5) and np.allclose(outs[0][2], outs[1][2], rtol=1e-4, atol=1e-5)
    assert O.rel_err(outs[0][3], outs[1][3], 1.0) <= 1e-3
