"""af_decode_layer_batch: B tokens through one decoder layer, the linear operators over the
union of the tokens' active sets.  Every token is judged on its own against the oracle's
single-token operators (the batched layer computes, per token, what the single-token layer
computes): stage by stage on the bits the GPU fed into each stage (strict floor), index sets
bit for bit against the definition, and end to end against the oracle's own chain."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import activeflow_oracle as O
from paper_2504_08378_amd import binding as B
from paper_2504_08378_amd import model as M
from gpu_util import TAP_NAMES, ctx, teacher_forced_layer_errors, to_dev, to_host  # noqa: F401

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _ocfg(shape):
    return O.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn)


def _widths(shape):
    return (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)


def _batch_taps(ctx, shape, Bt):
    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    qdim, qkv_out = shape.n_heads * hd, (shape.n_heads + 2 * shape.n_kv_heads) * hd
    sizes = (d, qkv_out, qdim, d, d, 2 * f, f)
    full = {n: to_host(ctx.layer_tap(i, s * Bt)).reshape(Bt, s) for i, (n, s) in enumerate(zip(TAP_NAMES, sizes))}
    return [{n: full[n][b] for n in TAP_NAMES} for b in range(Bt)]


def _run_batch(ctx, shape, w, H, caches, kv_lens, kv_cap, sel):
    Bt = H.shape[0]
    lay = M.DeviceLayer(ctx, shape, w)
    widths = _widths(shape)
    idx = [torch.zeros((Bt, n), dtype=torch.int32, device="cuda") for n in widths]
    cnt = [torch.zeros(Bt, dtype=torch.int32, device="cuda") for _ in widths]
    sets = B.IdxSets()
    for p in range(4):
        sets.idx[p] = idx[p].data_ptr()
        sets.count[p] = cnt[p].data_ptr()
    Kd = [to_dev(K) for K, _ in caches]
    Vd = [to_dev(V) for _, V in caches]
    hin = to_dev(H)
    hout = torch.zeros_like(hin)
    un = torch.zeros(4, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    cfg = M.layer_cfg(shape)
    ctx.decode_layer_batch(cfg, lay.struct(), hin, hout, Kd, Vd, kv_lens, kv_cap, kv_lens, sel, sets, un)
    ctx.synchronize()
    assert ctx.last_device_error() == 0
    return to_host(hout), [to_host(t) for t in idx], [to_host(t) for t in cnt], to_host(un), Kd, Vd


def _check_tokens(ctx, shape, w, H, caches, kv_lens, osel, out, idx, cnt, un, Kd, Vd, free_running=True):
    Bt = H.shape[0]
    cfg = _ocfg(shape)
    taps = _batch_taps(ctx, shape, Bt)
    nh, nkv, hd = shape.n_heads, shape.n_kv_heads, shape.head_dim
    for b in range(Bt):
        K, V = caches[b]
        n_b = [int(cnt[p][b]) for p in range(4)]
        idx_b = [idx[p][b, : n_b[p]] for p in range(4)]
        errs, own = teacher_forced_layer_errors(O, cfg, w, H[b], K, V, kv_lens[b], kv_lens[b], taps[b], out[b],
                                                idx_b, osel)
        for p in range(4):   # each token's set is the definition applied to that token's own input
            assert np.array_equal(idx_b[p], own[p]), (b, p)
        assert max(errs.values()) <= TOL, (b, errs)
        # the token's key / value went into its own cache at its own length
        qkv = taps[b]["qkv"]
        k_new = O.round_f16(O.rope(qkv[nh * hd:(nh + nkv) * hd].reshape(nkv, hd), kv_lens[b], 10000.0))
        assert O.rel_err(to_host(Kd[b])[:, kv_lens[b], :], k_new) <= TOL, b
        assert np.array_equal(to_host(Vd[b])[:, kv_lens[b], :], qkv[(nh + nkv) * hd:].reshape(nkv, hd)), b
        if free_running:   # and the whole layer against the oracle's own chain for this token
            tr = O.decode_layer(cfg, w, H[b], K.copy(), V.copy(), kv_lens[b], kv_lens[b], osel)
            assert np.array_equal(idx_b[0], tr.idx[0]), b   # same input bits at the first point
            assert O.rel_err(out[b], tr.hidden, 1.0) <= TOL, b
    # the union the operators ran over
    for p in range(4):
        U = O.union_indices([idx[p][b, : int(cnt[p][b])] for b in range(Bt)])
        assert int(un[p]) == len(U), p


def _inputs(shape, Bt, kv_cap, kv_lens, seed=0):
    w = S.layer_weights(seed, shape, 0)
    sc = S.channel_scales(seed, shape.d_model, shape.name)
    H = np.stack([S.activation(seed, sc, "hidden", b) for b in range(Bt)])
    caches = [S.kv_cache(seed, shape.n_kv_heads, kv_cap, shape.head_dim, kv_lens[b], shape.name, b)
              for b in range(Bt)]
    return w, H, caches


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_gqa"])
@pytest.mark.parametrize("Bt", [1, 2, 3, 4, 8])
def test_batch_layer_topk(ctx, shape_name, Bt):
    shape = S.MODEL_SHAPES[shape_name]
    kv_cap = 96
    kv_lens = [(7 + 11 * b) % 80 for b in range(Bt)]   # every token at its own length
    w, H, caches = _inputs(shape, Bt, kv_cap, kv_lens)
    ks = tuple(O.keep_count(n, 50) for n in _widths(shape))
    res = _run_batch(ctx, shape, w, H, caches, kv_lens, kv_cap, M.select_cfg(B.AF_SEL_TOPK, ks))
    assert all((res[2][p] == ks[p]).all() for p in range(4))
    _check_tokens(ctx, shape, w, H, caches, kv_lens, O.SelectCfg(O.SEL_TOPK, ks), *res)


@pytest.mark.parametrize("Bt", [1, 4, 8])
def test_batch_layer_threshold(ctx, Bt):
    """Threshold selection: the tokens keep different numbers of channels."""
    shape = S.MODEL_SHAPES["tiny_gqa"]
    kv_cap = 64
    kv_lens = [3 + 5 * b for b in range(Bt)]
    w, H, caches = _inputs(shape, Bt, kv_cap, kv_lens, seed=1)
    t = (0.7, 0.02, 0.7, 0.01)
    res = _run_batch(ctx, shape, w, H, caches, kv_lens, kv_cap, M.select_cfg(B.AF_SEL_THRESHOLD, t=t))
    if Bt > 1:
        assert len({int(c) for c in res[2][0]}) > 1
    # free-running comparison left out: a threshold can fall between two values that differ in the
    # last bit between the two chains; the stage-by-stage check uses the same bits on both sides
    _check_tokens(ctx, shape, w, H, caches, kv_lens, O.SelectCfg(O.SEL_THRESHOLD, t=t), *res, free_running=False)


def test_batch_of_identical_tokens_equals_single_token_layer(ctx):
    """B copies of one token (same cache, same position): every row equals row 0, the union has k
    channels, and the result agrees with af_decode_layer on that token."""
    shape = S.MODEL_SHAPES["tiny"]
    kv_cap, kv_len, Bt = 64, 21, 4
    w, H1, caches1 = _inputs(shape, 1, kv_cap, [kv_len])
    H = np.repeat(H1, Bt, axis=0)
    caches = [caches1[0]] * Bt
    ks = tuple(O.keep_count(n, 50) for n in _widths(shape))
    out, idx, cnt, un, _, _ = _run_batch(ctx, shape, w, H, caches, [kv_len] * Bt, kv_cap,
                                         M.select_cfg(B.AF_SEL_TOPK, ks))
    assert all(np.array_equal(out[0], out[b]) for b in range(Bt))
    assert [int(v) for v in un] == list(ks)
    K, V = caches1[0]
    st = M.DeviceStack(ctx, shape, [M.DeviceLayer(ctx, shape, w)], [(K.copy(), V.copy())], kv_cap)
    hin = to_dev(H1[0]); hout = torch.zeros_like(hin)
    st.layer(0, hin, hout, kv_len, kv_len, M.select_cfg(B.AF_SEL_TOPK, ks))
    ctx.synchronize()
    single = to_host(hout)
    for p in range(4):
        assert np.array_equal(idx[p][0, : ks[p]], st.sets[0].fetch(p, ks[p])), p
    assert O.rel_err(out[0], single.astype(np.float64), 1.0) <= TOL


def test_batch_layer_rejects_what_it_cannot_run(ctx):
    shape = S.MODEL_SHAPES["tiny"]
    w, H, caches = _inputs(shape, 2, 32, [4, 5])
    ks = tuple(O.keep_count(n, 50) for n in _widths(shape))
    with pytest.raises(B.AfError):   # a position beyond the cache
        _run_batch(ctx, shape, w, H, caches, [4, 32], 32, M.select_cfg(B.AF_SEL_TOPK, ks))
    with pytest.raises(B.AfError):   # reuse is a single-token feature
        _run_batch(ctx, shape, w, H, caches, [4, 5], 32, M.select_cfg(B.AF_SEL_TOPK, ks, reuse_mask=1))


@pytest.mark.parametrize("Bt", [4])
def test_batch_layer_70b_shape(ctx, Bt):
    """BASELINE config 4 as a whole layer: 70B shape (64 query / 8 key-value heads), B tokens, each
    selecting its own top 50 %; every stage of every token at the strict floor."""
    shape = S.MODEL_SHAPES["70b"]
    kv_cap, kv_lens = 528, [512, 300, 17, 450][:Bt]
    w = S.layer_weights(0, shape, 0, threads=8)
    sc = S.channel_scales(0, shape.d_model, shape.name)
    H = np.stack([S.activation(0, sc, "hidden", b) for b in range(Bt)])
    caches = [S.kv_cache(0, shape.n_kv_heads, kv_cap, shape.head_dim, kv_lens[b], shape.name, b) for b in range(Bt)]
    ks = tuple(O.keep_count(n, 50) for n in _widths(shape))
    res = _run_batch(ctx, shape, w, H, caches, kv_lens, kv_cap, M.select_cfg(B.AF_SEL_TOPK, ks))
    _check_tokens(ctx, shape, w, H, caches, kv_lens, O.SelectCfg(O.SEL_TOPK, ks), *res, free_running=False)


def _random_batch_cases(count, seed=11):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        hd = int(rng.choice([64, 128]))
        n_kv = int(rng.choice([1, 2, 4]))
        nh = n_kv * int(rng.choice([1, 2, 4]))
        cases.append((i, 32 * int(rng.integers(2, 24)), nh, n_kv, hd, 32 * int(rng.integers(3, 60)),
                      int(rng.integers(1, 9)), int(rng.choice([0, 30, 50, 70, 90])), str(rng.choice(["topk", "threshold"]))))
    return cases


@pytest.mark.parametrize("i,d,nh,n_kv,hd,f,Bt,sp,rule", _random_batch_cases(10))
def test_batch_layer_random_shapes(ctx, i, d, nh, n_kv, hd, f, Bt, sp, rule):
    """Seeded shapes off the beaten path (odd widths, query width != model width, any batch size
    from 1 to 8, caches of unrelated lengths), every token stage by stage."""
    shape = S.ModelShape(f"brand{i}", 1, d, nh, n_kv, hd, f)
    rng = np.random.default_rng(1000 + i)
    kv_cap = 160
    kv_lens = [int(v) for v in rng.integers(0, kv_cap - 1, size=Bt)]
    w, H, caches = _inputs(shape, Bt, kv_cap, kv_lens, seed=200 + i)
    ks = tuple(O.keep_count(n, sp) for n in _widths(shape))
    if rule == "topk":
        gsel, osel = M.select_cfg(B.AF_SEL_TOPK, ks), O.SelectCfg(O.SEL_TOPK, ks)
    else:   # thresholds near the same keep rate, from the first token's activations in the oracle
        K, V = caches[0]
        tr = O.decode_layer(_ocfg(shape), w, H[0], K.copy(), V.copy(), kv_lens[0], kv_lens[0], O.SelectCfg(O.SEL_TOPK, ks))
        ts = tuple(float(np.float32(np.sort(np.abs(tr.x[p].astype(np.float64)))[len(tr.x[p]) - max(ks[p], 1)]))
                   for p in range(4))
        gsel, osel = M.select_cfg(B.AF_SEL_THRESHOLD, t=ts), O.SelectCfg(O.SEL_THRESHOLD, t=ts)
    res = _run_batch(ctx, shape, w, H, caches, kv_lens, kv_cap, gsel)
    _check_tokens(ctx, shape, w, H, caches, kv_lens, osel, *res, free_running=False)
