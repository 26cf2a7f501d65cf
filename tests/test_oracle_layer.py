"""Pins for the oracle's glue operators, decode_layer and decode_stack (block structure:
Fig. "simplified transformer layer", Section 2.2; cross-layer reuse: Section 3).

The dense block is re-implemented here in a different formulation (complex-number rotary
embedding, einsum attention with scipy's softmax, expit-based SiLU, no intermediate fp16
rounding); special cases pin each glue operator by closed form."""
import numpy as np
import pytest
from scipy.special import expit, softmax

import synth_inputs as S
from oracle import activeflow_oracle as O


def _cfg(shape):
    return O.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn)


def _inputs(shape, seed=0, kv_len=9, cap=16):
    w = S.layer_weights(seed, shape, 0)
    sc = S.channel_scales(seed, shape.d_model, shape.name)
    h = S.activation(seed, sc, "hidden", 0)
    K, V = S.kv_cache(seed, shape.n_kv_heads, cap, shape.head_dim, kv_len, shape.name, 0)
    return w, h, K, V


def _textbook_dense_block(cfg, w, h, K, V, kv_len, pos):
    """Plain fp64 pre-norm block, written independently of the oracle."""
    f8 = lambda a: np.asarray(a).astype(np.float64)
    d, nh, nkv, hd = cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    h = f8(h)
    xn = h * f8(w["g_attn"]) / np.sqrt((h ** 2).sum() / d + cfg.rms_eps)
    q = np.einsum("oi,i->o", f8(w["Wq"]), xn).reshape(nh, hd)
    k = np.einsum("oi,i->o", f8(w["Wk"]), xn).reshape(nkv, hd)
    v = np.einsum("oi,i->o", f8(w["Wv"]), xn).reshape(nkv, hd)
    freqs = np.exp(-np.log(cfg.rope_theta) * np.arange(0, hd, 2) / hd)
    rot = np.exp(1j * pos * freqs)

    def rotary(t):                      # pair (i, i + hd/2) as one complex number
        z = (t[:, : hd // 2] + 1j * t[:, hd // 2:]) * rot
        return np.concatenate([z.real, z.imag], axis=1)

    q, k = rotary(q), rotary(k)
    Kf = np.concatenate([f8(K[:, :kv_len]), k[:, None, :]], axis=1)          # [nkv][T][hd]
    Vf = np.concatenate([f8(V[:, :kv_len]), v[:, None, :]], axis=1)
    rep = nh // nkv
    Kf, Vf = np.repeat(Kf, rep, axis=0), np.repeat(Vf, rep, axis=0)
    p = softmax(np.einsum("hd,htd->ht", q, Kf) / np.sqrt(hd), axis=1)
    a = np.einsum("ht,htd->hd", p, Vf).reshape(-1)
    h1 = h + np.einsum("oi,i->o", f8(w["Wo"]), a)
    x2 = h1 * f8(w["g_ffn"]) / np.sqrt((h1 ** 2).sum() / d + cfg.rms_eps)
    g = np.einsum("oi,i->o", f8(w["Wgate"]), x2)
    u = np.einsum("oi,i->o", f8(w["Wup"]), x2)
    return h1 + np.einsum("oi,i->o", f8(w["Wdown"]), g * expit(g) * u)


@pytest.mark.parametrize("name", ["tiny", "tiny_gqa"])
def test_dense_mode_matches_textbook_block(name):
    shape = S.MODEL_SHAPES[name]
    cfg = _cfg(shape)
    w, h, K, V = _inputs(shape)
    ref = _textbook_dense_block(cfg, w, h, K, V, 9, 9)
    tr = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9, O.SelectCfg(mode=O.SEL_DENSE))
    # the oracle rounds inter-operator tensors to fp16 (2^-11 each); a dropped term, a wrong
    # sign or a transposed operand would be off by O(1)
    diff = np.abs(tr.hidden.astype(np.float64) - ref)
    assert np.all(diff < 2e-3 * np.maximum(np.abs(ref), np.sqrt(np.mean(ref ** 2))))
    assert O.rel_err(tr.hidden, ref) < 2e-2
    for p in range(4):
        assert tr.idx[p].tolist() == list(range(len(tr.x[p])))


def test_sparse_mode_is_masked_textbook_block():
    """With the masks applied by hand (zeroing dropped activations before each dense
    product) the textbook operators reproduce the sparse layer."""
    shape = S.MODEL_SHAPES["tiny"]
    cfg = _cfg(shape)
    w, h, K, V = _inputs(shape)
    ks = (128, 128, 128, 344)
    tr = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9, O.SelectCfg(mode=O.SEL_TOPK, k=ks))
    f8 = lambda a: np.asarray(a).astype(np.float64)
    for p, (x, names, got) in enumerate([
        (tr.x[0], ("Wq", "Wk", "Wv"), tr.qkv),
        (tr.x[2], ("Wgate", "Wup"), tr.gateup),
    ]):
        p = 0 if names[0] == "Wq" else 2
        xm = f8(x).copy()
        drop = np.setdiff1d(np.arange(len(xm)), tr.idx[p])
        xm[drop] = 0.0
        exp = np.concatenate([np.einsum("oi,i->o", f8(w[nm]), xm) for nm in names])
        assert np.array_equal(got, exp.astype(np.float16))
        assert len(tr.idx[p]) == ks[p]
    # residual adds: o and down
    xm = f8(tr.x[1]).copy(); xm[np.setdiff1d(np.arange(len(xm)), tr.idx[1])] = 0
    assert np.array_equal(tr.h_mid, (f8(h) + np.einsum("oi,i->o", f8(w["Wo"]), xm)).astype(np.float16))
    xm = f8(tr.x[3]).copy(); xm[np.setdiff1d(np.arange(len(xm)), tr.idx[3])] = 0
    assert np.array_equal(tr.hidden, (f8(tr.h_mid) + np.einsum("oi,i->o", f8(w["Wdown"]), xm)).astype(np.float16))
    # x3 is silu(gate) * up on the fp16 gate/up values
    f = cfg.d_ffn
    g, u = f8(tr.gateup[:f]), f8(tr.gateup[f:])
    assert np.array_equal(tr.x[3], (g * expit(g) * u).astype(np.float16))


def test_full_k_equals_dense_and_reuse_of_own_sets():
    shape = S.MODEL_SHAPES["tiny"]
    cfg = _cfg(shape)
    w, h, K, V = _inputs(shape)
    dense = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9, O.SelectCfg(mode=O.SEL_DENSE))
    full = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9,
                          O.SelectCfg(mode=O.SEL_TOPK, k=(256, 256, 256, 688)))
    assert np.array_equal(dense.hidden, full.hidden)
    ks = (100, 128, 77, 300)
    a = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9, O.SelectCfg(mode=O.SEL_TOPK, k=ks))
    b = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9,
                       O.SelectCfg(mode=O.SEL_TOPK, k=ks, reuse_mask=0b1111), sets=a.idx)
    assert np.array_equal(a.hidden, b.hidden)
    # a forced set is used as given, even if it is not what the input would select
    forced = [np.arange(0, 200, 2, dtype=np.int32)] + a.idx[1:]
    c = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9,
                       O.SelectCfg(mode=O.SEL_TOPK, k=ks, reuse_mask=0b0001), sets=forced)
    assert c.idx[0].tolist() == forced[0].tolist() and not np.array_equal(c.qkv, a.qkv)
    # threshold mode: same sets as top-k when t sits between the k-th and (k+1)-th magnitude
    ts = []
    for p in range(4):
        m = np.sort(np.abs(a.x[p].astype(np.float64)))[::-1]
        ts.append(float(m[ks[p]]) if m[ks[p] - 1] > m[ks[p]] else None)
    if all(t is not None for t in ts):
        th = O.decode_layer(cfg, w, h, K.copy(), V.copy(), 9, 9, O.SelectCfg(mode=O.SEL_THRESHOLD, t=tuple(ts)))
        assert np.array_equal(th.hidden, a.hidden)


def test_kv_append_and_gqa_expansion():
    shape = S.MODEL_SHAPES["tiny_gqa"]
    cfg = _cfg(shape)
    w, h, K, V = _inputs(shape)
    K1, V1 = K.copy(), V.copy()
    ks = (256, 256, 256, 688)
    tr = O.decode_layer(cfg, w, h, K1, V1, 9, 9, O.SelectCfg(mode=O.SEL_TOPK, k=ks))
    assert np.array_equal(K1[:, 9], tr.k_new) and np.array_equal(V1[:, 9], tr.v_new)
    assert np.array_equal(K1[:, :9], K[:, :9]) and np.all(K1[:, 10:] == 0)
    # grouped-query attention == multi-head attention on repeated kv heads
    rep = shape.n_heads // shape.n_kv_heads
    q = np.random.default_rng(0).standard_normal((shape.n_heads, shape.head_dim))
    a = O.attention_decode(q, K1, V1, 10)
    b = O.attention_decode(q, np.repeat(K1, rep, axis=0), np.repeat(V1, rep, axis=0), 10)
    assert np.array_equal(a, b)


def test_glue_closed_forms():
    g = np.random.default_rng(1)
    # rmsnorm: constant vector -> sign * gain (eps -> 0)
    gain = (1 + 0.1 * g.standard_normal(8)).astype(np.float16)
    assert np.allclose(O.rmsnorm(np.full(8, -3.0, np.float16), gain, 0.0), -gain.astype(np.float64))
    h = g.standard_normal(64).astype(np.float16)
    y = O.rmsnorm(h, np.ones(64, np.float16), 0.0)
    assert abs(np.mean(y * y) - 1.0) < 1e-12
    # rope: identity at pos 0, norm preserving, scores depend on the position difference only
    v = g.standard_normal((3, 64)); u = g.standard_normal((3, 64))
    assert np.array_equal(O.rope(v, 0, 10000.0), v)
    assert np.allclose(np.linalg.norm(O.rope(v, 77, 10000.0), axis=1), np.linalg.norm(v, axis=1))
    s1 = np.sum(O.rope(v, 100, 10000.0) * O.rope(u, 90, 10000.0), axis=1)
    s2 = np.sum(O.rope(v, 15, 10000.0) * O.rope(u, 5, 10000.0), axis=1)
    assert np.allclose(s1, s2)
    # first pair rotates by exactly pos radians (frequency theta^0 = 1)
    e = np.zeros((1, 64)); e[0, 0] = 1.0
    r = O.rope(e, 2, 10000.0)
    assert np.allclose([r[0, 0], r[0, 32]], [np.cos(2.0), np.sin(2.0)])
    # attention: one key -> its value; identical keys -> mean of the values
    K = g.standard_normal((2, 5, 8)).astype(np.float16); V = g.standard_normal((2, 5, 8)).astype(np.float16)
    q = g.standard_normal((2, 8))
    assert np.allclose(O.attention_decode(q, K, V, 1), V[:, 0].astype(np.float64))
    Kc = np.repeat(K[:, :1], 5, axis=1)
    assert np.allclose(O.attention_decode(q, Kc, V, 5), V.astype(np.float64).mean(axis=1))
    # a dominant key takes all the weight
    Kd = np.zeros((1, 4, 8), np.float16); Kd[0, 2] = 100.0
    qd = np.ones((1, 8))
    Vd = g.standard_normal((1, 4, 8)).astype(np.float16)
    assert np.allclose(O.attention_decode(qd, Kd, Vd, 4), Vd[:, 2].astype(np.float64))
    # silu
    assert O.silu(np.array([0.0]))[0] == 0.0 and abs(O.silu(np.array([30.0]))[0] - 30.0) < 1e-10
    assert np.allclose(O.silu(np.array([-1.0, 2.0])), [-1.0 / (1 + np.e), 2.0 / (1 + np.exp(-2.0))])


def test_stack_reuse_groups():
    shape = S.MODEL_SHAPES["tiny"]
    cfg = _cfg(shape)
    L = 4
    layers = [S.layer_weights(0, shape, l) for l in range(L)]
    sc = S.channel_scales(0, shape.d_model, shape.name)
    h = S.activation(0, sc, "hidden", 0)
    kv = [S.kv_cache(0, shape.n_kv_heads, 16, shape.head_dim, 9, shape.name, l) for l in range(L)]
    mk = lambda: ([k.copy() for k, _ in kv], [v.copy() for _, v in kv])
    sel = O.SelectCfg(mode=O.SEL_TOPK, k=(128, 128, 128, 344))

    # by hand: chain decode_layer
    Ks, Vs = mk()
    hh, manual = h, []
    for l in range(L):
        tr = O.decode_layer(cfg, layers[l], hh, Ks[l], Vs[l], 9, 9, sel)
        manual.append(tr); hh = tr.hidden
    Ks, Vs = mk()
    t1, _ = O.decode_stack(cfg, layers, h, Ks, Vs, 9, 9, sel, group=1)
    Ks, Vs = mk()
    t2, _ = O.decode_stack(cfg, layers, h, Ks, Vs, 9, 9, sel, group=4, reuse_points=0)
    for l in range(L):
        assert np.array_equal(t1[l].hidden, manual[l].hidden)
        assert np.array_equal(t2[l].hidden, manual[l].hidden)

    # group of 4, all four points reused: followers carry the leader's sets
    Ks, Vs = mk()
    t3, ov = O.decode_stack(cfg, layers, h, Ks, Vs, 9, 9, sel, group=4, reuse_points=0b1111, want_overlap=True)
    assert np.array_equal(t3[0].hidden, manual[0].hidden)
    for l in range(1, L):
        for p in range(4):
            assert np.array_equal(t3[l].idx[p], t3[0].idx[p])
            own = O.select_topk(t3[l].x[p], sel.k[p])
            assert ov[l][p] == len(set(own.tolist()) & set(t3[0].idx[p].tolist())) / sel.k[p]
    assert ov[0] == [None] * 4
    # only qkv and gate/up reused: o and down select for themselves
    Ks, Vs = mk()
    t4, ov4 = O.decode_stack(cfg, layers, h, Ks, Vs, 9, 9, sel, group=2, reuse_points=0b0101, want_overlap=True)
    assert np.array_equal(t4[1].idx[0], t4[0].idx[0]) and np.array_equal(t4[3].idx[2], t4[2].idx[2])
    assert np.array_equal(t4[1].idx[1], O.select_topk(t4[1].x[1], 128))
    assert ov4[1][1] is None and ov4[1][0] is not None and ov4[2] == [None] * 4


def test_overlap_is_one_when_blocks_add_nothing():
    """With zero o/down matrices the residual stream never changes, so (equal gains) the
    follower layers would pick exactly the leader's qkv set."""
    shape = S.MODEL_SHAPES["tiny"]
    cfg = _cfg(shape)
    base = S.layer_weights(0, shape, 0)
    layers = []
    for l in range(3):
        w = dict(S.layer_weights(0, shape, l))
        w["Wo"] = np.zeros_like(w["Wo"]); w["Wdown"] = np.zeros_like(w["Wdown"])
        w["g_attn"] = base["g_attn"]
        layers.append(w)
    sc = S.channel_scales(0, shape.d_model, shape.name)
    h = S.activation(0, sc, "hidden", 0)
    kv = [S.kv_cache(0, shape.n_kv_heads, 16, shape.head_dim, 9, shape.name, l) for l in range(3)]
    sel = O.SelectCfg(mode=O.SEL_TOPK, k=(128, 128, 128, 344))
    tr, ov = O.decode_stack(cfg, layers, h, [k for k, _ in kv], [v for _, v in kv], 9, 9, sel,
                            group=3, reuse_points=0b0001, want_overlap=True)
    assert ov[1][0] == 1.0 and ov[2][0] == 1.0
    assert np.array_equal(tr[2].hidden, h)
