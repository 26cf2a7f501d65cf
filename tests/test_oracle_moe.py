"""Pins for the oracle's mixture-of-experts block (the Mixtral-8x7B deployment the paper
reports).  The router is checked against a textbook formulation, the block against the dense
block it reduces to, and against a scalar re-statement on a toy."""
import math

import numpy as np
import pytest
from scipy.special import softmax

import synth_inputs as S
from oracle import activeflow_oracle as O


def _setup(shape_name="tiny_moe", seed=0, kv_len=7, cap=12):
    shape = S.MODEL_SHAPES[shape_name]
    w = S.moe_layer_weights(seed, shape, 0)
    K, V = S.kv_cache(seed, shape.n_kv_heads, cap, shape.head_dim, kv_len, shape.name, 0)
    h = S.activation(seed, S.channel_scales(seed, shape.d_model, shape.name), "hidden", 0)
    cfg = O.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn)
    widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
    return shape, cfg, w, K, V, h, widths, kv_len


def test_router_against_textbook_softmax_topk():
    g = np.random.default_rng(0)
    for E, top in ((8, 2), (4, 2), (5, 3), (3, 1)):
        Wr = (g.standard_normal((E, 64)) * 0.1).astype(np.float16)
        x = g.standard_normal(64).astype(np.float16)
        experts, weights, logits = O.moe_route(x, Wr, top)
        ref_logits = [math.fsum(float(Wr[e, j]) * float(x[j]) for j in range(64)) for e in range(E)]
        assert np.allclose(logits, ref_logits, rtol=1e-12, atol=1e-15)
        # softmax over all experts, keep the top, renormalise == softmax over the kept logits
        p = softmax(np.array(ref_logits))
        best = sorted(range(E), key=lambda e: (-ref_logits[e], e))[:top]
        assert experts.tolist() == best
        assert np.allclose(weights, p[best] / p[best].sum(), rtol=1e-12)
        assert abs(weights.sum() - 1.0) < 1e-12 and np.all(np.diff(weights) <= 0)


def test_router_ties_go_to_the_lower_expert():
    Wr = np.zeros((4, 8), np.float16); Wr[1, 0] = 1; Wr[3, 0] = 1; Wr[2, 0] = 0.5
    x = np.zeros(8, np.float16); x[0] = 2
    experts, weights, _ = O.moe_route(x, Wr, 2)
    assert experts.tolist() == [1, 3] and np.allclose(weights, [0.5, 0.5])
    experts, _, _ = O.moe_route(np.zeros(8, np.float16), Wr, 2)       # all logits equal
    assert experts.tolist() == [0, 1]


def test_identical_experts_reduce_to_the_dense_block():
    """With every expert equal, the weighted sum of expert outputs is the one expert's output
    (router weights sum to 1), so the block equals decode_layer up to the extra fp16 rounding
    of the residual stream between the two slots."""
    shape, cfg, w, K, V, h, widths, kv_len = _setup()
    for key in ("Wgate", "Wup", "Wdown"):
        w[key] = [w[key][0]] * shape.n_experts
    sel = O.SelectCfg(O.SEL_TOPK, tuple(O.keep_count(n, 50) for n in widths))
    tr = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), kv_len, kv_len, sel)
    wd = dict(w); wd["Wgate"], wd["Wup"], wd["Wdown"] = w["Wgate"][0], w["Wup"][0], w["Wdown"][0]
    dense = O.decode_layer(cfg, wd, h, K.copy(), V.copy(), kv_len, kv_len, sel)
    assert np.array_equal(tr.h_mid, dense.h_mid) and np.array_equal(tr.idx[2], dense.idx[2])
    assert np.array_equal(tr.x_down[0], dense.x[3]) and np.array_equal(tr.x_down[1], dense.x[3])
    assert np.array_equal(tr.idx_down[0], dense.idx[3])
    a, b = tr.hidden.astype(np.float64), dense.hidden.astype(np.float64)
    assert np.max(np.abs(a - b)) <= 2.0 ** -10 * np.maximum(np.abs(b), 1e-3).max()
    assert O.rel_err(tr.hidden, dense.hidden) <= 2e-3


def test_block_against_scalar_restatement():
    """The feed-forward half re-stated with Python floats from the trace's own h_mid."""
    shape, cfg, w, K, V, h, widths, kv_len = _setup(seed=3)
    ks = tuple(O.keep_count(n, 70) for n in widths)
    tr = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), kv_len, kv_len, O.SelectCfg(O.SEL_TOPK, ks))
    d, f = shape.d_model, shape.d_ffn
    hm = [float(v) for v in tr.h_mid]
    ms = math.fsum(v * v for v in hm) / d
    x2 = np.array([hm[j] / math.sqrt(ms + cfg.rms_eps) * float(w["g_ffn"][j]) for j in range(d)]).astype(np.float16)
    assert np.array_equal(x2, tr.x[2])
    keep = sorted(sorted(range(d), key=lambda j: (-abs(float(x2[j])), j))[:ks[2]])
    assert keep == tr.idx[2].tolist()
    logits = [math.fsum(float(w["Wr"][e, j]) * float(x2[j]) for j in range(d)) for e in range(shape.n_experts)]
    best = sorted(range(shape.n_experts), key=lambda e: (-logits[e], e))[:2]
    assert best == tr.experts.tolist()
    zs = [math.exp(logits[e] - logits[best[0]]) for e in best]
    wts = [z / sum(zs) for z in zs]
    assert np.allclose(wts, tr.weights, rtol=1e-12)
    hcur = tr.h_mid.astype(np.float64)
    rows = [0, 5, d - 1]
    for s, e in enumerate(best):
        gate = [math.fsum(float(w["Wgate"][e][o, j]) * float(x2[j]) for j in keep) for o in range(f)]
        up = [math.fsum(float(w["Wup"][e][o, j]) * float(x2[j]) for j in keep) for o in range(f)]
        g16 = np.array(gate).astype(np.float16).astype(np.float64); u16 = np.array(up).astype(np.float16).astype(np.float64)
        act = (g16 / (1.0 + np.exp(-g16)) * u16).astype(np.float16)
        assert np.array_equal(act, tr.x_down[s])
        keep3 = sorted(sorted(range(f), key=lambda j: (-abs(float(act[j])), j))[:ks[3]])
        assert keep3 == tr.idx_down[s].tolist()
        nxt = hcur.copy()
        for o in rows:
            y = math.fsum(float(w["Wdown"][e][o, j]) * float(act[j]) for j in keep3)
            nxt[o] = float(np.float16(hcur[o] + wts[s] * y))
            assert nxt[o] == float(tr.h_slots[s][o])
        hcur = tr.h_slots[s].astype(np.float64)
    assert np.array_equal(tr.hidden, tr.h_slots[-1])


def test_threshold_and_dense_modes_and_kv_append():
    shape, cfg, w, K, V, h, widths, kv_len = _setup(seed=4)
    K1, V1 = K.copy(), V.copy()
    dense = O.decode_moe_layer(cfg, w, h, K1, V1, kv_len, kv_len, O.SelectCfg(O.SEL_DENSE))
    assert all(len(dense.idx[p]) == widths[p] for p in range(4))
    assert np.array_equal(K1[:, kv_len], dense.k_new) and np.array_equal(V1[:, kv_len], dense.v_new)
    # a threshold below every magnitude is the dense block; one above everything leaves only the residual
    lo = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), kv_len, kv_len, O.SelectCfg(O.SEL_THRESHOLD, t=(-1,) * 4))
    assert np.array_equal(lo.hidden, dense.hidden)
    hi = O.decode_moe_layer(cfg, w, h, K.copy(), V.copy(), kv_len, kv_len, O.SelectCfg(O.SEL_THRESHOLD, t=(1e9,) * 4))
    assert np.array_equal(hi.hidden, np.asarray(h, np.float16))
