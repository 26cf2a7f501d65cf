"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import pytest
import torch


def to_dev(a, device="cuda"):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(device)
    torch.cuda.synchronize()
    return t


def to_host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


@pytest.fixture(scope="module")
def ctx():
    from paper_2504_08378_amd import binding as B
    c = B.Context(0)
    yield c
    c.close()


# ---- teacher-forced layer check ----------------------------------------------------------------
TAP_NAMES = ("x_qkv", "qkv", "attn", "h_mid", "x_gateup", "gateup", "x_down")


def layer_taps(ctx, shape):
    """The seven inter-operator tensors of the last decode_layer call, as NumPy fp16."""
    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    qdim, qkv_out = shape.n_heads * hd, (shape.n_heads + 2 * shape.n_kv_heads) * hd
    sizes = (d, qkv_out, qdim, d, d, 2 * f, f)
    return {n: to_host(ctx.layer_tap(i, s)) for i, (n, s) in enumerate(zip(TAP_NAMES, sizes))}


def teacher_forced_layer_errors(O, cfg, w, h_in, K, V, kv_len, pos, taps, h_out, idx_gpu, sel,
                                weights_q4=False):
    """Every stage of a layer judged on its own: the oracle operator is applied to the bits the
    GPU itself fed into that stage (the tap of the stage before and the GPU's index set), so a
    last-bit difference that entered earlier cannot leak into the comparison and the strict
    error measure (floor 0.01 rms) applies everywhere.  `w` holds the oracle-side weights
    (fp16 matrices, or (nibbles, scales) pairs).  Returns ({stage: rel_err}, {point: the set
    the definition selects on the GPU's own input})."""
    nh, nkv, hd, f = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn
    r16 = O.round_f16
    lin = lambda name, x, idx: O._linear(w[name], x, idx, weights_q4)
    errs, own = {}, {}
    x0, qkv, attn, hmid, x2, gu, x3 = (taps[n] for n in TAP_NAMES)
    errs["x_qkv"] = O.rel_err(x0, r16(O.rmsnorm(h_in, w["g_attn"], cfg.rms_eps)))
    own[0] = O._select(x0, 0, sel, None)
    i0, i1, i2, i3 = idx_gpu
    errs["qkv"] = O.rel_err(qkv, r16(np.concatenate([lin("Wq", x0, i0), lin("Wk", x0, i0), lin("Wv", x0, i0)])))
    q16 = qkv[: nh * hd].reshape(nh, hd)
    k16 = qkv[nh * hd: (nh + nkv) * hd].reshape(nkv, hd)
    v16 = qkv[(nh + nkv) * hd:].reshape(nkv, hd)
    Kc, Vc = K.copy(), V.copy()
    Kc[:, kv_len, :] = r16(O.rope(k16, pos, cfg.rope_theta))
    Vc[:, kv_len, :] = v16
    errs["attn"] = O.rel_err(attn, r16(O.attention_decode(O.rope(q16, pos, cfg.rope_theta), Kc, Vc,
                                                          kv_len + 1).reshape(-1)))
    own[1] = O._select(attn, 1, sel, None)
    errs["h_mid"] = O.rel_err(hmid, r16(np.asarray(h_in).astype(np.float64) + lin("Wo", attn, i1)))
    errs["x_gateup"] = O.rel_err(x2, r16(O.rmsnorm(hmid, w["g_ffn"], cfg.rms_eps)))
    own[2] = O._select(x2, 2, sel, None)
    errs["gateup"] = O.rel_err(gu, r16(np.concatenate([lin("Wgate", x2, i2), lin("Wup", x2, i2)])))
    errs["x_down"] = O.rel_err(x3, r16(O.silu(gu[:f]) * gu[f:].astype(np.float64)))
    own[3] = O._select(x3, 3, sel, None)
    errs["hidden"] = O.rel_err(h_out, r16(hmid.astype(np.float64) + lin("Wdown", x3, i3)))
    return errs, own
