"""CPU oracle for the active-weight decode path (TEST INFRASTRUCTURE ONLY).

This file is a plain, slow, fp64 NumPy statement of what the HIP library must
compute.  It is the yardstick for parity tests, the smoke check and the
`cpu_baseline` leg of the benchmark; the product path never imports it, and it
imports nothing from the product.  It shares no code, tables or helpers with
the HIP kernels.

What it follows (ActiveFlow, arXiv 2504.08378):
  * Section 2.1 ("Top-K sparsity"): for every linear operator only the input
    activations of largest magnitude take part in the product; the paper states
    the rule both as top-k and as "magnitude above a threshold" (Section 6,
    "Caching", keeps one threshold per sparsity level) -> select_topk,
    select_threshold, calibrate_threshold.
  * Section 4, pipeline operations T and C: T turns the activation into the
    indices of the active weight channels; C computes the operator on those
    channels only.  Because the result is exactly W (x * mask), the oracle
    writes that definition out with the dense out-major matrix -> sparse_gemv.
  * Section 3: the index set found at one layer is used for the same operator
    of the next layers of its group (N = 4) -> decode_stack(reuse...), overlap.
  * Section 6 ("Flash loading") and Section 7.1: weights are 4-bit with the
    matrix transposed so that a channel read carries its scales -> the q4
    functions (the quantiser itself is this build's own definition, see below);
    quantize_q4_cl is the arrangement with the groups inside a channel's row.
  * Fig. "simplified transformer layer" (Section 2.2): pre-norm block with
    residual connections -> decode_layer; the same block with a mixture-of-experts
    feed-forward half (the Mixtral-8x7B deployment of Sections 1 and 7)
    -> moe_route, decode_moe_layer.
  * Eq. 9: sparsity sp is the fraction of channels dropped -> keep_count.

Readings taken where the paper is silent: ties go to the lower channel index;
index lists are ascending; the magnitude order is the integer order of the
fp16 bit pattern with the sign cleared (so +0 == -0, Inf above finite, NaN
above Inf); a threshold is strict (> t) and compared in fp32; one selection on
a shared input serves q, k, v (and gate, up).  The 4-bit quantiser: groups of
32 consecutive input channels per output row, scale s = fp16(max|w| / 7)
(fp32 division), q = clamp(rint(w / s), -7, 7) (fp32 division, ties to even),
s == 0 -> q = 0, stored nibble = q + 8, value = (nibble - 8) * s.

All floating-point work is fp64 on the given fp16 bits; tensors that travel
between operators are rounded to fp16 (ties to even) where the device stores
fp16.  Pins for every function live in tests/test_oracle_*.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEL_TOPK = 0
SEL_THRESHOLD = 1
SEL_DENSE = 2

# selection points of a decoder layer, in execution order
P_QKV, P_O, P_GATEUP, P_DOWN = 0, 1, 2, 3
POINT_NAMES = ("qkv", "o", "gateup", "down")


# --------------------------------------------------------------------------
# selection (Section 2.1; Section 4 operation T)
# --------------------------------------------------------------------------
def keep_count(n: int, sparsity_percent: int) -> int:
    """k for a sparsity level: the paper's Eq. 9 counts (1 - sp) of the channels
    as active; integer form k = n - floor(sp * n / 100)."""
    return n - (int(sparsity_percent) * int(n)) // 100


def magnitude_key(x) -> np.ndarray:
    """Integer magnitude order of fp16 values: bit pattern with the sign cleared."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    return x.view(np.uint16) & np.uint16(0x7FFF)


def select_topk(x, k: int) -> np.ndarray:
    """The k channels of largest |x_j|, ties to the lower index, ascending int32."""
    key = magnitude_key(x).astype(np.int64)
    n = key.shape[0]
    if not 0 <= k <= n:
        raise ValueError("k out of range")
    j = np.arange(n)
    # primary key: magnitude descending; secondary: index ascending
    order = np.lexsort((j, -key))
    return np.sort(order[:k]).astype(np.int32)


def select_threshold(x, t: float) -> np.ndarray:
    """{j : |x_j| > t}, compared in fp32 (fp16 -> fp32 is exact), ascending int32."""
    mag = np.abs(np.asarray(x, dtype=np.float16).astype(np.float32))
    return np.nonzero(mag > np.float32(t))[0].astype(np.int32)


def calibrate_threshold(samples, sparsity_percent: int) -> float:
    """Threshold of one operator for one sparsity level (Section 6, "Caching": the
    index kernel keeps one activation threshold per sparsity level and compares
    against it; Section 2.1 calls the result Top-K sparsity, so the threshold
    stands for the top-k rule on typical inputs).

    The paper does not say how the thresholds are found.  Reading taken: pool the
    magnitudes of a calibration stream of the operator's input vectors (NaN left
    out), N values; with m = keep_count(N, sp) the threshold is the (m+1)-th
    largest pooled magnitude, so that the strict rule |x| > t keeps at most m of
    the pooled values -- exactly the pooled top-m when no value ties with the
    boundary.  m == N (nothing to drop) gives -1.0, which every magnitude exceeds.
    The value returned is an fp16 magnitude (or -1.0), exact in fp32."""
    mags = np.concatenate([np.abs(np.asarray(v, dtype=np.float16).astype(np.float64)).ravel()
                           for v in samples]) if len(samples) else np.zeros(0)
    mags = mags[~np.isnan(mags)]
    N = mags.size
    m = keep_count(N, sparsity_percent)
    if m >= N:
        return -1.0
    return float(np.sort(mags)[::-1][m])


# --------------------------------------------------------------------------
# sparse GEMV (Section 4 operation C) -- the dense definition W (x * mask)
# --------------------------------------------------------------------------
def _mask(n: int, idx) -> np.ndarray:
    m = np.zeros(n, dtype=np.float64)
    m[np.asarray(idx, dtype=np.int64)] = 1.0
    return m


def sparse_gemv(W, x, idx) -> np.ndarray:
    """y = W (x * mask(idx)); W is the out-major [out][in] matrix; fp64 result."""
    W = np.asarray(W)
    xm = np.asarray(x).astype(np.float64) * _mask(W.shape[1], idx)
    return W.astype(np.float64) @ xm


def round_f16(v) -> np.ndarray:
    """Round to fp16, ties to even (what a device store of an fp16 tensor does)."""
    return np.asarray(v, dtype=np.float64).astype(np.float16)


# --------------------------------------------------------------------------
# 4-bit group quantisation (Section 6 "Flash loading", Section 7.1)
# --------------------------------------------------------------------------
Q4_GROUP = 32


def quantize_q4_g32(W):
    """W[out][in] fp16 -> (nib uint8 [out][in] in 1..15, scales fp16 [in/32][out])."""
    W = np.asarray(W, dtype=np.float16)
    out, n_in = W.shape
    if n_in % Q4_GROUP:
        raise ValueError("in must be a multiple of 32")
    w32 = W.astype(np.float32).reshape(out, n_in // Q4_GROUP, Q4_GROUP)
    amax = np.max(np.abs(w32), axis=2)                                    # exact
    s16 = (amax / np.float32(7.0)).astype(np.float32).astype(np.float16)  # fp32 divide, then RNE
    s32 = s16.astype(np.float32)[:, :, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.rint((w32 / s32).astype(np.float32))
    q = np.where(s32 == 0, np.float32(0), np.clip(r, -7, 7)).astype(np.int32)
    nib = (q + 8).astype(np.uint8).reshape(out, n_in)
    return nib, np.ascontiguousarray(s16.T)


def pack_q4(nib) -> np.ndarray:
    """Logical packed form [in][out/2]: byte i of row j = column 2i (low nibble) and 2i+1 (high)."""
    nib = np.asarray(nib, dtype=np.uint8)
    t = np.ascontiguousarray(nib.T)                    # [in][out]
    return (t[:, 0::2] | (t[:, 1::2] << 4)).astype(np.uint8)


def unpack_q4(packed, out: int) -> np.ndarray:
    """Inverse of pack_q4: [in][out/2] bytes -> nib [out][in]."""
    packed = np.asarray(packed, dtype=np.uint8)
    t = np.empty((packed.shape[0], out), dtype=np.uint8)
    t[:, 0::2] = packed & 0xF
    t[:, 1::2] = packed >> 4
    return np.ascontiguousarray(t.T)


def dequant_q4_g32(nib, scales) -> np.ndarray:
    """(nib - 8) * scale of the group the input channel falls in, fp64 [out][in]."""
    nib = np.asarray(nib)
    s = np.asarray(scales).astype(np.float64)          # [in/32][out]
    q = nib.astype(np.float64) - 8.0
    return q * np.repeat(s.T, Q4_GROUP, axis=1)


def sparse_gemv_q4(nib, scales, x, idx) -> np.ndarray:
    return sparse_gemv(dequant_q4_g32(nib, scales), x, idx)


def quantize_q4_cl(W):
    """Channel-local variant: the groups lie inside one input channel's row of the
    transposed matrix (Section 6 "Flash loading": the transpose lets a channel read bring
    all the scales it needs), 32 consecutive output columns per group.  Same scale and
    rounding rules as quantize_q4_g32.  W[out][in] fp16 -> (nib uint8 [out][in],
    scales fp16 [in][out/32])."""
    W = np.asarray(W, dtype=np.float16)
    out, n_in = W.shape
    if out % Q4_GROUP:
        raise ValueError("out must be a multiple of 32")
    w32 = W.astype(np.float32).T.reshape(n_in, out // Q4_GROUP, Q4_GROUP)   # [in][group][32]
    amax = np.max(np.abs(w32), axis=2)
    s16 = (amax / np.float32(7.0)).astype(np.float32).astype(np.float16)
    s32 = s16.astype(np.float32)[:, :, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.rint((w32 / s32).astype(np.float32))
    q = np.where(s32 == 0, np.float32(0), np.clip(r, -7, 7)).astype(np.int32)
    nib = (q + 8).astype(np.uint8).reshape(n_in, out).T
    return np.ascontiguousarray(nib), np.ascontiguousarray(s16)


def dequant_q4_cl(nib, scales) -> np.ndarray:
    """(nib - 8) * scale of (input channel, group of 32 output columns), fp64 [out][in]."""
    nib = np.asarray(nib)
    s = np.asarray(scales).astype(np.float64)          # [in][out/32]
    q = nib.astype(np.float64) - 8.0
    return q * np.repeat(s, Q4_GROUP, axis=1).T


def sparse_gemv_q4_cl(nib, scales, x, idx) -> np.ndarray:
    return sparse_gemv(dequant_q4_cl(nib, scales), x, idx)


# --------------------------------------------------------------------------
# small-batch union (each token keeps its own mask)
# --------------------------------------------------------------------------
def union_indices(idx_b) -> np.ndarray:
    """Sorted union of the per-token index sets."""
    if len(idx_b) == 0:
        return np.zeros(0, dtype=np.int32)
    return np.unique(np.concatenate([np.asarray(i, dtype=np.int32) for i in idx_b])).astype(np.int32)


def union_gemv(W, X, idx_b) -> np.ndarray:
    """Y[b] = W (X[b] * mask(idx_b[b])): B independent single-token products."""
    return np.stack([sparse_gemv(W, X[b], idx_b[b]) for b in range(len(idx_b))])


# --------------------------------------------------------------------------
# cross-layer reuse metric (Section 3; Section 2.2 "Top-K precision")
# --------------------------------------------------------------------------
def overlap(reused, true_idx) -> float:
    """|reused & true| / |true| (1.0 when the true set is empty)."""
    t = np.asarray(true_idx)
    if t.size == 0:
        return 1.0
    return float(np.intersect1d(np.asarray(reused), t).size) / float(t.size)


# --------------------------------------------------------------------------
# glue operators of the pre-norm LLaMA-style block (Fig. in Section 2.2)
# --------------------------------------------------------------------------
def rmsnorm(h, g, eps: float) -> np.ndarray:
    h = np.asarray(h).astype(np.float64)
    return h / np.sqrt(np.mean(h * h) + eps) * np.asarray(g).astype(np.float64)


def rope(v, pos: int, theta: float) -> np.ndarray:
    """Rotate-half rotary embedding of v[..., head_dim] at position pos."""
    v = np.asarray(v, dtype=np.float64)
    hd = v.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=np.float64)
    ang = pos * theta ** (-2.0 * i / hd)
    c, s = np.cos(ang), np.sin(ang)
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(v) -> np.ndarray:
    v = np.asarray(v, dtype=np.float64)
    return v / (1.0 + np.exp(-v))


def attention_decode(q, K, V, n_keys: int) -> np.ndarray:
    """softmax(q K^T / sqrt(hd)) V over the first n_keys cache slots.

    q [n_heads][hd] fp64; K, V [n_kv][cap][hd]; query head h reads kv head
    h // (n_heads / n_kv).  Returns [n_heads][hd] fp64.
    """
    n_heads, hd = q.shape
    rep = n_heads // K.shape[0]
    out = np.empty((n_heads, hd), dtype=np.float64)
    for h in range(n_heads):
        Kh = K[h // rep, :n_keys].astype(np.float64)
        Vh = V[h // rep, :n_keys].astype(np.float64)
        s = Kh @ q[h] / np.sqrt(float(hd))
        p = np.exp(s - s.max())
        p /= p.sum()
        out[h] = p @ Vh
    return out


@dataclass
class LayerCfg:
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0


@dataclass
class SelectCfg:
    """mode: SEL_TOPK (k per point), SEL_THRESHOLD (t per point) or SEL_DENSE.
    reuse_mask bit p set -> do not select at point p, use the set handed in."""
    mode: int = SEL_TOPK
    k: tuple = (0, 0, 0, 0)
    t: tuple = (0.0, 0.0, 0.0, 0.0)
    reuse_mask: int = 0


@dataclass
class LayerTrace:
    """Everything a parity test needs from one layer, stage by stage."""
    x: list = field(default_factory=lambda: [None] * 4)     # fp16 input of each selection point
    idx: list = field(default_factory=lambda: [None] * 4)   # int32 index set used at each point
    qkv: np.ndarray = None          # fp16 [qkv_out] (before rope)
    attn: np.ndarray = None         # fp16 [n_heads*hd]
    h_mid: np.ndarray = None        # fp16 [d] after the attention block
    gateup: np.ndarray = None       # fp16 [2*ffn]
    hidden: np.ndarray = None       # fp16 [d] layer output
    k_new: np.ndarray = None        # fp16 [n_kv][hd] appended key (rotated)
    v_new: np.ndarray = None        # fp16 [n_kv][hd]


def _select(x16, p: int, sel: SelectCfg, given):
    n = x16.shape[0]
    if sel.reuse_mask >> p & 1:
        return np.asarray(given[p], dtype=np.int32)
    if sel.mode == SEL_TOPK:
        return select_topk(x16, sel.k[p])
    if sel.mode == SEL_THRESHOLD:
        return select_threshold(x16, sel.t[p])
    return np.arange(n, dtype=np.int32)


def _linear(W, x16, idx, weights_q4):
    """weights_q4: False (fp16 matrix), True (group-32-along-input pair) or "cl"
    (channel-local pair)."""
    if weights_q4 == "cl":
        nib, s = W
        return sparse_gemv_q4_cl(nib, s, x16, idx)
    if weights_q4:
        nib, s = W
        return sparse_gemv_q4(nib, s, x16, idx)
    return sparse_gemv(W, x16, idx)


def _attention_block(cfg, w, h0, K, V, kv_len, pos, sel, sets, weights_q4, tr):
    """The attention half of the block: norm, selection, q|k|v, rotary embedding, cache
    append, attention, selection, output projection, residual add.  Fills the trace's
    attention-side fields and returns h_mid (fp16)."""
    nh, nkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    x0 = round_f16(rmsnorm(h0, w["g_attn"], cfg.rms_eps))
    i0 = _select(x0, P_QKV, sel, sets)
    q = _linear(w["Wq"], x0, i0, weights_q4)
    k = _linear(w["Wk"], x0, i0, weights_q4)
    v = _linear(w["Wv"], x0, i0, weights_q4)
    qkv16 = round_f16(np.concatenate([q, k, v]))
    q16 = qkv16[: nh * hd].reshape(nh, hd)
    k16 = qkv16[nh * hd: (nh + nkv) * hd].reshape(nkv, hd)
    v16 = qkv16[(nh + nkv) * hd:].reshape(nkv, hd)
    qr = rope(q16, pos, cfg.rope_theta)
    k_new = round_f16(rope(k16, pos, cfg.rope_theta))
    K[:, kv_len, :] = k_new
    V[:, kv_len, :] = v16
    a16 = round_f16(attention_decode(qr, K, V, kv_len + 1).reshape(-1))
    i1 = _select(a16, P_O, sel, sets)
    h1 = round_f16(h0.astype(np.float64) + _linear(w["Wo"], a16, i1, weights_q4))
    tr.x[:2] = [x0, a16]
    tr.idx[:2] = [i0, i1]
    tr.qkv, tr.attn, tr.h_mid = qkv16, a16, h1
    tr.k_new, tr.v_new = k_new, v16.copy()
    return h1


def decode_layer(cfg: LayerCfg, w: dict, hidden, K, V, kv_len: int, pos: int,
                 sel: SelectCfg, sets=None, weights_q4: bool = False) -> LayerTrace:
    """One batch-1 decode step of a pre-norm block with activation sparsity at the
    inputs of qkv, o, gate/up and down.

    w holds out-major matrices Wq, Wk, Wv, Wo, Wgate, Wup, Wdown (fp16, or
    (nib, scales) pairs when weights_q4) and gains g_attn, g_ffn.  K, V
    [n_kv][cap][hd] fp16 are updated in place at slot kv_len.  `sets` gives the
    index sets for points whose reuse bit is set.  Returns the stage trace.
    """
    tr = LayerTrace()
    h0 = np.asarray(hidden, dtype=np.float16)
    h1 = _attention_block(cfg, w, h0, K, V, kv_len, pos, sel, sets, weights_q4, tr)

    # feed-forward block
    x2 = round_f16(rmsnorm(h1, w["g_ffn"], cfg.rms_eps))
    i2 = _select(x2, P_GATEUP, sel, sets)
    g = _linear(w["Wgate"], x2, i2, weights_q4)
    u = _linear(w["Wup"], x2, i2, weights_q4)
    gu16 = round_f16(np.concatenate([g, u]))
    f = cfg.d_ffn
    x3 = round_f16(silu(gu16[:f]) * gu16[f:].astype(np.float64))
    i3 = _select(x3, P_DOWN, sel, sets)
    h2 = round_f16(h1.astype(np.float64) + _linear(w["Wdown"], x3, i3, weights_q4))

    tr.x[2:] = [x2, x3]
    tr.idx[2:] = [i2, i3]
    tr.gateup, tr.hidden = gu16, h2
    return tr


# --------------------------------------------------------------------------
# mixture-of-experts block (the Mixtral-8x7B deployment of Sections 1 and 7)
# --------------------------------------------------------------------------
def moe_route(x16, Wr, top: int = 2):
    """Router of a sparse mixture-of-experts block: logits = Wr x over all channels of the
    normed input (the router is tiny and stays dense), the `top` experts of largest logit
    (ties to the lower expert index), slot 0 the largest; weights = softmax over the chosen
    logits.  Returns (experts int32 [top], weights fp64 [top], logits fp64 [E])."""
    logits = np.asarray(Wr, dtype=np.float16).astype(np.float64) @ np.asarray(x16, np.float16).astype(np.float64)
    order = np.lexsort((np.arange(len(logits)), -logits))[:top]
    z = logits[order]
    e = np.exp(z - z.max())
    return order.astype(np.int32), e / e.sum(), logits


@dataclass
class MoeTrace(LayerTrace):
    experts: np.ndarray = None      # int32 [top], slot order
    weights: np.ndarray = None      # fp64 [top]
    logits: np.ndarray = None       # fp64 [E]
    x_down: list = None             # fp16 [ffn] per slot: silu(gate) * up of that expert
    idx_down: list = None           # int32 index set per slot
    h_slots: list = None            # fp16 [d]: residual stream after each slot's expert


def decode_moe_layer(cfg: LayerCfg, w: dict, hidden, K, V, kv_len: int, pos: int,
                     sel: SelectCfg, top: int = 2, weights_q4=False) -> MoeTrace:
    """Decode step of a block whose feed-forward half is a sparse mixture of experts.

    The paper deploys Mixtral-8x7B with its method but gives no MoE-specific rule, so the
    dense block's rules are carried over (readings): operations T and C sit in front of
    every linear operator; the normed input is shared by the router and by all experts'
    gate/up projections, so one selection at point 2 serves every chosen expert; each
    chosen expert's down projection selects on its own silu(gate)*up (point 3, the same k
    or threshold for every expert).  Expert outputs are added to the fp16 residual stream
    one slot at a time, weighted by the router: h <- fp16(h + w_s * down_s(...)).

    w: the attention-side keys of decode_layer, g_ffn, Wr [E][d], and lists Wgate[e],
    Wup[e] [ffn][d], Wdown[e] [d][ffn] (with weights_q4, every matrix but the router is a
    (nib, scales) pair as in decode_layer)."""
    tr = MoeTrace()
    h0 = np.asarray(hidden, dtype=np.float16)
    h1 = _attention_block(cfg, w, h0, K, V, kv_len, pos, sel, None, weights_q4, tr)
    x2 = round_f16(rmsnorm(h1, w["g_ffn"], cfg.rms_eps))
    experts, weights, logits = moe_route(x2, w["Wr"], top)
    i2 = _select(x2, P_GATEUP, sel, None)
    f = cfg.d_ffn
    h = h1
    tr.x_down, tr.idx_down, tr.h_slots, gus = [], [], [], []
    for s, e in enumerate(experts):
        g = _linear(w["Wgate"][e], x2, i2, weights_q4)
        u = _linear(w["Wup"][e], x2, i2, weights_q4)
        gu16 = round_f16(np.concatenate([g, u]))
        x3 = round_f16(silu(gu16[:f]) * gu16[f:].astype(np.float64))
        i3 = _select(x3, P_DOWN, sel, None)
        h = round_f16(h.astype(np.float64) + weights[s] * _linear(w["Wdown"][e], x3, i3, weights_q4))
        gus.append(gu16); tr.x_down.append(x3); tr.idx_down.append(i3); tr.h_slots.append(h)
    tr.x[2:] = [x2, tr.x_down[0]]
    tr.idx[2:] = [i2, tr.idx_down[0]]
    tr.gateup = np.concatenate(gus)
    tr.experts, tr.weights, tr.logits = experts, weights, logits
    tr.hidden = h
    return tr


def decode_stack(cfg: LayerCfg, layers: list, hidden, Ks: list, Vs: list, kv_len: int, pos: int,
                 sel: SelectCfg, group: int = 1, reuse_points: int = 0, weights_q4: bool = False,
                 want_overlap: bool = False):
    """Run the layers in order.  With group > 1 (Section 3, N = 4 in the paper) layer
    l with l % group == 0 selects; the other layers of its group reuse its sets at
    the points whose bit is set in reuse_points.  Returns (traces, overlap) where
    overlap[l][p] compares the set used with the set the layer's own input would
    have selected (None for points that selected themselves or when not wanted).
    `sel` is one SelectCfg for all layers or a list with one per layer (calibrated
    thresholds differ from operator to operator)."""
    traces, ov = [], []
    sets = [None] * 4
    h = hidden
    per_layer = sel if isinstance(sel, (list, tuple)) else [sel] * len(layers)
    for l, w in enumerate(layers):
        sel = per_layer[l]
        follower = group > 1 and (l % group) != 0
        mask = sel.reuse_mask | (reuse_points if follower else 0)
        s = SelectCfg(sel.mode, sel.k, sel.t, mask)
        tr = decode_layer(cfg, w, h, Ks[l], Vs[l], kv_len, pos, s, sets, weights_q4)
        row = [None] * 4
        if want_overlap:
            own = SelectCfg(sel.mode, sel.k, sel.t, 0)
            for p in range(4):
                if mask >> p & 1:
                    row[p] = overlap(tr.idx[p], _select(tr.x[p], p, own, None))
        if not follower:
            sets = list(tr.idx)
        traces.append(tr)
        ov.append(row)
        h = tr.hidden
    return traces, ov


def rel_err(got, ref, floor_frac: float = 0.01) -> float:
    """Output error measure used by the parity tests:
    max_i |got_i - ref_i| / max(|ref_i|, floor_frac * rms(ref)).

    floor_frac = 0.01 judges a single operator fed with bit-identical inputs.  Stages deep
    inside a layer see inputs that already differ from the oracle's in the last fp16 bit of
    a few elements; that perturbation reaches every output as an absolute error
    proportional to rms(ref), so chained stages are judged with floor_frac = 1."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if ref.size == 0:
        return 0.0
    floor = floor_frac * np.sqrt(np.mean(ref * ref))
    den = np.maximum(np.abs(ref), floor)
    den = np.where(den == 0, 1.0, den)
    return float(np.max(np.abs(got - ref) / den))


# --------------------------------------------------------------------------
# dynamic weight caching (Section 4.2) and the cost model (Section 4.1)
# --------------------------------------------------------------------------
class LfuCache:
    """Least-frequently-used cache of weight channels of one tensor (Section 4.2,
    "Dynamic LLM Weight Caching"): one usage counter per channel, all zero at the
    start; the cache holds at most `capacity` channels.

    One token (step): the needed channels found in the cache are hits; every needed
    channel's counter goes up by one; then the missed channels, in ascending order,
    try to enter: into a free slot if there is one, otherwise in place of the
    least-used cached channel that this token does not need.

    Readings.  (1) The text lets a newcomer in when its count is "higher" than the
    least-used channel's, but its own worked example replaces channel 1 (count 1) by
    channel 7 (count 1): the example decides, the test is >=.  (2) Among equally
    little-used cached channels the lowest index leaves first.  (3) A channel the
    current token needs is never the victim.  (4) The hit ratio of a token is
    hits / needed channels, taken before anything enters."""

    def __init__(self, n_channels: int, capacity: int, initial=()):
        self.n, self.capacity = int(n_channels), int(capacity)
        self.count = [0] * self.n
        self.cached = set(int(c) for c in initial)
        if len(self.cached) > self.capacity or any(not 0 <= c < self.n for c in self.cached):
            raise ValueError("bad initial cache content")
        self.tokens = self.needed = self.hits = self.evictions = 0

    def step(self, idx):
        """Returns (hits, loaded, evicted list) for one token's needed channels."""
        need = sorted(set(int(j) for j in idx))
        hit = [j for j in need if j in self.cached]
        miss = [j for j in need if j not in self.cached]
        for j in need:
            self.count[j] += 1
        evicted = []
        for j in miss:
            if len(self.cached) < self.capacity:
                self.cached.add(j)
                continue
            victims = [c for c in self.cached if c not in need]
            if not victims:
                continue
            m = min(victims, key=lambda c: (self.count[c], c))
            if self.count[j] >= self.count[m]:
                self.cached.remove(m)
                self.cached.add(j)
                evicted.append(m)
        self.tokens += 1
        self.needed += len(need)
        self.hits += len(hit)
        self.evictions += len(evicted)
        return len(hit), len(miss), evicted


def cost_model(sp, hr, si, bw_mem, bw_flash_small, bw_flash_large, S_l, N, M_cache, M_kv):
    """Eq. 1-9 of Section 4.1 as printed (the prose around them names two terms wrongly;
    the equations are taken).  Sizes in bytes, bandwidths in bytes/s, times in seconds.
    Returns a dict with M_cl, M, T_load, T_comp, T_onload, T_preload, T_overlap, T_decode."""
    M_cl = S_l * (1.0 - sp) * N                                   # Eq. 9
    T_load = M_cl * (1.0 - hr) / bw_flash_small                   # Eq. 3
    T_comp = M_cl / bw_mem                                        # Eq. 4
    T_onload = S_l * (1.0 - sp) * (1.0 - hr) * (1.0 - si) / bw_flash_small   # Eq. 6
    T_preload = M_cl * (1.0 - hr) / bw_flash_large                # Eq. 7
    T_overlap = T_onload + max(T_preload, T_comp)                 # Eq. 5
    return {"M_cl": M_cl, "M": M_cl + M_cache + M_kv,             # Eq. 8
            "T_load": T_load, "T_comp": T_comp, "T_onload": T_onload, "T_preload": T_preload,
            "T_overlap": T_overlap, "T_decode": T_load + T_overlap + T_comp}   # Eq. 1


def plan_search(M_max, S_m, S_l, M_kv, si, bw_mem, bw_flash_small, bw_flash_large, hr_of_fraction,
                n_max=64, min_gain=0.0):
    """Greedy parameter search of Section 4.1 ("Preload-and-computation-balanced cross-layer
    group search").  sp = 1 - M_max / S_m (clamped to [0, 1)); then N = 1, 2, ...: the group
    takes M_cl (Eq. 9), the cache gets what the budget leaves, M_cache = M_max - M_cl - M_kv
    (Eq. 2 and 8 with equality), its hit rate is hr_of_fraction(M_cache / (S_m (1 - sp))), a
    caller-supplied curve (the paper measures it, Fig. "cache rate and load rate").  Stops
    when the budget is exhausted, when T_preload <= T_comp, or when T_preload changed by less
    than min_gain against the previous N.  Reading: the paper says the decode time is
    minimised "recursively" over these steps; the candidate of lowest T_decode among the ones
    visited is returned.  Returns (sp, N, M_cache, costs dict, visited list)."""
    sp = min(max(1.0 - M_max / S_m, 0.0), 1.0 - 1e-12)
    best, visited, prev = None, [], None
    for N in range(1, n_max + 1):
        M_cl = S_l * (1.0 - sp) * N
        M_cache = M_max - M_cl - M_kv
        if M_cache < 0:
            break
        hr = hr_of_fraction(M_cache / (S_m * (1.0 - sp)))
        c = cost_model(sp, hr, si, bw_mem, bw_flash_small, bw_flash_large, S_l, N, M_cache, M_kv)
        visited.append((N, M_cache, hr, c))
        if best is None or c["T_decode"] < best[3]["T_decode"]:
            best = (N, M_cache, hr, c)
        if c["T_preload"] <= c["T_comp"]:
            break
        if prev is not None and abs(prev - c["T_preload"]) < min_gain:
            break
        prev = c["T_preload"]
    if best is None:
        return sp, 0, 0.0, None, visited
    return sp, best[0], best[1], best[3], visited
