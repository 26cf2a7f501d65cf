"""Device-resident decoder stack: uploads host weights, packs them through the C ABI into the
fused in-major layout, owns the KV caches / index-set buffers, and marshals the layer and
stack calls.  Buffers and pointers only; every computation happens in libactiveflow.so."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as B


def layer_cfg(shape, weight_kind=B.AF_W_F16, rms_eps=1e-5, rope_theta=10000.0) -> B.LayerCfg:
    return B.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      rms_eps, rope_theta, weight_kind)


def select_cfg(mode, k=(0, 0, 0, 0), t=(0.0, 0.0, 0.0, 0.0), reuse_mask=0, flags=0) -> B.SelectCfg:
    s = B.SelectCfg()
    s.flags = flags
    s.mode = mode
    for p in range(4):
        s.k[p] = int(k[p])
        s.t[p] = float(t[p])
    s.reuse_mask = reuse_mask
    return s


class DeviceLayer:
    """Packed weights of one layer.  `host` maps Wq, Wk, Wv, Wo, Wgate, Wup, Wdown (fp16
    [out][in] NumPy arrays or torch tensors) and g_attn, g_ffn."""

    def __init__(self, ctx: B.Context, shape, host: dict, weight_kind=B.AF_W_F16):
        self.ctx, self.shape, self.kind = ctx, shape, weight_kind
        d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
        nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
        dev = ctx.device
        self.keep = []
        up = lambda a: (a.to(dev).contiguous() if torch.is_tensor(a)
                        else torch.from_numpy(np.ascontiguousarray(a)).to(dev))

        def fused(parts, n_in):
            ld = sum(p.shape[0] for p in parts)
            if weight_kind == B.AF_W_F16:
                Wt = torch.empty((n_in, ld), dtype=torch.float16, device=dev)
                S = None
            elif weight_kind == B.AF_W_Q4CL:
                Wt = torch.empty((n_in, ld // 2), dtype=torch.uint8, device=dev)
                S = torch.empty((n_in, ld // 32), dtype=torch.float16, device=dev)
            else:
                Wt = torch.empty((n_in, ld // 2), dtype=torch.uint8, device=dev)
                S = torch.empty((n_in // 32, ld), dtype=torch.float16, device=dev)
            col = 0
            for p in parts:
                Wd = up(p)
                torch.cuda.current_stream().synchronize()
                if weight_kind == B.AF_W_F16:
                    ctx.pack_inmajor_f16(Wd, Wt, col0=col)
                elif weight_kind == B.AF_W_Q4CL:
                    ctx.pack_q4_cl(Wd, Wt, S, col0=col)
                else:
                    ctx.pack_q4_g32(Wd, Wt, S, col0=col)
                ctx.synchronize()
                col += p.shape[0]
                del Wd
            return Wt, S

        self.Wqkv, self.Sqkv = fused([host["Wq"], host["Wk"], host["Wv"]], d)
        self.Wo, self.So = fused([host["Wo"]], nq)
        self.Wgateup, self.Sgateup = fused([host["Wgate"], host["Wup"]], d)
        self.Wdown, self.Sdown = fused([host["Wdown"]], f)
        self.g_attn = up(host["g_attn"])
        self.g_ffn = up(host["g_ffn"])
        torch.cuda.current_stream().synchronize()

    def struct(self) -> B.LayerWeights:
        p = lambda t: t.data_ptr() if t is not None else None
        return B.LayerWeights(p(self.Wqkv), p(self.Wo), p(self.Wgateup), p(self.Wdown),
                              p(self.Sqkv), p(self.So), p(self.Sgateup), p(self.Sdown),
                              p(self.g_attn), p(self.g_ffn))


class IdxSetBuffers:
    """Device buffers for the four index sets of one layer."""

    def __init__(self, ctx: B.Context, shape):
        widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
        self.widths = widths
        self.idx = [torch.zeros(w, dtype=torch.int32, device=ctx.device) for w in widths]
        self.count = [torch.zeros(1, dtype=torch.int32, device=ctx.device) for _ in widths]

    def struct(self) -> B.IdxSets:
        s = B.IdxSets()
        for p in range(4):
            s.idx[p] = self.idx[p].data_ptr()
            s.count[p] = self.count[p].data_ptr()
        return s

    def load(self, sets):
        """Copy host index lists in (for forced / reused sets)."""
        for p in range(4):
            if sets[p] is None:
                continue
            a = np.asarray(sets[p], dtype=np.int32)
            self.idx[p][: a.size] = torch.from_numpy(a).to(self.idx[p].device)
            self.count[p].fill_(int(a.size))
        torch.cuda.current_stream().synchronize()

    def fetch(self, p: int, n: int | None = None) -> np.ndarray:
        if n is None:
            n = int(self.count[p].item())
        return self.idx[p][:n].cpu().numpy()


class DeviceStack:
    """A stack of DeviceLayers with KV caches and per-layer index-set buffers."""

    def __init__(self, ctx: B.Context, shape, layers: list, kv: list, kv_cap: int,
                 weight_kind=B.AF_W_F16):
        self.ctx, self.shape, self.kind = ctx, shape, weight_kind
        self.layers = layers
        self.n_layers = len(layers)
        dev = ctx.device
        up = lambda a: a.to(dev) if torch.is_tensor(a) else torch.from_numpy(a).to(dev)
        self.K = [up(k) for k, _ in kv]
        self.V = [up(v) for _, v in kv]
        self.kv_cap = kv_cap
        self.sets = [IdxSetBuffers(ctx, shape) for _ in layers]
        self.cfg = layer_cfg(shape, weight_kind)
        self.w_array = (B.LayerWeights * self.n_layers)(*[l.struct() for l in layers])
        self.sets_array = (B.IdxSets * self.n_layers)(*[s.struct() for s in self.sets])
        self.k_ptrs = (C.c_void_p * self.n_layers)(*[k.data_ptr() for k in self.K])
        self.v_ptrs = (C.c_void_p * self.n_layers)(*[v.data_ptr() for v in self.V])
        self.hidden_out = torch.zeros(shape.d_model, dtype=torch.float16, device=dev)
        torch.cuda.current_stream().synchronize()

    def layer(self, l: int, hidden_in, hidden_out, kv_len: int, pos: int, sel: B.SelectCfg):
        self.ctx.decode_layer(self.cfg, self.layers[l].struct(), hidden_in, hidden_out, self.K[l],
                              self.V[l], kv_len, self.kv_cap, pos, sel, self.sets[l].struct())

    def run(self, hidden_in, kv_len: int, pos: int, sel, group: int = 1,
            reuse_points: int = 0, hidden_out=None):
        out = self.hidden_out if hidden_out is None else hidden_out
        self.ctx.decode_stack(self.cfg, self.w_array, self.n_layers, hidden_in, out, self.k_ptrs,
                              self.v_ptrs, kv_len, self.kv_cap, pos, sel, group, reuse_points,
                              self.sets_array)
        return out


class DeviceMoeLayer:
    """Packed weights and buffers of one mixture-of-experts block.  `host` holds the
    attention-side matrices, g_attn, g_ffn, the router Wr [E][d] and per-expert lists Wgate,
    Wup [ffn][d], Wdown [d][ffn] (fp16 NumPy arrays or torch tensors)."""

    def __init__(self, ctx: B.Context, shape, host: dict, top: int = 2, weight_kind=B.AF_W_F16):
        self.ctx, self.shape, self.top, self.kind = ctx, shape, top, weight_kind
        d, f, hd, E = shape.d_model, shape.d_ffn, shape.head_dim, shape.n_experts
        nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
        dev = ctx.device
        up = lambda a: (a.to(dev).contiguous() if torch.is_tensor(a)
                        else torch.from_numpy(np.ascontiguousarray(a)).to(dev))

        def alloc(lead, n_in, ld):
            """Weight (and scale) tensors of matrices [n_in][ld], with leading dims `lead`."""
            if weight_kind == B.AF_W_F16:
                return torch.empty(lead + (n_in, ld), dtype=torch.float16, device=dev), None
            Wt = torch.empty(lead + (n_in, ld // 2), dtype=torch.uint8, device=dev)
            if weight_kind == B.AF_W_Q4CL:
                return Wt, torch.empty(lead + (n_in, ld // 32), dtype=torch.float16, device=dev)
            return Wt, torch.empty(lead + (n_in // 32, ld), dtype=torch.float16, device=dev)

        def pack_into(parts, Wt, Sc):
            col = 0
            for p in parts:
                Wd = up(p)
                torch.cuda.current_stream().synchronize()
                if weight_kind == B.AF_W_F16:
                    ctx.pack_inmajor_f16(Wd, Wt, col0=col)
                elif weight_kind == B.AF_W_Q4CL:
                    ctx.pack_q4_cl(Wd, Wt, Sc, col0=col)
                else:
                    ctx.pack_q4_g32(Wd, Wt, Sc, col0=col)
                ctx.synchronize()
                col += p.shape[0]
                del Wd

        self.Wqkv, self.Sqkv = alloc((), d, nq + 2 * nkv)
        pack_into([host["Wq"], host["Wk"], host["Wv"]], self.Wqkv, self.Sqkv)
        self.Wo, self.So = alloc((), nq, d)
        pack_into([host["Wo"]], self.Wo, self.So)
        self.Wgateup, self.Sgateup = alloc((E,), d, 2 * f)
        self.Wdown, self.Sdown = alloc((E,), f, d)
        for e in range(E):
            pack_into([host["Wgate"][e], host["Wup"][e]], self.Wgateup[e],
                      None if self.Sgateup is None else self.Sgateup[e])
            pack_into([host["Wdown"][e]], self.Wdown[e], None if self.Sdown is None else self.Sdown[e])
        self.Wr = up(host["Wr"])
        self.g_attn, self.g_ffn = up(host["g_attn"]), up(host["g_ffn"])
        self.cfg = B.MoeCfg(layer_cfg(shape, weight_kind), E, top)
        widths = (d, nq, d) + (f,) * top
        self.widths = widths
        self.idx = [torch.zeros(n, dtype=torch.int32, device=dev) for n in widths]
        self.count = [torch.zeros(1, dtype=torch.int32, device=dev) for _ in widths]
        self.experts = torch.zeros(top, dtype=torch.int32, device=dev)
        self.weights = torch.zeros(top, dtype=torch.float32, device=dev)
        self.logits = torch.zeros(E, dtype=torch.float32, device=dev)
        torch.cuda.current_stream().synchronize()

    def weights_struct(self) -> B.MoeWeights:
        p = lambda t: t.data_ptr() if t is not None else None
        return B.MoeWeights(p(self.Wqkv), p(self.Wo), p(self.g_attn), p(self.g_ffn), p(self.Wr),
                            p(self.Wgateup), p(self.Wdown), p(self.Sqkv), p(self.So), p(self.Sgateup),
                            p(self.Sdown))

    def sets_struct(self) -> B.MoeSets:
        s = B.MoeSets()
        for p in range(len(self.widths)):
            s.idx[p] = self.idx[p].data_ptr()
            s.count[p] = self.count[p].data_ptr()
        return s

    def route_struct(self) -> B.MoeRoute:
        return B.MoeRoute(self.experts.data_ptr(), self.weights.data_ptr(), self.logits.data_ptr())

    def run(self, hidden_in, hidden_out, K, V, kv_len: int, kv_cap: int, pos: int, sel: B.SelectCfg):
        self.ctx.decode_moe_layer(self.cfg, self.weights_struct(), hidden_in, hidden_out, K, V, kv_len,
                                  kv_cap, pos, sel, self.sets_struct(), self.route_struct())
