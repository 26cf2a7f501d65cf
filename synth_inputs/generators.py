"""Random tensor generators (see the package docstring for the recipe)."""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    """Decoder-stack dimensions of one synthetic workload."""

    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    n_experts: int = 0      # > 0: the feed-forward half is a mixture of experts of width d_ffn

    @property
    def qkv_out(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ffn
        return d * self.qkv_out + self.n_heads * self.head_dim * d + 2 * d * f + f * d


MODEL_SHAPES = {
    # a few-tile toy used by fast tests (ragged: ffn is not a power of two)
    "tiny": ModelShape("tiny", 4, 256, 4, 4, 64, 688),
    "tiny_gqa": ModelShape("tiny_gqa", 2, 512, 8, 2, 64, 1376),
    # the head width of the real models (128) at toy size, grouped-query
    "tiny_hd128": ModelShape("tiny_hd128", 2, 512, 4, 2, 128, 1376),
    "7b": ModelShape("7b", 32, 4096, 32, 32, 128, 11008),
    "13b": ModelShape("13b", 40, 5120, 40, 40, 128, 13824),
    "70b": ModelShape("70b", 1, 8192, 64, 8, 128, 28672),
    # mixture-of-experts blocks: a toy and the Mixtral-8x7B block (8 experts, top-2)
    "tiny_moe": ModelShape("tiny_moe", 2, 512, 8, 2, 64, 1376, n_experts=4),
    "mixtral": ModelShape("mixtral", 32, 4096, 32, 8, 128, 14336, n_experts=8),
}


def _tag_words(tag) -> list[int]:
    words = []
    for t in tag:
        if isinstance(t, (int, np.integer)):
            words.append(int(t) & 0xFFFFFFFF)
        else:
            words.append(zlib.crc32(str(t).encode()) & 0xFFFFFFFF)
    return words


def rng_for(seed: int, *tag) -> np.random.Generator:
    """Child stream for one tensor: PCG64 seeded from (seed, tag words)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed)] + _tag_words(tag))))


def weight_matrix(seed: int, out: int, n_in: int, *tag, threads: int = 1) -> np.ndarray:
    """W[out][in] ~ N(0, 0.02) as fp16.  Row blocks use their own child streams so
    the result does not depend on `threads`."""
    block = 1024
    w = np.empty((out, n_in), dtype=np.float16)

    def fill(b0: int) -> None:
        b1 = min(out, b0 + block)
        g = rng_for(seed, "W", *tag, b0)
        v = g.standard_normal((b1 - b0, n_in), dtype=np.float32)
        v *= np.float32(0.02)
        w[b0:b1] = v.astype(np.float16)

    starts = list(range(0, out, block))
    if threads > 1 and len(starts) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, starts))
    else:
        for b0 in starts:
            fill(b0)
    return w


def channel_scales(seed: int, n: int, *tag) -> np.ndarray:
    """Per-channel scale vector s[n] (fp64): log-normal(sigma=0.5) with 0.1 % of the
    channels (at least one) boosted 20x."""
    g = rng_for(seed, "chan_scale", *tag, n)
    s = np.exp(0.5 * g.standard_normal(n))
    n_out = max(1, int(round(0.001 * n)))
    outliers = g.choice(n, size=n_out, replace=False)
    s[outliers] *= 20.0
    return s


def activation(seed: int, scales: np.ndarray, *tag) -> np.ndarray:
    """One token's activation vector x[n] in fp16: Laplace(0,1) times the channel scales."""
    g = rng_for(seed, "act", *tag)
    lap = g.laplace(0.0, 1.0, size=scales.shape[0])
    return (lap * scales).astype(np.float16)


def norm_gain(seed: int, n: int, *tag) -> np.ndarray:
    g = rng_for(seed, "gain", *tag)
    return (1.0 + 0.02 * g.standard_normal(n)).astype(np.float16)


def kv_cache(seed: int, n_kv_heads: int, cap: int, head_dim: int, filled: int, *tag):
    """K and V caches [n_kv][cap][head_dim] fp16; the first `filled` slots ~ N(0,1),
    the rest zero."""
    out = []
    for which in ("K", "V"):
        g = rng_for(seed, "kv", which, *tag)
        c = np.zeros((n_kv_heads, cap, head_dim), dtype=np.float16)
        c[:, :filled, :] = g.standard_normal((n_kv_heads, filled, head_dim), dtype=np.float32).astype(np.float16)
        out.append(c)
    return out[0], out[1]


def layer_weights(seed: int, shape: ModelShape, layer: int, threads: int = 1) -> dict:
    """Out-major fp16 matrices of one decoder layer plus the two norm gains.

    Keys: Wq, Wk, Wv [heads*hd][d]; Wo [d][heads*hd]; Wgate, Wup [ffn][d];
    Wdown [d][ffn]; g_attn, g_ffn [d].
    """
    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
    mk = lambda name, o, i: weight_matrix(seed, o, i, shape.name, layer, name, threads=threads)
    return {
        "Wq": mk("q", nq, d),
        "Wk": mk("k", nkv, d),
        "Wv": mk("v", nkv, d),
        "Wo": mk("o", d, nq),
        "Wgate": mk("gate", f, d),
        "Wup": mk("up", f, d),
        "Wdown": mk("down", d, f),
        "g_attn": norm_gain(seed, d, shape.name, layer, "attn"),
        "g_ffn": norm_gain(seed, d, shape.name, layer, "ffn"),
    }


def moe_layer_weights(seed: int, shape: ModelShape, layer: int, threads: int = 1) -> dict:
    """A layer whose feed-forward half is a mixture of shape.n_experts experts: the
    attention-side tensors of layer_weights(), g_ffn, the router Wr [E][d] ~ N(0, 0.02) and
    per-expert lists Wgate[e], Wup[e] [ffn][d], Wdown[e] [d][ffn]."""
    d, f, hd, E = shape.d_model, shape.d_ffn, shape.head_dim, shape.n_experts
    nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
    mk = lambda name, o, i: weight_matrix(seed, o, i, shape.name, layer, name, threads=threads)
    return {
        "Wq": mk("q", nq, d), "Wk": mk("k", nkv, d), "Wv": mk("v", nkv, d), "Wo": mk("o", d, nq),
        "Wr": mk("router", E, d),
        "Wgate": [mk(f"gate{e}", f, d) for e in range(E)],
        "Wup": [mk(f"up{e}", f, d) for e in range(E)],
        "Wdown": [mk(f"down{e}", d, f) for e in range(E)],
        "g_attn": norm_gain(seed, d, shape.name, layer, "attn"),
        "g_ffn": norm_gain(seed, d, shape.name, layer, "ffn"),
    }


def device_moe_layer_weights(seed: int, shape: ModelShape, layer: int, device="cuda") -> dict:
    """moe_layer_weights() drawn on the GPU (same distributions, torch's generator)."""
    import torch

    base = device_layer_weights(seed, shape, layer, device)
    d, f, E = shape.d_model, shape.d_ffn, shape.n_experts
    gen = torch.Generator(device=device)

    def mk(name, o, i):
        gen.manual_seed((int(seed) * 1000003 + zlib.crc32(f"{shape.name}/{layer}/{name}".encode())) & 0x7FFFFFFFFFFFFFFF)
        return (torch.randn((o, i), generator=gen, device=device, dtype=torch.float32) * 0.02).to(torch.float16)

    base["Wr"] = mk("router", E, d)
    base["Wgate"] = [base["Wgate"]] + [mk(f"gate{e}", f, d) for e in range(1, E)]
    base["Wup"] = [base["Wup"]] + [mk(f"up{e}", f, d) for e in range(1, E)]
    base["Wdown"] = [base["Wdown"]] + [mk(f"down{e}", d, f) for e in range(1, E)]
    return base


def device_layer_weights(seed: int, shape: ModelShape, layer: int, device="cuda") -> dict:
    """Same tensors as layer_weights(), drawn on the GPU with torch's seeded generator (a
    different random stream, same distribution) so that multi-GB stacks are ready in
    seconds.  Returns out-major fp16 torch tensors; callers that need the values on the
    host copy them back."""
    import torch

    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
    gen = torch.Generator(device=device)

    def mk(name, o, i):
        gen.manual_seed((int(seed) * 1000003 + zlib.crc32(f"{shape.name}/{layer}/{name}".encode())) & 0x7FFFFFFFFFFFFFFF)
        w = torch.randn((o, i), generator=gen, device=device, dtype=torch.float32)
        return (w * 0.02).to(torch.float16)

    def gain(name):
        gen.manual_seed((int(seed) * 1000003 + zlib.crc32(f"{shape.name}/{layer}/gain/{name}".encode())) & 0x7FFFFFFFFFFFFFFF)
        return (1.0 + 0.02 * torch.randn(d, generator=gen, device=device, dtype=torch.float32)).to(torch.float16)

    return {
        "Wq": mk("q", nq, d), "Wk": mk("k", nkv, d), "Wv": mk("v", nkv, d), "Wo": mk("o", d, nq),
        "Wgate": mk("gate", f, d), "Wup": mk("up", f, d), "Wdown": mk("down", d, f),
        "g_attn": gain("attn"), "g_ffn": gain("ffn"),
    }


def device_kv_cache(seed: int, shape: ModelShape, layer: int, cap: int, filled: int, device="cuda"):
    """K and V caches [n_kv][cap][hd] fp16 on the GPU, first `filled` slots ~ N(0,1)."""
    import torch

    gen = torch.Generator(device=device)
    out = []
    for which in ("K", "V"):
        gen.manual_seed((int(seed) * 1000003 + zlib.crc32(f"{shape.name}/{layer}/kv/{which}".encode())) & 0x7FFFFFFFFFFFFFFF)
        c = torch.zeros((shape.n_kv_heads, cap, shape.head_dim), dtype=torch.float16, device=device)
        c[:, :filled] = torch.randn((shape.n_kv_heads, filled, shape.head_dim), generator=gen,
                                    device=device, dtype=torch.float32).to(torch.float16)
        out.append(c)
    return out[0], out[1]
