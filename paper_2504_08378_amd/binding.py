"""ctypes binding of include/activeflow.h: argument marshalling only.

Every function here takes torch CUDA tensors (used purely as device buffers), checks
dtype/contiguity, passes raw device pointers to the C ABI and raises AfError on a non-zero
status.  No arithmetic of the method happens in Python.  There is no CPU fallback: if the
shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libactiveflow.so")

AF_F16, AF_F32 = 0, 1
AF_W_F16, AF_W_Q4G32, AF_W_Q4CL = 0, 1, 2
AF_SEL_TOPK, AF_SEL_THRESHOLD, AF_SEL_DENSE = 0, 1, 2
AF_SEL_SKIP_SETS = 1
AF_PRO_NONE, AF_PRO_RMSNORM, AF_PRO_SILUMUL = 0, 1, 2
AF_MAX_N, AF_MAX_BATCH = 32768, 8
AF_CALIB_BINS = 32768
AF_NOALLOC_MAX_OUT, AF_ENOALLOC_LIMIT = 65536, -6
AF_OPT_LAYER_KERNEL, AF_OPT_VALIDATE, AF_OPT_TUNE_LX, AF_OPT_TUNE_WAVES = 1, 2, 3, 4
AF_OPT_TUNE_SPLIT, AF_OPT_TUNE_WORKGROUPS, AF_OPT_MOE_ROUTER_KERNEL = 5, 6, 7
AF_OPT_TUNE_ATTN_SPLITS = 8
AF_DEVERR_SPIN, AF_DEVERR_IDX = 1, 2

EXPORTS = [
    "af_create", "af_destroy", "af_set_stream", "af_strerror", "af_workspace_bytes",
    "af_set_workspace", "af_select_topk", "af_select_threshold", "af_pack_inmajor_f16",
    "af_pack_q4_g32", "af_sparse_gemv_f16", "af_sparse_gemv_q4", "af_sparse_gemv_q4_cl", "af_pack_q4_cl", "af_select_gemv_f16", "af_sparse_gemv_union_f16",
    "af_decode_layer", "af_decode_stack", "af_layer_tap", "af_capture_begin", "af_capture_end",
    "af_graph_launch", "af_graph_destroy", "af_probe_sink_floats", "af_probe_stream_read",
    "af_calib_accumulate", "af_calib_accumulate_layer", "af_calib_thresholds",
    "af_decode_moe_layer", "af_select_gemv_experts_f16",
    "af_lfu_create", "af_lfu_destroy", "af_lfu_step", "af_lfu_stats", "af_lfu_cached",
    "af_cost_eval", "af_plan_search", "af_sparse_gemv_f16_noalloc",
    "af_profile_set", "af_wall_clock_khz", "af_set_option", "af_last_device_error",
    "af_unpack_q4_g32", "af_probe_stream_read_variant", "af_decode_layer_batch",
]
AF_MOE_MAX_EXPERTS, AF_MOE_MAX_TOP = 16, 4


class AfError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({strerror(status)})")


class LayerCfg(C.Structure):
    _fields_ = [("d_model", C.c_int), ("n_heads", C.c_int), ("n_kv_heads", C.c_int),
                ("head_dim", C.c_int), ("d_ffn", C.c_int), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("weight_kind", C.c_int)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("Wqkv", "Wo", "Wgateup", "Wdown", "Sqkv", "So", "Sgateup", "Sdown",
                 "g_attn_norm", "g_ffn_norm")]


class IdxSets(C.Structure):
    _fields_ = [("idx", C.c_void_p * 4), ("count", C.c_void_p * 4)]


class SelectCfg(C.Structure):
    _fields_ = [("mode", C.c_int), ("k", C.c_int * 4), ("t", C.c_float * 4),
                ("reuse_mask", C.c_uint), ("flags", C.c_uint)]


class MoeCfg(C.Structure):
    _fields_ = [("base", LayerCfg), ("n_experts", C.c_int), ("top", C.c_int)]


class MoeWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("Wqkv", "Wo", "g_attn_norm", "g_ffn_norm", "Wr", "Wgateup", "Wdown",
                 "Sqkv", "So", "Sgateup", "Sdown")]


class MoeSets(C.Structure):
    _fields_ = [("idx", C.c_void_p * (3 + AF_MOE_MAX_TOP)), ("count", C.c_void_p * (3 + AF_MOE_MAX_TOP))]


class MoeRoute(C.Structure):
    _fields_ = [("experts", C.c_void_p), ("weights", C.c_void_p), ("logits", C.c_void_p)]


class CostIn(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("sp", "hr", "si", "bw_mem", "bw_flash_small", "bw_flash_large",
                                          "S_l", "N", "M_cache", "M_kv")]


class CostOut(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("M_cl", "M", "T_load", "T_comp", "T_onload", "T_preload",
                                          "T_overlap", "T_decode")]


class PlanIn(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("M_max", "S_m", "S_l", "M_kv", "si", "bw_mem", "bw_flash_small",
                                          "bw_flash_large")] + \
               [("hr_fraction", C.POINTER(C.c_double)), ("hr_value", C.POINTER(C.c_double)),
                ("n_hr", C.c_int), ("n_max", C.c_int), ("min_gain", C.c_double)]


class PlanOut(C.Structure):
    _fields_ = [("sp", C.c_double), ("N", C.c_int), ("visited", C.c_int), ("M_cache", C.c_double),
                ("hr", C.c_double), ("cost", CostOut)]


_lib = None


def lib() -> C.CDLL:
    """Load libactiveflow.so (built in-tree by paper_2504_08378_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_08378_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i, f, u, sz = C.c_void_p, C.c_int, C.c_float, C.c_uint, C.c_size_t
    sig = {
        "af_create": (i, [C.POINTER(vp), i, vp]),
        "af_destroy": (i, [vp]),
        "af_set_stream": (i, [vp, vp]),
        "af_strerror": (C.c_char_p, [i]),
        "af_workspace_bytes": (sz, [i, i, i]),
        "af_set_workspace": (i, [vp, vp, sz, i, i, i]),
        "af_select_topk": (i, [vp, vp, i, i, vp]),
        "af_select_threshold": (i, [vp, vp, i, f, vp, vp]),
        "af_pack_inmajor_f16": (i, [vp, vp, i, i, vp, i, i]),
        "af_pack_q4_g32": (i, [vp, vp, i, i, vp, vp, i, i]),
        "af_sparse_gemv_f16": (i, [vp, vp, i, i, i, vp, vp, i, vp, vp, i, vp]),
        "af_sparse_gemv_f16_noalloc": (i, [vp, vp, i, i, i, vp, vp, i, vp, vp, i, vp]),
        "af_sparse_gemv_q4": (i, [vp, vp, vp, i, i, i, vp, vp, i, vp, vp, i, vp]),
        "af_sparse_gemv_q4_cl": (i, [vp, vp, vp, i, i, i, vp, vp, i, vp, vp, i, vp]),
        "af_pack_q4_cl": (i, [vp, vp, i, i, vp, vp, i, i]),
        "af_select_gemv_f16": (i, [vp, vp, i, i, i, i, vp, vp, f, i, i, f, vp, vp, vp, vp, i, vp]),
        "af_sparse_gemv_union_f16": (i, [vp, vp, i, i, i, vp, i, vp, i, vp, vp, vp, i]),
        "af_decode_layer": (i, [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeights), vp, vp, vp, vp,
                                i, i, i, C.POINTER(SelectCfg), C.POINTER(IdxSets)]),
        "af_decode_stack": (i, [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeights), i, vp, vp,
                                C.POINTER(vp), C.POINTER(vp), i, i, i, C.POINTER(SelectCfg), i, i, u,
                                C.POINTER(IdxSets)]),
        "af_decode_layer_batch": (i, [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeights), i, vp, vp,
                                      C.POINTER(vp), C.POINTER(vp), C.POINTER(i), i, C.POINTER(i),
                                      C.POINTER(SelectCfg), C.POINTER(IdxSets), vp]),
        "af_layer_tap": (i, [vp, i, C.POINTER(vp)]),
        "af_capture_begin": (i, [vp]),
        "af_capture_end": (i, [vp, C.POINTER(vp)]),
        "af_graph_launch": (i, [vp, vp]),
        "af_graph_destroy": (i, [vp]),
        "af_probe_sink_floats": (i, [vp]),
        "af_probe_stream_read": (i, [vp, vp, sz, vp, i]),
        "af_probe_stream_read_variant": (i, [vp, vp, sz, vp, i, i, i, i]),
        "af_calib_accumulate": (i, [vp, vp, i, vp]),
        "af_calib_accumulate_layer": (i, [vp, C.POINTER(LayerCfg), C.POINTER(vp)]),
        "af_calib_thresholds": (i, [vp, vp, C.POINTER(C.c_int), i, vp]),
        "af_select_gemv_experts_f16": (i, [vp, vp, vp, i, C.c_longlong, vp, i, i, i, i, vp, vp, f, i, i, f,
                                           vp, vp, vp, vp, i, vp]),
        "af_lfu_create": (i, [C.POINTER(vp), i, i, C.POINTER(C.c_int32), i]),
        "af_lfu_destroy": (i, [vp]),
        "af_lfu_step": (i, [vp, C.POINTER(C.c_int32), i, C.POINTER(i), C.POINTER(i), C.POINTER(C.c_int32),
                            C.POINTER(i)]),
        "af_lfu_stats": (i, [vp] + [C.POINTER(C.c_longlong)] * 4),
        "af_lfu_cached": (i, [vp, C.POINTER(C.c_int32), C.POINTER(i)]),
        "af_profile_set": (i, [vp, vp, i]),
        "af_wall_clock_khz": (i, [vp]),
        "af_set_option": (i, [vp, i, i]),
        "af_unpack_q4_g32": (i, [vp, vp, vp, i, i, i, i, vp, vp]),
        "af_last_device_error": (i, [vp, C.POINTER(i), i]),
        "af_cost_eval": (i, [C.POINTER(CostIn), C.POINTER(CostOut)]),
        "af_plan_search": (i, [C.POINTER(PlanIn), C.POINTER(PlanOut)]),
        "af_decode_moe_layer": (i, [vp, C.POINTER(MoeCfg), C.POINTER(MoeWeights), vp, vp, vp, vp,
                                    i, i, i, C.POINTER(SelectCfg), C.POINTER(MoeSets),
                                    C.POINTER(MoeRoute)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().af_strerror(status).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise AfError(status, what)


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


class Context:
    """One af_ctx bound to a device and a torch stream, with its workspace tensor."""

    def __init__(self, device: int = 0, stream: torch.cuda.Stream | None = None,
                 max_in: int = AF_MAX_N, max_out: int = 65536, max_batch: int = AF_MAX_BATCH,
                 with_workspace: bool = True):
        L = lib()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the active-weight path has no CPU fallback")
        self.device = torch.device("cuda", device)
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        h = C.c_void_p()
        _check(L.af_create(C.byref(h), device, C.c_void_p(self.stream.cuda_stream)), "af_create")
        self._h = h
        self.workspace = None
        self.max_in, self.max_out, self.max_batch = max_in, max_out, max_batch
        if not with_workspace:   # only the entry points that bring their own scratch work then
            return
        nbytes = L.af_workspace_bytes(max_in, max_out, max_batch)
        if nbytes == 0:
            raise ValueError("invalid workspace limits")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        _check(L.af_set_workspace(h, _ptr(self.workspace), nbytes, max_in, max_out, max_batch),
               "af_set_workspace")
        self.max_in, self.max_out, self.max_batch = max_in, max_out, max_batch

    def close(self):
        if getattr(self, "_h", None) is not None:
            self.synchronize()
            lib().af_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def synchronize(self):
        self.stream.synchronize()

    # ---- selection -------------------------------------------------------------------
    def select_topk(self, x, k: int, idx=None):
        n = x.numel()
        if idx is None:
            idx = torch.empty(max(k, 1), dtype=torch.int32, device=self.device)
        _check(lib().af_select_topk(self._h, _ptr(x, torch.float16, "x"), n, k,
                                    _ptr(idx, torch.int32, "idx")), "af_select_topk")
        return idx[:k]

    def select_threshold(self, x, t: float, idx=None, count=None):
        n = x.numel()
        if idx is None:
            idx = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        if count is None:
            count = torch.empty(1, dtype=torch.int32, device=self.device)
        _check(lib().af_select_threshold(self._h, _ptr(x, torch.float16, "x"), n, float(t),
                                         _ptr(idx, torch.int32, "idx"),
                                         _ptr(count, torch.int32, "count")), "af_select_threshold")
        return idx, count

    # ---- packing ---------------------------------------------------------------------
    def pack_inmajor_f16(self, W, Wt=None, ld=None, col0=0):
        out, n_in = W.shape
        if Wt is None:
            ld = out if ld is None else ld
            Wt = torch.empty((n_in, ld), dtype=torch.float16, device=self.device)
        ld = Wt.shape[1]
        _check(lib().af_pack_inmajor_f16(self._h, _ptr(W, torch.float16, "W"), out, n_in,
                                         _ptr(Wt, torch.float16, "Wt"), ld, col0),
               "af_pack_inmajor_f16")
        return Wt

    def pack_q4_g32(self, W, packed=None, scales=None, ld=None, col0=0):
        out, n_in = W.shape
        if packed is None:
            ld = out if ld is None else ld
            packed = torch.empty((n_in, ld // 2), dtype=torch.uint8, device=self.device)
            scales = torch.empty((n_in // 32, ld), dtype=torch.float16, device=self.device)
        ld = scales.shape[1]
        _check(lib().af_pack_q4_g32(self._h, _ptr(W, torch.float16, "W"), out, n_in,
                                    _ptr(packed, torch.uint8, "packed"),
                                    _ptr(scales, torch.float16, "scales"), ld, col0),
               "af_pack_q4_g32")
        return packed, scales

    def unpack_q4_g32(self, packed, scales, out: int, col0: int = 0):
        """(q int8 [out][in], w fp32 [out][in]) of the columns col0..col0+out of a packed matrix."""
        n_in, ld = packed.shape[0], scales.shape[1]
        q = torch.empty((out, n_in), dtype=torch.int8, device=self.device)
        w = torch.empty((out, n_in), dtype=torch.float32, device=self.device)
        _check(lib().af_unpack_q4_g32(self._h, _ptr(packed, torch.uint8, "packed"),
                                      _ptr(scales, torch.float16, "scales"), out, n_in, ld, col0,
                                      _ptr(q, torch.int8, "q"), _ptr(w, torch.float32, "w")),
               "af_unpack_q4_g32")
        return q, w

    def pack_q4_cl(self, W, packed=None, scales=None, ld=None, col0=0):
        """Channel-local groups: scales [in][ld/32]."""
        out, n_in = W.shape
        if packed is None:
            ld = out if ld is None else ld
            packed = torch.empty((n_in, ld // 2), dtype=torch.uint8, device=self.device)
            scales = torch.empty((n_in, ld // 32), dtype=torch.float16, device=self.device)
        ld = scales.shape[1] * 32
        _check(lib().af_pack_q4_cl(self._h, _ptr(W, torch.float16, "W"), out, n_in,
                                   _ptr(packed, torch.uint8, "packed"),
                                   _ptr(scales, torch.float16, "scales"), ld, col0),
               "af_pack_q4_cl")
        return packed, scales

    # ---- GEMV ------------------------------------------------------------------------
    def sparse_gemv_f16(self, Wt, x, idx=None, nidx=None, nidx_dev=None, y=None, y_kind=AF_F16,
                        residual=None, out=None):
        n_in, ld = Wt.shape
        out = ld if out is None else out
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        if idx is not None and nidx is None:
            nidx = idx.numel()
        _check(lib().af_sparse_gemv_f16(
            self._h, _ptr(Wt, torch.float16, "Wt"), n_in, out, ld, _ptr(x, torch.float16, "x"),
            _ptr(idx, torch.int32, "idx"), int(nidx or 0), _ptr(nidx_dev, torch.int32, "nidx_dev"),
            _ptr(y, None, "y"), y_kind, _ptr(residual, torch.float16, "residual")),
            "af_sparse_gemv_f16")
        return y

    def sparse_gemv_f16_noalloc(self, Wt, x, idx=None, nidx=None, nidx_dev=None, y=None,
                                y_kind=AF_F16, residual=None, out=None):
        """af_sparse_gemv_f16_noalloc: y must be given by callers that may not allocate; when it
        is omitted here the output tensor is made before the call, the call itself allocates
        nothing."""
        n_in, ld = Wt.shape
        out = ld if out is None else out
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        if idx is not None and nidx is None:
            nidx = idx.numel()
        _check(lib().af_sparse_gemv_f16_noalloc(
            self._h, _ptr(Wt, torch.float16, "Wt"), n_in, out, ld, _ptr(x, torch.float16, "x"),
            _ptr(idx, torch.int32, "idx"), int(nidx or 0), _ptr(nidx_dev, torch.int32, "nidx_dev"),
            _ptr(y, None, "y"), y_kind, _ptr(residual, torch.float16, "residual")),
            "af_sparse_gemv_f16_noalloc")
        return y

    def sparse_gemv_q4(self, packed, scales, x, idx=None, nidx=None, nidx_dev=None, y=None,
                       y_kind=AF_F16, residual=None, out=None):
        n_in = packed.shape[0]
        ld = scales.shape[1]
        out = ld if out is None else out
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        if idx is not None and nidx is None:
            nidx = idx.numel()
        _check(lib().af_sparse_gemv_q4(
            self._h, _ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float16, "scales"),
            n_in, out, ld, _ptr(x, torch.float16, "x"), _ptr(idx, torch.int32, "idx"),
            int(nidx or 0), _ptr(nidx_dev, torch.int32, "nidx_dev"), _ptr(y, None, "y"), y_kind,
            _ptr(residual, torch.float16, "residual")), "af_sparse_gemv_q4")
        return y

    def sparse_gemv_q4_cl(self, packed, scales, x, idx=None, nidx=None, nidx_dev=None, y=None,
                          y_kind=AF_F16, residual=None, out=None):
        n_in = packed.shape[0]
        ld = scales.shape[1] * 32
        out = ld if out is None else out
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        if idx is not None and nidx is None:
            nidx = idx.numel()
        _check(lib().af_sparse_gemv_q4_cl(
            self._h, _ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float16, "scales"),
            n_in, out, ld, _ptr(x, torch.float16, "x"), _ptr(idx, torch.int32, "idx"),
            int(nidx or 0), _ptr(nidx_dev, torch.int32, "nidx_dev"), _ptr(y, None, "y"), y_kind,
            _ptr(residual, torch.float16, "residual")), "af_sparse_gemv_q4_cl")
        return y

    def select_gemv_f16(self, Wt, src, producer=AF_PRO_NONE, gain=None, eps=1e-5,
                        sel_mode=AF_SEL_TOPK, k=0, t=0.0, x_out=None, idx_out=None, count_out=None,
                        y=None, y_kind=AF_F16, residual=None, out=None):
        n_in, ld = Wt.shape
        out = ld if out is None else out
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        _check(lib().af_select_gemv_f16(
            self._h, _ptr(Wt, torch.float16, "Wt"), n_in, out, ld, producer,
            _ptr(src, torch.float16, "src"), _ptr(gain, torch.float16, "gain"), float(eps),
            sel_mode, int(k), float(t), _ptr(x_out, torch.float16, "x_out"),
            _ptr(idx_out, torch.int32, "idx_out"), _ptr(count_out, torch.int32, "count_out"),
            _ptr(y, None, "y"), y_kind, _ptr(residual, torch.float16, "residual")),
            "af_select_gemv_f16")
        return y

    def sparse_gemv_union_f16(self, Wt, X, idx_b, y_kind=AF_F16, out=None):
        n_in, ld = Wt.shape
        out = ld if out is None else out
        B, k = idx_b.shape
        Y = torch.empty((B, out), dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                        device=self.device)
        union_idx = torch.empty(n_in, dtype=torch.int32, device=self.device)
        union_n = torch.empty(1, dtype=torch.int32, device=self.device)
        _check(lib().af_sparse_gemv_union_f16(
            self._h, _ptr(Wt, torch.float16, "Wt"), n_in, out, ld, _ptr(X, torch.float16, "X"), B,
            _ptr(idx_b, torch.int32, "idx_b"), k, _ptr(union_idx, torch.int32, "union_idx"),
            _ptr(union_n, torch.int32, "union_n"), _ptr(Y, None, "Y"), y_kind),
            "af_sparse_gemv_union_f16")
        return Y, union_idx, union_n

    # ---- layer / stack ---------------------------------------------------------------
    def decode_layer(self, cfg: LayerCfg, w: LayerWeights, hidden_in, hidden_out, k_cache, v_cache,
                     kv_len: int, kv_cap: int, pos: int, sel: SelectCfg, sets: IdxSets | None):
        _check(lib().af_decode_layer(
            self._h, C.byref(cfg), C.byref(w), _ptr(hidden_in, torch.float16, "hidden_in"),
            _ptr(hidden_out, torch.float16, "hidden_out"), _ptr(k_cache, torch.float16, "k_cache"),
            _ptr(v_cache, torch.float16, "v_cache"), kv_len, kv_cap, pos, C.byref(sel),
            C.byref(sets) if sets is not None else None), "af_decode_layer")

    def decode_layer_batch(self, cfg: LayerCfg, w: LayerWeights, hidden_in, hidden_out, k_caches,
                           v_caches, kv_len, kv_cap: int, pos, sel: SelectCfg, sets: IdxSets,
                           union_n=None):
        """B tokens at once: hidden_in / hidden_out fp16 [B][d]; k_caches, v_caches: sequences of B
        cache tensors; kv_len, pos: sequences of B ints; sets: idx[p] int32 [B][n_p], count[p] [B]."""
        Bt = int(hidden_in.shape[0])
        kp = (C.c_void_p * Bt)(*[_ptr(t, torch.float16, "k_cache").value for t in k_caches])
        vp_ = (C.c_void_p * Bt)(*[_ptr(t, torch.float16, "v_cache").value for t in v_caches])
        kl = (C.c_int * Bt)(*[int(v) for v in kv_len])
        ps = (C.c_int * Bt)(*[int(v) for v in pos])
        _check(lib().af_decode_layer_batch(
            self._h, C.byref(cfg), C.byref(w), Bt, _ptr(hidden_in, torch.float16, "hidden_in"),
            _ptr(hidden_out, torch.float16, "hidden_out"), kp, vp_, kl, kv_cap, ps, C.byref(sel),
            C.byref(sets), _ptr(union_n, torch.int32, "union_n")), "af_decode_layer_batch")

    def decode_stack(self, cfg: LayerCfg, w_array, n_layers: int, hidden_in, hidden_out,
                     k_ptrs, v_ptrs, kv_len: int, kv_cap: int, pos: int, sel,
                     group: int, reuse_points: int, sets_array):
        """sel: one SelectCfg for all layers, or a sequence with one per layer."""
        if isinstance(sel, SelectCfg):
            sel_arr, n_sel = (SelectCfg * 1)(sel), 1
        else:
            sel_arr, n_sel = (SelectCfg * len(sel))(*sel), len(sel)
        _check(lib().af_decode_stack(
            self._h, C.byref(cfg), w_array, n_layers, _ptr(hidden_in, torch.float16, "hidden_in"),
            _ptr(hidden_out, torch.float16, "hidden_out"), k_ptrs, v_ptrs, kv_len, kv_cap, pos,
            sel_arr, n_sel, group, reuse_points, sets_array), "af_decode_stack")

    def select_gemv_experts_f16(self, Wt_all, expert_sel, n_slots, src, producer=AF_PRO_NONE, gain=None,
                                eps=1e-5, sel_mode=AF_SEL_TOPK, k=0, t=0.0, x_out=None, idx_out=None,
                                count_out=None, y=None, y_kind=AF_F16, residual=None, y_scale=None):
        """Wt_all [E][in][cols]: slot s of y uses expert expert_sel[s] (device int32)."""
        E, n_in, cols = Wt_all.shape
        out = cols * n_slots
        if y is None:
            y = torch.empty(out, dtype=torch.float16 if y_kind == AF_F16 else torch.float32,
                            device=self.device)
        _check(lib().af_select_gemv_experts_f16(
            self._h, _ptr(Wt_all, torch.float16, "Wt_all"), _ptr(expert_sel, torch.int32, "expert_sel"),
            n_slots, n_in * cols, _ptr(y_scale, torch.float32, "y_scale"), n_in, out, cols, producer,
            _ptr(src, torch.float16, "src"), _ptr(gain, torch.float16, "gain"), float(eps), sel_mode,
            int(k), float(t), _ptr(x_out, torch.float16, "x_out"), _ptr(idx_out, torch.int32, "idx_out"),
            _ptr(count_out, torch.int32, "count_out"), _ptr(y, None, "y"), y_kind,
            _ptr(residual, torch.float16, "residual")), "af_select_gemv_experts_f16")
        return y

    def decode_moe_layer(self, cfg: MoeCfg, w: MoeWeights, hidden_in, hidden_out, k_cache, v_cache,
                         kv_len: int, kv_cap: int, pos: int, sel: SelectCfg, sets, route: MoeRoute):
        _check(lib().af_decode_moe_layer(
            self._h, C.byref(cfg), C.byref(w), _ptr(hidden_in, torch.float16, "hidden_in"),
            _ptr(hidden_out, torch.float16, "hidden_out"), _ptr(k_cache, torch.float16, "k_cache"),
            _ptr(v_cache, torch.float16, "v_cache"), kv_len, kv_cap, pos, C.byref(sel),
            C.byref(sets) if sets is not None else None, C.byref(route)), "af_decode_moe_layer")

    def layer_tap(self, which: int, n: int):
        """fp16 view (a copy) of an inter-operator tensor of the last decode_layer call."""
        p = C.c_void_p()
        _check(lib().af_layer_tap(self._h, which, C.byref(p)), "af_layer_tap")
        base = self.workspace.data_ptr()
        off = p.value - base
        return self.workspace[off: off + 2 * n].view(torch.float16).clone()

    # ---- graphs ----------------------------------------------------------------------
    def capture_begin(self):
        _check(lib().af_capture_begin(self._h), "af_capture_begin")

    def capture_end(self):
        g = C.c_void_p()
        _check(lib().af_capture_end(self._h, C.byref(g)), "af_capture_end")
        return g

    def graph_launch(self, g):
        _check(lib().af_graph_launch(self._h, g), "af_graph_launch")

    def graph_destroy(self, g):
        _check(lib().af_graph_destroy(g), "af_graph_destroy")

    def probe_stream_read_variant(self, buf, sink, wgs_per_cu, threads, in_flight, nontemporal):
        _check(lib().af_probe_stream_read_variant(self._h, _ptr(buf, torch.uint8), buf.numel(),
                                                  _ptr(sink, torch.float32), wgs_per_cu, threads,
                                                  in_flight, 1 if nontemporal else 0),
               "af_probe_stream_read_variant")

    # ---- threshold calibration ---------------------------------------------------------
    def calib_hist(self):
        return torch.zeros(AF_CALIB_BINS, dtype=torch.int32, device=self.device)

    def calib_accumulate(self, x, hist):
        _check(lib().af_calib_accumulate(self._h, _ptr(x, torch.float16, "x"), x.numel(),
                                         _ptr(hist, torch.int32, "hist")), "af_calib_accumulate")

    def calib_accumulate_layer(self, cfg: LayerCfg, hists):
        arr = (C.c_void_p * 4)(*[_ptr(h, torch.int32, "hist").value for h in hists])
        _check(lib().af_calib_accumulate_layer(self._h, C.byref(cfg), arr),
               "af_calib_accumulate_layer")

    def calib_thresholds(self, hist, sparsity_pct):
        lv = (C.c_int * len(sparsity_pct))(*[int(v) for v in sparsity_pct])
        out = torch.empty(len(sparsity_pct), dtype=torch.float32, device=self.device)
        _check(lib().af_calib_thresholds(self._h, _ptr(hist, torch.int32, "hist"), lv,
                                         len(sparsity_pct), _ptr(out, torch.float32)),
               "af_calib_thresholds")
        return out

    # ---- measurement -----------------------------------------------------------------
    def profile_set(self, stamps=None):
        """stamps: int64 CUDA tensor [n_slots, 2] (entry min, exit max per launch), or None."""
        if stamps is None:
            _check(lib().af_profile_set(self._h, None, 0), "af_profile_set")
        else:
            _check(lib().af_profile_set(self._h, _ptr(stamps, torch.int64, "stamps"),
                                        stamps.numel() // 2), "af_profile_set")

    def set_option(self, option: int, value: int):
        _check(lib().af_set_option(self._h, option, value), "af_set_option")

    def last_device_error(self, clear: bool = True) -> int:
        flags = C.c_int(0)
        _check(lib().af_last_device_error(self._h, C.byref(flags), 1 if clear else 0),
               "af_last_device_error")
        return flags.value

    def wall_clock_khz(self) -> int:
        return int(lib().af_wall_clock_khz(self._h))

    def probe_sink(self):
        return torch.zeros(lib().af_probe_sink_floats(self._h), dtype=torch.float32,
                           device=self.device)

    def probe_stream_read(self, buf, sink, wgs_per_cu: int = 8, offset: int = 0,
                          nbytes: int | None = None):
        """Queue one plain streaming read of buf[offset:offset+nbytes] (a uint8 CUDA tensor)."""
        nbytes = buf.numel() - offset if nbytes is None else nbytes
        _check(lib().af_probe_stream_read(self._h, C.c_void_p(_ptr(buf, torch.uint8).value + offset),
                                          nbytes, _ptr(sink, torch.float32), wgs_per_cu),
               "af_probe_stream_read")


# ---- host-side tools (no GPU needed) -------------------------------------------------------
class LfuCache:
    """Dynamic weight-cache simulator (Section 4.2) on host memory."""

    def __init__(self, n_channels: int, capacity: int, initial=()):
        init = (C.c_int32 * max(1, len(initial)))(*[int(v) for v in initial])
        h = C.c_void_p()
        _check(lib().af_lfu_create(C.byref(h), n_channels, capacity, init, len(initial)), "af_lfu_create")
        self._h, self.capacity = h, capacity
        self._ev = (C.c_int32 * max(1, capacity))()

    def step(self, idx):
        """idx: ascending unique channels of one token.  Returns (hits, loaded, evicted list)."""
        arr = (C.c_int32 * max(1, len(idx)))(*[int(v) for v in idx])
        h, l, ne = C.c_int(), C.c_int(), C.c_int()
        _check(lib().af_lfu_step(self._h, arr, len(idx), C.byref(h), C.byref(l), self._ev, C.byref(ne)),
               "af_lfu_step")
        return h.value, l.value, list(self._ev[: ne.value])

    def stats(self):
        v = [C.c_longlong() for _ in range(4)]
        _check(lib().af_lfu_stats(self._h, *[C.byref(x) for x in v]), "af_lfu_stats")
        return dict(zip(("tokens", "needed", "hits", "evictions"), [x.value for x in v]))

    def cached(self):
        out = (C.c_int32 * max(1, self.capacity))()
        n = C.c_int()
        _check(lib().af_lfu_cached(self._h, out, C.byref(n)), "af_lfu_cached")
        return list(out[: n.value])

    def close(self):
        if self._h:
            lib().af_lfu_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cost_eval(**kw) -> dict:
    cin, out = CostIn(**kw), CostOut()
    _check(lib().af_cost_eval(C.byref(cin), C.byref(out)), "af_cost_eval")
    return {n: getattr(out, n) for n, _ in CostOut._fields_}


def plan_search(M_max, S_m, S_l, M_kv, si, bw_mem, bw_flash_small, bw_flash_large, hr_points, n_max=64,
                min_gain=0.0) -> dict:
    """hr_points: [(cache fraction, hit rate), ...] with ascending fractions."""
    fr = (C.c_double * len(hr_points))(*[float(p[0]) for p in hr_points])
    hv = (C.c_double * len(hr_points))(*[float(p[1]) for p in hr_points])
    pin = PlanIn(M_max, S_m, S_l, M_kv, si, bw_mem, bw_flash_small, bw_flash_large, fr, hv, len(hr_points),
                 n_max, min_gain)
    out = PlanOut()
    _check(lib().af_plan_search(C.byref(pin), C.byref(out)), "af_plan_search")
    return {"sp": out.sp, "N": out.N, "visited": out.visited, "M_cache": out.M_cache, "hr": out.hr,
            "cost": {n: getattr(out.cost, n) for n, _ in CostOut._fields_}}
