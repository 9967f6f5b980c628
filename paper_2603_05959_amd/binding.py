"""ctypes binding of libovggt.so: same names as the C ABI (include/ovggt.h),
argument marshalling only.  Every step of the path runs in the HIP kernels;
torch supplies device memory and the stream.  There is no CPU fallback: a
missing library raises at first use."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("OVGGT_LIB") or os.path.join(_PKG, "libovggt.so")   # OVGGT_LIB: alternate build

OVGGT_F32, OVGGT_BF16 = 0, 1
OVGGT_ALL_LAYERS = -1
OVGGT_OK, OVGGT_ERR_ARG, OVGGT_ERR_STATE, OVGGT_ERR_NOMEM, OVGGT_ERR_HIP = 0, -1, -2, -3, -4
OVGGT_ERR_TOO_LARGE = -5
OVGGT_STATUS_BUDGET, OVGGT_STATUS_NONFINITE, OVGGT_STATUS_VRANGE = 1, 2, 4

EXPORTS = (
    "ovggt_cache_query_bytes", "ovggt_cache_init", "ovggt_global_attn", "ovggt_score_select",
    "ovggt_cache_compact", "ovggt_cache_destroy", "ovggt_cache_size", "ovggt_cache_frames",
    "ovggt_cache_status", "ovggt_cache_export", "ovggt_cache_import", "ovggt_cache_last_moves",
    "ovggt_profile_enable", "ovggt_profile_read", "ovggt_profile_overhead", "ovggt_strerror",
    "ovggt_cache_set_protect", "ovggt_dap_create", "ovggt_dap_step", "ovggt_dap_active", "ovggt_dap_destroy",
    "ovggt_attn_plan_stats", "ovggt_cache_flush", "ovggt_cache_advance",
    "ovggt_global_attn_static_ws",
)
PROF_CLASSES = ("append", "attn", "combine", "score_select", "compact")


class ovggt_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("tokens_per_frame", C.c_int32), ("resid_dim", C.c_int32), ("budget", C.c_int32),
                ("dtype", C.c_int32), ("score_mode", C.c_int32), ("softmax_scale", C.c_float),
                ("out_dtype", C.c_int32), ("smooth_alpha", C.c_float), ("patch_h", C.c_int32),
                ("patch_w", C.c_int32), ("n_special", C.c_int32), ("smooth_kernel", C.c_float * 9),
                ("hybrid_beta", C.c_float)]


class OvggtError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib() -> C.CDLL:
    """Load libovggt.so (built by paper_2603_05959_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2603_05959_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u8p, u32p = C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p
    szp = C.POINTER(C.c_size_t)
    cfgp = C.POINTER(ovggt_config)
    L.ovggt_cache_query_bytes.argtypes = [cfgp, szp, szp, szp]
    L.ovggt_cache_init.argtypes = [C.POINTER(vp), cfgp, vp, vp, vp, vp]
    L.ovggt_global_attn.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp]
    L.ovggt_global_attn_static_ws.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp]
    L.ovggt_score_select.argtypes = [vp, C.c_int, vp, u8p, vp]
    L.ovggt_cache_compact.argtypes = [vp, C.c_int, vp]
    L.ovggt_cache_flush.argtypes = [vp, C.c_int, vp]
    L.ovggt_cache_advance.argtypes = [vp, C.c_int, i64]
    L.ovggt_cache_destroy.argtypes = [vp]
    L.ovggt_cache_size.argtypes = [vp, C.c_int, C.POINTER(i32)]
    L.ovggt_cache_frames.argtypes = [vp, C.c_int, C.POINTER(i64)]
    L.ovggt_cache_status.argtypes = [vp, C.c_int, C.POINTER(i32), vp]
    L.ovggt_cache_export.argtypes = [vp, C.c_int, u32p, vp, vp, vp, u8p, vp]
    L.ovggt_cache_import.argtypes = [vp, C.c_int, i32, i64, u32p, vp, vp, vp, u8p, vp]
    L.ovggt_cache_last_moves.argtypes = [vp, C.c_int, u32p, u32p, C.POINTER(i32), vp]
    L.ovggt_profile_enable.argtypes = [vp, C.c_int, C.c_int]
    L.ovggt_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), vp]
    L.ovggt_profile_overhead.argtypes = [vp, C.c_int, C.POINTER(C.c_double), vp]
    L.ovggt_cache_set_protect.argtypes = [vp, C.c_int, i64, u8p, C.c_int, vp]
    L.ovggt_dap_create.argtypes = [C.POINTER(vp), i32, i32, C.c_double, C.c_double, i32, i32]
    L.ovggt_dap_step.argtypes = [vp, i64, C.c_double, vp, C.POINTER(i64), u8p, C.POINTER(i64)]
    L.ovggt_dap_active.argtypes = [vp, C.POINTER(i64), i32, C.POINTER(i32)]
    L.ovggt_dap_destroy.argtypes = [vp]
    L.ovggt_attn_plan_stats.argtypes = [cfgp, i32, i32, i32, C.POINTER(i32), C.POINTER(C.c_float)]
    L.ovggt_strerror.argtypes = [C.c_int]
    L.ovggt_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name != "ovggt_strerror":
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def strerror(code: int) -> str:
    return lib().ovggt_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != OVGGT_OK:
        raise OvggtError(code, where)


def _ptr(t) -> int:
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def make_config(n_layers, n_heads, head_dim, tokens_per_frame, resid_dim, budget, dtype,
                score_mode=0, softmax_scale=0.0, out_dtype="f32", smooth=None, hybrid_beta=0.0) -> ovggt_config:
    """smooth: None, or (alpha, patch_h, patch_w, n_special, kernel) with kernel nine floats, row-major.
    hybrid_beta: Eq. 7's beta, read when score_mode is 1."""
    codes = {"f32": OVGGT_F32, "bf16": OVGGT_BF16}
    cfg = ovggt_config(n_layers, n_heads, head_dim, tokens_per_frame, resid_dim, budget,
                       codes.get(dtype, dtype), score_mode, softmax_scale, codes.get(out_dtype, out_dtype))
    if smooth is not None:
        alpha, ph, pw, ns, kern = smooth
        cfg.smooth_alpha, cfg.patch_h, cfg.patch_w, cfg.n_special = float(alpha), int(ph), int(pw), int(ns)
        cfg.smooth_kernel = (C.c_float * 9)(*[float(x) for x in np.asarray(kern, dtype=np.float32).reshape(9)])
    cfg.hybrid_beta = float(hybrid_beta)
    return cfg


# ---- the C entry points, one wrapper each -----------------------------------
def ovggt_cache_query_bytes(cfg: ovggt_config) -> tuple[int, int, int]:
    kv, meta, ws = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().ovggt_cache_query_bytes(C.byref(cfg), C.byref(kv), C.byref(meta), C.byref(ws)),
           "ovggt_cache_query_bytes")
    return kv.value, meta.value, ws.value


def ovggt_cache_init(cfg: ovggt_config, kv_dev, meta_dev, ws_dev, stream: int = 0) -> int:
    h = C.c_void_p()
    _check(lib().ovggt_cache_init(C.byref(h), C.byref(cfg), _ptr(kv_dev), _ptr(meta_dev), _ptr(ws_dev), stream),
           "ovggt_cache_init")
    return h.value


def ovggt_global_attn(h, layer, q, k_new, v_new, out, stream: int = 0) -> None:
    _check(lib().ovggt_global_attn(h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream),
           "ovggt_global_attn")


def ovggt_global_attn_static_ws(h, layer, q, k_new, v_new, out, stream: int = 0) -> None:
    _check(lib().ovggt_global_attn_static_ws(h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream),
           "ovggt_global_attn_static_ws")


def ovggt_score_select(h, layer, resid, anchor_flags, stream: int = 0) -> None:
    _check(lib().ovggt_score_select(h, layer, _ptr(resid), _ptr(anchor_flags), stream), "ovggt_score_select")


def ovggt_cache_compact(h, layer, stream: int = 0) -> None:
    _check(lib().ovggt_cache_compact(h, layer, stream), "ovggt_cache_compact")


def ovggt_cache_flush(h, layer, stream: int = 0) -> None:
    _check(lib().ovggt_cache_flush(h, layer, stream), "ovggt_cache_flush")


def ovggt_cache_advance(h, layer, frames: int = 1) -> None:
    _check(lib().ovggt_cache_advance(h, layer, frames), "ovggt_cache_advance")


def ovggt_cache_destroy(h) -> None:
    _check(lib().ovggt_cache_destroy(h), "ovggt_cache_destroy")


def ovggt_cache_size(h, layer) -> int:
    n = C.c_int32()
    _check(lib().ovggt_cache_size(h, layer, C.byref(n)), "ovggt_cache_size")
    return n.value


def ovggt_cache_frames(h, layer) -> int:
    t = C.c_int64()
    _check(lib().ovggt_cache_frames(h, layer, C.byref(t)), "ovggt_cache_frames")
    return t.value


def ovggt_cache_status(h, layer, stream: int = 0) -> int:
    s = C.c_int32()
    _check(lib().ovggt_cache_status(h, layer, C.byref(s), stream), "ovggt_cache_status")
    return s.value


def ovggt_cache_export(h, layer, ids, k, v, ss, flags, stream: int = 0) -> None:
    _check(lib().ovggt_cache_export(h, layer, _ptr(ids), _ptr(k), _ptr(v), _ptr(ss), _ptr(flags), stream),
           "ovggt_cache_export")


def ovggt_cache_import(h, layer, n, frames, ids, k, v, ss, flags, stream: int = 0) -> None:
    _check(lib().ovggt_cache_import(h, layer, n, frames, _ptr(ids), _ptr(k), _ptr(v), _ptr(ss), _ptr(flags), stream),
           "ovggt_cache_import")


def ovggt_cache_last_moves(h, layer, dst, src, stream: int = 0) -> int:
    n = C.c_int32()
    _check(lib().ovggt_cache_last_moves(h, layer, _ptr(dst), _ptr(src), C.byref(n), stream),
           "ovggt_cache_last_moves")
    return n.value


def ovggt_cache_set_protect(h, layer, frame: int, mask, on: bool, stream: int = 0) -> None:
    _check(lib().ovggt_cache_set_protect(h, layer, frame, _ptr(mask), 1 if on else 0, stream),
           "ovggt_cache_set_protect")


def ovggt_dap_create(k_max: int, min_gap: int, tau: float, eta: float, n_special: int, n_patches: int):
    h = C.c_void_p()
    _check(lib().ovggt_dap_create(C.byref(h), k_max, min_gap, tau, eta, n_special, n_patches), "ovggt_dap_create")
    return h


def ovggt_dap_step(h, t: int, rho: float, conf, mask_out):
    """Returns (register_frame, demote_frame), each -1 for none; mask_out is filled on registration."""
    reg, dem = C.c_int64(), C.c_int64()
    _check(lib().ovggt_dap_step(h, t, rho, _ptr(conf), C.byref(reg), _ptr(mask_out), C.byref(dem)), "ovggt_dap_step")
    return reg.value, dem.value


def ovggt_dap_active(h, cap: int = 64) -> list:
    frames = (C.c_int64 * cap)()
    n = C.c_int32()
    _check(lib().ovggt_dap_active(h, frames, cap, C.byref(n)), "ovggt_dap_active")
    return [frames[i] for i in range(min(n.value, cap))]


def ovggt_dap_destroy(h) -> None:
    _check(lib().ovggt_dap_destroy(h), "ovggt_dap_destroy")


def ovggt_attn_plan_stats(cfg: ovggt_config, layers_in_launch: int, n_total: int, n_wgs: int) -> dict:
    out = (C.c_int32 * 8)()
    cost = (C.c_float * 2)()
    _check(lib().ovggt_attn_plan_stats(C.byref(cfg), layers_in_launch, n_total, n_wgs, out, cost),
           "ovggt_attn_plan_stats")
    keys = ("n_wgs", "rounds", "segments", "balanced", "pieces_max", "tiles_min", "tiles_max", "shared_items")
    d = dict(zip(keys, list(out)))
    d["cost_max"], d["cost_mean"] = cost[0], cost[1]
    return d


def ovggt_profile_enable(h, level: int, every: int = 1) -> None:
    _check(lib().ovggt_profile_enable(h, level, every), "ovggt_profile_enable")


def ovggt_profile_read(h, stream: int = 0) -> dict:
    ms = (C.c_double * len(PROF_CLASSES))()
    cnt = (C.c_int64 * len(PROF_CLASSES))()
    _check(lib().ovggt_profile_read(h, ms, cnt, stream), "ovggt_profile_read")
    return {name: (ms[i], cnt[i]) for i, name in enumerate(PROF_CLASSES)}


def ovggt_profile_overhead(h, reps: int = 64, stream: int = 0) -> float:
    ms = C.c_double()
    _check(lib().ovggt_profile_overhead(h, reps, C.byref(ms), stream), "ovggt_profile_overhead")
    return ms.value


# ---- convenience owner of the device buffers ---------------------------------
@dataclass
class _Bufs:
    kv: object
    meta: object
    ws: object


class Cache:
    """Allocates the three device buffers with torch and drives the C calls.
    Holds no logic of its own beyond marshalling."""

    def __init__(self, n_layers, n_heads, head_dim, tokens_per_frame, resid_dim, budget, dtype,
                 softmax_scale=0.0, device="cuda:0", out_dtype="f32", smooth=None, hybrid_beta=None):
        import torch
        self.torch = torch
        self.cfg = make_config(n_layers, n_heads, head_dim, tokens_per_frame, resid_dim, budget, dtype,
                               0 if hybrid_beta is None else 1, softmax_scale, out_dtype, smooth,
                               0.0 if hybrid_beta is None else hybrid_beta)
        self.dtype = dtype
        self.out_dtype = out_dtype
        self.L, self.H, self.d, self.M, self.Cdim, self.B = n_layers, n_heads, head_dim, tokens_per_frame, resid_dim, budget
        kvb, mb, wsb = ovggt_cache_query_bytes(self.cfg)
        self.bytes = (kvb, mb, wsb)
        self.device = torch.device(device)
        self.bufs = _Bufs(torch.empty(kvb, dtype=torch.uint8, device=self.device),
                          torch.empty(mb, dtype=torch.uint8, device=self.device),
                          torch.empty(wsb, dtype=torch.uint8, device=self.device))
        self.h = ovggt_cache_init(self.cfg, self.bufs.kv, self.bufs.meta, self.bufs.ws, self.stream)

    @property
    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def global_attn(self, q, k_new, v_new, out, layer=OVGGT_ALL_LAYERS):
        ovggt_global_attn(self.h, layer, q, k_new, v_new, out, self.stream)

    def score_select(self, resid, anchor_flags, layer=OVGGT_ALL_LAYERS):
        ovggt_score_select(self.h, layer, resid, anchor_flags, self.stream)

    def compact(self, layer=OVGGT_ALL_LAYERS):
        ovggt_cache_compact(self.h, layer, self.stream)

    def flush(self, layer=OVGGT_ALL_LAYERS):
        ovggt_cache_flush(self.h, layer, self.stream)

    def advance(self, frames=1, layer=OVGGT_ALL_LAYERS):
        ovggt_cache_advance(self.h, layer, frames)

    def step(self, q, k_new, v_new, resid, anchor_flags, out, layer=OVGGT_ALL_LAYERS):
        self.global_attn(q, k_new, v_new, out, layer)
        self.score_select(resid, anchor_flags, layer)
        self.compact(layer)

    def new_output(self):
        """Output tensor [L, M, H, d] of the handle's out_dtype."""
        t = self.torch
        return t.empty((self.L, self.M, self.H, self.d), device=self.device,
                       dtype=t.float32 if self.out_dtype == "f32" else t.bfloat16)

    def size(self, layer=0) -> int:
        return ovggt_cache_size(self.h, layer)

    def frames(self, layer=0) -> int:
        return ovggt_cache_frames(self.h, layer)

    def status(self, layer=0) -> int:
        return ovggt_cache_status(self.h, layer, self.stream)

    def export(self, layer=0) -> dict:
        """Logical view of a layer as numpy arrays (K/V as float32 values)."""
        n = self.size(layer)
        ids = np.zeros(n, np.uint32); ss = np.zeros(n, np.float32); flags = np.zeros(n, np.uint8)
        edt = np.uint16 if self.dtype == "bf16" else np.float32
        k = np.zeros((n, self.H, self.d), edt); v = np.zeros((n, self.H, self.d), edt)
        ovggt_cache_export(self.h, layer, ids, k, v, ss, flags, self.stream)
        if self.dtype == "bf16":
            k = (k.astype(np.uint32) << np.uint32(16)).view(np.float32)
            v = (v.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return {"ids": ids, "k": k, "v": v, "ss": ss, "flags": flags}

    def import_(self, layer, frames, ids, k_bits, v_bits, ss, flags):
        """k_bits / v_bits: numpy arrays already in the storage dtype (uint16 bf16 bits or float32)."""
        ids = np.ascontiguousarray(ids, np.uint32); ss = np.ascontiguousarray(ss, np.float32)
        flags = np.ascontiguousarray(flags, np.uint8)
        k_bits = np.ascontiguousarray(k_bits); v_bits = np.ascontiguousarray(v_bits)
        ovggt_cache_import(self.h, layer, len(ids), frames, ids, k_bits, v_bits, ss, flags, self.stream)

    def set_protect(self, frame, mask, on, layer=OVGGT_ALL_LAYERS):
        """mask: device uint8 tensor [M] or None (every token of the frame)."""
        ovggt_cache_set_protect(self.h, layer, frame, mask, on, self.stream)

    def last_moves(self, layer=0):
        dst = np.zeros(self.M, np.uint32); src = np.zeros(self.M, np.uint32)
        n = ovggt_cache_last_moves(self.h, layer, dst, src, self.stream)
        return dst[:n], src[:n]

    def close(self):
        if self.h:
            self.torch.cuda.synchronize(self.device)
            ovggt_cache_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def to_device(a: np.ndarray, dtype: str, device="cuda:0"):
    """numpy float32 (already quantised) -> torch tensor of the run dtype on the device."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.float32 and dtype == "bf16":
        return t.to(device).to(torch.bfloat16)       # exact: values are bf16-representable
    return t.to(device)
