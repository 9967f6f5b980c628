"""Seeded synthetic VGGT-shaped streams.

This module only *draws inputs*: per-frame Q/K/V tensors, per-token FFN-residual
rows and the anchor bits a Dynamic-Anchor-Protection policy would hand to the
cache.  It contains none of the method's arithmetic (no attention, no scoring,
no selection) and is the single piece of code that both the CPU oracle's tests
and the HIP path's tests/bench consume, so both sides see identical bytes.

Shapes follow the paper's streaming setting (Sec. 3.1): M = 1 camera + 4
register + N_p patch tokens per frame, 16 heads x 64, model width 1024, one
cache per global-attention layer.  Value distributions are stand-ins for real
StreamVGGT activations (datasets and weights are not available): the paper does
not report residual-norm statistics, so log-normal / Pareto norms are used.

Every tensor is a pure function of (seed, layer, frame, tensor id): a Philox
counter-based generator is keyed on that tuple, so any frame of any stream can
be regenerated in isolation and in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

BASE_SEED = 260305959

_TID_Q, _TID_K, _TID_V, _TID_R, _TID_NORM, _TID_DUP, _TID_DAP = 1, 2, 3, 4, 5, 6, 7


@dataclass(frozen=True)
class StreamConfig:
    name: str
    M: int                 # tokens per frame
    H: int                 # heads
    d: int                 # head dim
    C: int                 # residual (model) width
    B: int                 # cache budget per layer, protected tokens included
    T: int                 # frames
    L: int                 # independent layers
    dtype: str             # "f32" | "bf16"
    n_special: int         # camera + register tokens at the head of each frame
    resid: str             # "rowsigma" | "lognormal_unit" | "pareto_dup"
    anchors: str           # "frame0+camera" | "frame0+special" | "cap10"
    seed: int = BASE_SEED

    def with_(self, **kw) -> "StreamConfig":
        return replace(self, **kw)


def preset(k: int, **overrides) -> StreamConfig:
    """The five benchmark workloads (index = position in the workload list), and 5: the camera head's cache."""
    if k == 0:
        c = StreamConfig("cfg0-tiny", 65, 2, 64, 128, 256, 10, 1, "f32", 1,
                         "rowsigma", "frame0+camera")
    elif k == 1:
        c = StreamConfig("cfg1-vggt-layer", 1374, 16, 64, 1024, 16384, 200, 1, "bf16", 5,
                         "lognormal_unit", "frame0+special")
    elif k == 2:
        c = StreamConfig("cfg2-24-layers", 1374, 16, 64, 1024, 16384, 500, 24, "bf16", 5,
                         "lognormal_unit", "frame0+special")
    elif k == 3:
        c = StreamConfig("cfg3-ultra-long", 1374, 16, 64, 1024, 32768, 2000, 1, "bf16", 5,
                         "pareto_dup", "frame0+special")
    elif k == 4:
        c = StreamConfig("cfg4-518x392", 1041, 16, 64, 1024, 8192, 1000, 1, "bf16", 5,
                         "lognormal_unit", "cap10")
    elif k == 5:
        # the camera head's cache (Supp. C): one token per frame, budget = the frames the 24-layer
        # aggregator budget of the 518x392 runs holds (24 * 8192 / 1041 = 188); head shape assumed
        c = StreamConfig("cfg5-camera-head", 1, 16, 64, 1024, 188, 2000, 1, "bf16", 1,
                         "lognormal_unit", "frame0")
    else:
        raise ValueError(f"no preset {k}")
    return c.with_(**overrides) if overrides else c


CFG4_BUDGETS = (4096, 8192, 32768, 65536)


def patch_grid(cfg: "StreamConfig") -> tuple[int, int]:
    """(rows, columns) of the frame's patch map: the most nearly square factorisation of
    M - n_special (37 x 37 for 518 x 518 input at patch size 14, 37 x 28 for 518 x 392)."""
    p = cfg.M - cfg.n_special
    w = max(x for x in range(1, int(p ** 0.5) + 1) if p % x == 0)
    return p // w, w


def gaussian_kernel3(sigma: float = 1.0) -> np.ndarray:
    """A normalised 3x3 Gaussian as float32 [3, 3]: the smoothing kernel handed to both the library
    and the oracle as a workload parameter (the paper gives no size or width for its G)."""
    w = np.exp(-0.5 * (np.array([-1.0, 0.0, 1.0]) / sigma) ** 2)
    k = np.outer(w, w)
    return (k / k.sum()).astype(np.float32)


# --------------------------------------------------------------------------- #
# number formats
# --------------------------------------------------------------------------- #
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantise(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the run's storage type; result is float32 holding exactly
    representable values (what both the oracle and the device then see)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(a))
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# counter-based draws
# --------------------------------------------------------------------------- #
def _rng(cfg: StreamConfig, layer: int, frame: int, tid: int) -> np.random.Generator:
    key = np.array([np.uint64(cfg.seed + layer),
                    (np.uint64(frame) << np.uint64(8)) | np.uint64(tid)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _base_resid(cfg: StreamConfig, layer: int, t: int) -> np.ndarray:
    """Residual rows of frame t before any duplication, float32 [M, C]."""
    g = _rng(cfg, layer, t, _TID_R).standard_normal((cfg.M, cfg.C), dtype=np.float32)
    z = _rng(cfg, layer, t, _TID_NORM)
    if cfg.resid == "rowsigma":
        sigma = np.exp(0.5 * z.standard_normal(cfg.M)).astype(np.float32)
        return g * sigma[:, None]
    unit = g / np.linalg.norm(g.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    if cfg.resid == "lognormal_unit":
        norm = np.exp(z.standard_normal(cfg.M))
    elif cfg.resid == "pareto_dup":
        u = 1.0 - z.random(cfg.M)            # (0, 1]
        norm = u ** (-1.0 / 1.5)             # Pareto(alpha=1.5, x_m=1)
    else:
        raise ValueError(cfg.resid)
    return unit * norm.astype(np.float32)[:, None]


def resid_rows(cfg: StreamConfig, layer: int, t: int) -> np.ndarray:
    """Quantised FFN-residual rows [M, C] of frame t."""
    r = _base_resid(cfg, layer, t)
    if cfg.resid == "pareto_dup":
        # 5 % of the rows become bit-identical copies of another row (of this
        # frame or of the previous one) so that equal scores really occur.
        g = _rng(cfg, layer, t, _TID_DUP)
        n_dup = max(1, (cfg.M * 5) // 100)
        dst = g.choice(cfg.M, size=n_dup, replace=False)
        src = g.integers(0, cfg.M, size=n_dup)
        from_prev = (g.random(n_dup) < 0.5) & (t > 0)
        prev = _base_resid(cfg, layer, t - 1) if from_prev.any() else None
        base = r.copy()
        for i, j, p in zip(dst, src, from_prev):
            r[i] = prev[j] if p else base[j]
    return quantise(r, cfg.dtype)


def anchor_bits(cfg: StreamConfig, t: int) -> np.ndarray:
    """uint8[M]: 1 where the caller's anchor policy protects the new token."""
    a = np.zeros(cfg.M, dtype=np.uint8)
    if cfg.anchors == "frame0+camera":
        if t == 0:
            a[:] = 1
        a[0] = 1
    elif cfg.anchors == "frame0+special":
        if t == 0:
            a[:] = 1
        a[:cfg.n_special] = 1
    elif cfg.anchors == "frame0":
        if t == 0:
            a[:] = 1
    elif cfg.anchors == "cap10":
        cap = cfg.B // 10
        if t == 0:
            a[:min(cap, cfg.M)] = 1
        elif cap > cfg.M and cfg.M + t * cfg.n_special <= cap:
            a[:cfg.n_special] = 1
    else:
        raise ValueError(cfg.anchors)
    return a


def n_protected(cfg: StreamConfig, t: int) -> int:
    """|P| after frame t when nothing protected was ever demoted."""
    return int(sum(int(anchor_bits(cfg, s).sum()) for s in range(t + 1)))


def frame_inputs(cfg: StreamConfig, layer: int, t: int, want=("q", "k", "v", "r", "a")) -> dict:
    """Inputs of one (layer, frame): q,k,v float32 [M,H,d]; r float32 [M,C];
    a uint8 [M].  All floats already rounded to cfg.dtype."""
    out = {}
    shape = (cfg.M, cfg.H, cfg.d)
    for name, tid in (("q", _TID_Q), ("k", _TID_K), ("v", _TID_V)):
        if name in want:
            x = _rng(cfg, layer, t, tid).standard_normal(shape, dtype=np.float32)
            out[name] = quantise(x, cfg.dtype)
    if "r" in want:
        out["r"] = resid_rows(cfg, layer, t)
    if "a" in want:
        out["a"] = anchor_bits(cfg, t)
    return out


def coverage_and_confidence(cfg: StreamConfig, t: int) -> tuple[float, np.ndarray]:
    """Stand-ins for the two model outputs the anchor policy consumes at frame t: the coverage
    ratio rho_t (uniform in [0, 1)) and the point head's per-patch confidence (log-normal, with
    a share of exact repeats so that equal confidences occur), float32 [M - n_special]."""
    rng = _rng(cfg, 0, t, _TID_DAP)
    rho = float(rng.random())
    n_p = cfg.M - cfg.n_special
    conf = np.exp(rng.standard_normal(n_p)).astype(np.float32)
    rep = rng.random(n_p) < 0.2
    conf[rep] = np.float32(1.0)
    return rho, conf


def rising_resid(cfg: StreamConfig, layer: int, t: int) -> np.ndarray:
    """Worst case for compaction: norms grow with t, so every new token
    survives and M scattered old ones are evicted each frame."""
    g = _rng(cfg, layer, t, _TID_R).standard_normal((cfg.M, cfg.C), dtype=np.float32)
    unit = g / np.linalg.norm(g.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    jitter = _rng(cfg, layer, t, _TID_NORM).random(cfg.M).astype(np.float32)
    return quantise(unit * (np.float32(1.0 + t) + jitter)[:, None], cfg.dtype)
