"""CPU oracle for the OVGGT streaming hot path.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
import this file; the product path never does.  It shares no code with the HIP
library and is written for readability, not speed: plain numpy, fp64 attention,
fp32 scores with a fixed summation order, a full sort for the top-k.

What it computes, per layer, for every incoming frame t (paper Sec. 3.1-3.3):

  1. append   C_t = [C_{t-1}; (K_t, V_t)]                        (Eq. 2)
  2. attend   O_t = softmax(Q_t K_c^T / sqrt(d)) V_c over every resident entry,
              the frame's own tokens included (the temporal causal attention
              CA of Sec. 3.1; causality is frame-level, so one frame at a time
              needs no mask)
  3. score    s_i = || FFN residual of token i ||_2               (Eq. 5)
  4. protect  tokens named by Dynamic Anchor Protection form P     (Sec. 3.3)
  5. select   C~_t = P  U  Top-k(U, B - |P|)                       (Eq. 8)
  6. compact  evicted entries leave the arrays; size becomes min(n, B)

Readings taken where the paper is silent (each is listed in the design notes):
  * every cached token keeps the activation score it received on entry
    (stored-score policy); the paper's hybrid re-scoring of history (Eq. 7) is
    `hybrid_rank` below and is only used when asked for;
  * ranking uses ss = s^2 (same order as s, no square-root rounding);
  * ss is an fp32 balanced-binary-tree sum of fp32 squares (so a GPU wave can
    reproduce it bit for bit);
  * ties are broken by token id: the older token (lower id) wins;
  * layout after eviction: the r-th vacated slot below B receives the r-th
    surviving entry at or above B, both in ascending slot order.

Pins (see tests/test_oracle_pins.py): single key => O = V; equal keys => mean
of V; dominant key; agreement with a two-pass fp32 formulation and with a
library attention routine; budget >= stream length reproduces uncompressed
causal streaming attention; |C~_t| = min((t+1)M, B); anchors never leave;
brute-force top-k on tiny inputs; whole-stream closed form of the kept set;
exact integer / power-of-two score rows and a crafted row that separates the
tree order from left-to-right order; Eq. 9's bound on |P|; the 2 L T M N_h d
footprint with the paper's "~10 GB at 100 frames" example.
Parity unpinned by the paper: the slot layout after eviction (our definition,
pinned only by exhaustive tiny cases and by permutation invariance of
attention), `hybrid_rank` beyond its degenerate cases, and the kernel size, width and
padding of the activation smoothing (`smoothed_keys_f32`, `smooth_scores`).
"""
from __future__ import annotations

import numpy as np


class BudgetError(Exception):
    """|P| exceeds the budget B: Eq. 8 would ask for a negative k."""


# --------------------------------------------------------------------------- #
# Eq. 5 -- activation score
# --------------------------------------------------------------------------- #
def tree_sum_sq_f32(r: np.ndarray) -> np.ndarray:
    """ss_i = sum_c r[i,c]^2 in fp32, rows of `r` [n, C].

    Each square is rounded to fp32 once; the C squares are zero-padded to a
    power of two and added pairwise, neighbours first ((0+1), (2+3), ...),
    level by level, every add rounded to fp32.
    """
    r = np.asarray(r, dtype=np.float32)
    if r.ndim == 1:
        r = r[None, :]
    return tree_sum_f32(r * r)                    # fp32 x fp32 -> fp32, one rounding


def tree_sum_f32(p: np.ndarray) -> np.ndarray:
    """Row sums of fp32 terms `p` [n, C] in the balanced-tree order described above."""
    p = np.asarray(p, dtype=np.float32)
    width = 1
    while width < p.shape[1]:
        width *= 2
    if width != p.shape[1]:
        p = np.concatenate([p, np.zeros((p.shape[0], width - p.shape[1]), np.float32)], axis=1)
    while p.shape[1] > 1:
        p = p[:, 0::2] + p[:, 1::2]               # fp32 adds
    return p[:, 0].astype(np.float32)


def activation_score(r: np.ndarray) -> np.ndarray:
    """s_i of Eq. 5 (informational; ranking uses ss)."""
    return np.sqrt(tree_sum_sq_f32(r))


# --------------------------------------------------------------------------- #
# Sec. 3.1 -- attention of the new frame's queries over the cache
# --------------------------------------------------------------------------- #
def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None) -> np.ndarray:
    """softmax(q k^T * scale) v per head, fp64.

    q [M,H,d], k and v [n,H,d] (every resident cache entry).  Returns [M,H,d].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    M, H, d = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((M, H, d), dtype=np.float64)
    for h in range(H):
        logits = (q[:, h, :] @ k[:, h, :].T) * scale          # [M, n]
        logits -= logits.max(axis=1, keepdims=True)
        w = np.exp(logits)
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v[:, h, :]
    return out


# --------------------------------------------------------------------------- #
# Eq. 8 -- which entries stay
# --------------------------------------------------------------------------- #
def rank_order(ss: np.ndarray, gid: np.ndarray) -> np.ndarray:
    """Indices sorted best-first: larger ss first, equal ss -> lower id first.
    A NaN score ranks as +0 (lowest)."""
    ss = np.asarray(ss, dtype=np.float32)
    key = np.where(np.isnan(ss), np.float32(0), ss).astype(np.float64)
    return np.lexsort((np.asarray(gid, dtype=np.int64), -key))


def select_keep(ss: np.ndarray, gid: np.ndarray, flag: np.ndarray, budget: int) -> np.ndarray:
    """Boolean keep mask over the n resident entries.

    n <= B keeps everything.  Otherwise the protected entries P (flag != 0) stay
    and the k = B - |P| best evictable entries join them.
    """
    n = len(ss)
    flag = np.asarray(flag) != 0
    if n <= budget:
        return np.ones(n, dtype=bool)
    n_prot = int(flag.sum())
    k = budget - n_prot
    if k < 0:
        raise BudgetError(f"|P|={n_prot} > B={budget}")
    evictable = np.flatnonzero(~flag)
    order = rank_order(np.asarray(ss)[evictable], np.asarray(gid)[evictable])
    keep = flag.copy()
    keep[evictable[order[:k]]] = True
    return keep


def hole_fill_moves(keep: np.ndarray, budget: int) -> tuple[np.ndarray, np.ndarray]:
    """(dst, src) slot pairs: vacated slots below B in ascending order receive
    the kept slots at or above B in ascending order."""
    keep = np.asarray(keep, dtype=bool)
    holes = np.flatnonzero(~keep[:budget])
    movers = budget + np.flatnonzero(keep[budget:])
    assert len(holes) == len(movers)
    return holes, movers


# --------------------------------------------------------------------------- #
# the per-layer streaming cache
# --------------------------------------------------------------------------- #
class OracleCache:
    """One layer's KV cache with scores, ids and protection flags per slot."""

    def __init__(self, M: int, H: int, d: int, budget: int, scale: float | None = None, smooth=None,
                 hybrid_beta: float | None = None):
        """smooth: None (rank key = ss), or (alpha, patch_h, patch_w, n_special, kernel 3x3) to rank
        by the smoothed activation map of Eq. 6 (see `smoothed_keys_f32`).
        hybrid_beta: None ranks every entry by the score it entered with; a value in [0, 1]
        ranks by Eq. 7 (see `hybrid_keys_f32`) whenever something has to be evicted, and the
        rank value r replaces the stored score of every evictable entry."""
        if budget < M:
            raise ValueError("budget must hold at least one frame")
        self.M, self.H, self.d, self.B = M, H, d, budget
        self.scale = scale
        self.smooth = smooth
        self.hybrid_beta = hybrid_beta
        self.k = np.zeros((0, H, d), np.float32)
        self.v = np.zeros((0, H, d), np.float32)
        self.gid = np.zeros(0, np.uint32)
        self.ss = np.zeros(0, np.float32)
        self.flag = np.zeros(0, np.uint8)
        self.t = 0                       # frames seen
        self.nan_seen = False

    @property
    def n(self) -> int:
        return len(self.gid)

    # step 1 (Eq. 2)
    def append(self, k_t: np.ndarray, v_t: np.ndarray) -> None:
        M = self.M
        assert k_t.shape == (M, self.H, self.d) and v_t.shape == k_t.shape
        self.k = np.concatenate([self.k, np.asarray(k_t, np.float32)])
        self.v = np.concatenate([self.v, np.asarray(v_t, np.float32)])
        self.gid = np.concatenate([self.gid, (self.t * M + np.arange(M)).astype(np.uint32)])
        self.ss = np.concatenate([self.ss, np.zeros(M, np.float32)])
        self.flag = np.concatenate([self.flag, np.zeros(M, np.uint8)])

    # step 2
    def attend(self, q_t: np.ndarray) -> np.ndarray:
        return attention(q_t, self.k, self.v, self.scale)

    # steps 3-6
    def update(self, resid_t: np.ndarray, anchor_t: np.ndarray | None) -> np.ndarray:
        """Score the M newest entries, flag anchors, select, compact.
        Returns the keep mask over the pre-compaction slots."""
        M, n = self.M, self.n
        ss_new = tree_sum_sq_f32(resid_t)
        assert ss_new.shape == (M,)
        if self.smooth is not None:
            ss_new = smoothed_keys_f32(ss_new, *self.smooth)
        flag_new = np.zeros(M, np.uint8) if anchor_t is None else (np.asarray(anchor_t) != 0).astype(np.uint8)
        ss = self.ss.copy(); ss[n - M:] = ss_new
        flag = self.flag.copy(); flag[n - M:] = flag_new
        if self.hybrid_beta is not None and n > self.B:
            s_new = ss_new if self.smooth is not None else np.sqrt(ss_new)       # fp32, correctly rounded
            r = hybrid_keys_f32(cached_half(self.k), flag, M, s_new, self.hybrid_beta)
            ss = np.where(flag != 0, ss, r).astype(np.float32)
        keep = select_keep(ss, self.gid, flag, self.B)     # raises before any state change
        self.ss, self.flag = ss, flag
        if np.isnan(ss_new).any():
            self.nan_seen = True
        if n > self.B:
            dst, src = hole_fill_moves(keep, self.B)
            for arr in (self.k, self.v, self.gid, self.ss, self.flag):
                arr[dst] = arr[src]
            self.k, self.v = self.k[:self.B], self.v[:self.B]
            self.gid, self.ss, self.flag = self.gid[:self.B], self.ss[:self.B], self.flag[:self.B]
        self.t += 1
        return keep

    # Sec. 3.3, historical anchors: protection granted or withdrawn after the tokens were cached
    def set_protect(self, frame: int, mask: np.ndarray | None, on: bool) -> int:
        """Flag (on) or release (off) the still-resident tokens of frame `frame` whose bit in
        `mask` [M] is set (None: every token of the frame).  Evicted tokens cannot be brought
        back, so a late registration covers what is left of the frame.  A released token returns
        to the evictable set with the score it holds.  Returns how many flags changed."""
        local = self.gid.astype(np.int64) - frame * self.M
        hit = (local >= 0) & (local < self.M)
        if mask is not None:
            m = np.asarray(mask) != 0
            hit &= m[np.clip(local, 0, self.M - 1)]
        new = np.uint8(1 if on else 0)
        changed = int((hit & (self.flag != new)).sum())
        self.flag[hit] = new
        return changed

    def step(self, q_t, k_t, v_t, resid_t, anchor_t, attend: bool = True):
        """One frame through steps 1-6; returns O_t (or None when attend=False:
        cache contents never depend on attention outputs)."""
        self.append(k_t, v_t)
        out = self.attend(q_t) if attend else None
        self.update(resid_t, anchor_t)
        return out


# --------------------------------------------------------------------------- #
# Sec. 3.3 -- which frames become historical anchors, and which tokens of them
# --------------------------------------------------------------------------- #
class DapPolicy:
    """The registration rule of Dynamic Anchor Protection, given the model's outputs as inputs.

    Frame 0 is the global initial anchor: the caller protects all of its tokens when they are
    inserted, it is never demoted and does not count towards K_max; it is the reference of the
    first coverage test.  At frame t > 0 with coverage ratio rho_t (fraction of the latest
    anchor's points that project inside the current image), a new anchor is registered when
    rho_t < tau and at least `min_gap` frames have passed since the last registration (frame 0
    counts as one).  Of the anchor frame's N_p patch tokens the ceil(eta * N_p) with the highest
    per-point confidence are protected (equal confidences: lower patch index first); aux tokens
    are not.  At most K_max historical anchors are active; registering one more demotes the
    oldest (first in, first out).  |P| <= M + K_max * ceil(eta * N_p) (Eq. 9).
    Ties, the role of frame 0 in the spacing rule and the treatment of aux tokens are this
    build's reading."""

    def __init__(self, k_max: int, min_gap: int, tau: float, eta: float, n_special: int, n_patches: int):
        assert k_max >= 1 and min_gap >= 1 and 0 < eta <= 1 and n_patches >= 1 and n_special >= 0
        self.k_max, self.min_gap, self.tau, self.eta = k_max, min_gap, float(tau), float(eta)
        self.n_special, self.n_patches = n_special, n_patches
        self.last_reg = 0
        self.active: list[int] = []                    # oldest first

    @property
    def per_anchor(self) -> int:
        return int(np.ceil(self.eta * self.n_patches))

    def step(self, t: int, rho: float, conf: np.ndarray):
        """Returns (mask, demoted): mask is a uint8 [M] array of the tokens of frame t to
        protect, or None when frame t does not become an anchor; demoted is the frame whose
        protection is to be released, or None."""
        if t <= 0 or not (rho < self.tau) or t - self.last_reg < self.min_gap:
            return None, None
        conf = np.asarray(conf, dtype=np.float32)
        assert conf.shape == (self.n_patches,)
        order = np.lexsort((np.arange(self.n_patches), -conf.astype(np.float64)))   # confidence desc, index asc
        mask = np.zeros(self.n_special + self.n_patches, np.uint8)
        mask[self.n_special + order[:self.per_anchor]] = 1
        demoted = self.active.pop(0) if len(self.active) == self.k_max else None
        self.active.append(t)
        self.last_reg = t
        return mask, demoted


# --------------------------------------------------------------------------- #
# widening rows: the paper's own treatment of history and of the score map
# --------------------------------------------------------------------------- #
def minmax01(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if x.size == 0:
        return x
    lo, hi = x.min(), x.max()
    return np.zeros_like(x) if hi == lo else (x - lo) / (hi - lo)


def hybrid_rank(k_hist: np.ndarray, s_new: np.ndarray, beta: float) -> tuple[np.ndarray, np.ndarray]:
    """Eq. 7: r = (1-beta) * minmax(1 - cos(k_i, kbar)) for evictable history,
    r = beta * minmax(s_i) for the current frame.  k_hist [n, H*d] with kbar the
    centroid of those rows.  PARITY UNPINNED beyond beta in {0,1} and range."""
    k = np.asarray(k_hist, dtype=np.float64).reshape(len(k_hist), -1)
    if len(k):
        kbar = k.mean(axis=0)
        cos = (k @ kbar) / (np.linalg.norm(k, axis=1) * np.linalg.norm(kbar))
        d = 1.0 - cos
    else:
        d = np.zeros(0)
    return (1.0 - beta) * minmax01(d), beta * minmax01(s_new)


def cached_half(k: np.ndarray) -> np.ndarray:
    """The keys as a bf16 cache holds them: the IEEE half nearest each given value (ties to
    even, 2^-24 grid below 2^-14), saturated at +-65504; returned as fp32."""
    with np.errstate(over="ignore"):
        return np.clip(np.asarray(k, np.float32), -65504.0, 65504.0).astype(np.float16).astype(np.float32)


def hybrid_keys_f32(k_half: np.ndarray, flag: np.ndarray, n_new: int, s_new: np.ndarray, beta: float) -> np.ndarray:
    """Eq. 7 rank values r for every resident entry, as one fixed fp32 operation sequence.

    k_half [n, H, d] (or [n, H*d]): half-representable key values; a token's key vector is the
    concatenation over heads.  The last n_new entries are the current frame, whose scores
    (s of Eq. 5, or Eq. 6's smoothed s) are `s_new`; the others are history.  Flagged entries
    are in P and get r = NaN here (callers ignore them).

    Centroid: the sum of the evictable history keys, accumulated exactly (every half is an
    integer multiple of 2^-24, the integer sum cannot overflow 64 bits below 2^17 entries),
    then rounded integer -> fp64 -> fp32 and scaled by 2^-24.  The cosine does not depend on
    the centroid's length, so the sum stands for the mean.  Per history token, in fp32:
    dot = tree(k_j * c_j), nk = tree(k_j^2), nc = tree(c_j^2) (the balanced tree of
    `tree_sum_f32`), cos = dot / (sqrt(nk) * sqrt(nc)) (0 when that product is 0), d = 1 - cos.
    Min-max: x^ = (x - min) / (max - min) over the evictable set of each source, all zeros when
    max = min; r = (1 - beta) * d^ for history, beta * s^ for the current frame.
    Which tokens form the centroid, whether keys are taken per head, and the degenerate
    cases are this build's reading (parity unpinned by the paper)."""
    f32 = np.float32
    k = np.asarray(k_half, dtype=np.float32)
    n = len(k)
    k = k.reshape(n, -1)
    flag = np.asarray(flag) != 0
    idx = np.arange(n)
    hist = (idx < n - n_new) & ~flag
    new = (idx >= n - n_new) & ~flag
    r = np.full(n, np.nan, np.float32)
    b = f32(beta)
    if hist.any():
        fixed = k[hist].astype(np.float64) * 2.0 ** 24
        assert np.array_equal(fixed, np.rint(fixed)) and np.abs(fixed).max(initial=0) < 2.0 ** 41 and hist.sum() < 2 ** 17
        csum = fixed.astype(np.int64).sum(axis=0)                       # exact
        c = csum.astype(np.float64).astype(np.float32) * f32(2.0 ** -24)  # two roundings, then an exact scaling
        kh = k[hist]
        nc = tree_sum_f32((c * c)[None, :])[0]
        nk = tree_sum_f32(kh * kh)
        dot = tree_sum_f32(kh * c[None, :])
        den = np.sqrt(nk) * np.sqrt(nc)
        with np.errstate(divide="ignore", invalid="ignore"):
            cos = np.where(den == 0, f32(0), dot / den).astype(np.float32)
        d = f32(1) - cos
        r[hist] = (f32(1) - b) * _minmax01_f32(d)
    if new.any():
        sn = np.asarray(s_new, dtype=np.float32)[new[n - n_new:]]
        r[new] = b * _minmax01_f32(sn)
    return r


def _minmax01_f32(x: np.ndarray) -> np.ndarray:
    lo, hi = x.min(), x.max()
    if hi == lo:
        return np.zeros_like(x)
    return (x - lo) / (hi - lo)


def smoothed_keys_f32(ss_new: np.ndarray, alpha: float, ph: int, pw: int, n_special: int, g) -> np.ndarray:
    """Rank keys of one frame's tokens under activation smoothing (Eq. 6).

    s = sqrt(ss) (Eq. 5's score) in fp32; the last ph*pw tokens are the patch map S in row-major
    order and become alpha*(G*S) + (1-alpha)*S; the first n_special (aux) tokens keep s, as the
    paper says.  G is a 3x3 kernel given by the caller (the paper fixes neither size nor width),
    applied with the border replicated: tap (a, b) weighs S[y+a-1, x+b-1], which is the
    convolution for the symmetric kernels Eq. 6 means.  Every operation is a separate fp32
    operation, taps added left to right in kernel order, so a GPU thread can repeat it bit for
    bit: the smoothed value decides which tokens survive.  Pinned against `smooth_scores` (the
    same formula in fp64), alpha = 0, a constant map, an impulse and a hand-computed 2x2 case;
    kernel size, width and padding remain this build's reading (parity unpinned by the paper)."""
    f32 = np.float32
    ss_new = np.asarray(ss_new, dtype=f32)
    assert n_special + ph * pw == len(ss_new)
    g = np.asarray(g, dtype=f32).reshape(3, 3)
    a = f32(alpha)
    with np.errstate(invalid="ignore"):
        s = np.sqrt(ss_new)                                   # correctly rounded in fp32
    S = s[n_special:].reshape(ph, pw)
    pad = np.pad(S, 1, mode="edge")
    conv = None
    for dy in range(3):
        for dx in range(3):
            prod = g[dy, dx] * pad[dy:dy + ph, dx:dx + pw]    # fp32 product, rounded
            conv = prod if conv is None else conv + prod      # fp32 add, rounded
    out = s.copy()
    out[n_special:] = (a * conv + (f32(1.0) - a) * S).reshape(-1)
    return out


def smooth_scores(s_patch: np.ndarray, alpha: float, g: np.ndarray) -> np.ndarray:
    """Eq. 6: S~ = alpha (G * S) + (1-alpha) S on the H_p x W_p patch map, with
    an explicit normalised kernel `g` and replicate padding, in fp64.  Pinned by
    alpha = 0 and a constant map; kernel size, sigma and padding are this
    build's reading (parity unpinned by the paper)."""
    s = np.asarray(s_patch, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    ry, rx = g.shape[0] // 2, g.shape[1] // 2
    pad = np.pad(s, ((ry, ry), (rx, rx)), mode="edge")
    conv = np.zeros_like(s)
    for dy in range(g.shape[0]):
        for dx in range(g.shape[1]):
            conv += g[dy, dx] * pad[dy:dy + s.shape[0], dx:dx + s.shape[1]]
    return alpha * conv + (1.0 - alpha) * s
