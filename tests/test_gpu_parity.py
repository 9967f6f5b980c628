"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Kept ids / slot layout / scores / flags / K / V must be
bit-exact; attention outputs must agree within 1e-4 (f32) or 2e-2 (bf16) of the
output RMS per frame (max-abs over the frame's [M,H,d] block)."""
import numpy as np
import pytest

from oracle import ovggt_oracle as oc
from paper_2603_05959_amd import binding as B
from paper_2603_05959_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _torch():
    import torch
    return torch


def make_cache(cfg, L=None, smooth=None, hybrid_beta=None):
    return B.Cache(L or cfg.L, cfg.H, cfg.d, cfg.M, cfg.C, cfg.B, cfg.dtype, smooth=smooth, hybrid_beta=hybrid_beta)


def dev(a, cfg):
    return B.to_device(a, cfg.dtype)


def rel_err(o_gpu, o_ref):
    return float(np.abs(o_gpu - o_ref).max() / np.sqrt((o_ref ** 2).mean()))


def stored_v(v, dtype):
    """What export returns for K and V: bf16 handles keep both as IEEE half (exact for
    every normal half value, 2^-24 grid below 2^-14) and hand them back as bf16."""
    if dtype != "bf16":
        return v
    with np.errstate(over="ignore"):
        h = np.clip(v, -65504.0, 65504.0).astype(np.float16).astype(np.float32)
    return synth.quantise(h, "bf16")


def compare_cache(cache, orc, layer=0, kv=True):
    e = cache.export(layer)
    assert len(e["ids"]) == orc.n
    assert np.array_equal(e["ids"], orc.gid), "kept ids / layout differ"
    assert np.array_equal(e["ss"].view(np.uint32), orc.ss.view(np.uint32)), "scores differ"
    assert np.array_equal(e["flags"], orc.flag)
    if kv:
        assert np.array_equal(e["k"], stored_v(orc.k, cache.dtype))
        assert np.array_equal(e["v"], stored_v(orc.v, cache.dtype))


def run_stream(cfg, layer=0, attn_frames=None, cache_every=1, resid_fn=None, q_rows=None, log=None, smooth=None,
               hybrid_beta=None, qkv_fn=None):
    """Drive both sides over cfg.T frames of one layer; returns max attention error."""
    torch = _torch()
    cache = make_cache(cfg, L=1, smooth=smooth, hybrid_beta=hybrid_beta)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, smooth=smooth, hybrid_beta=hybrid_beta)
    out = cache.new_output()[0]
    worst = 0.0
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, layer, t)
        if resid_fn is not None:
            f["r"] = resid_fn(cfg, layer, t)
        if qkv_fn is not None:
            qkv_fn(cfg, t, f)
        q, k, v, r = (dev(f[x], cfg) for x in "qkvr")
        a = torch.from_numpy(f["a"]).to("cuda:0")
        cache.step(q, k, v, r, a, out, layer=0)
        do_attn = attn_frames is None or t in attn_frames
        orc.append(f["k"], f["v"])
        if do_attn:
            o_gpu = out.float().cpu().numpy().astype(np.float64)
            if q_rows is None:
                o_ref = orc.attend(f["q"])
            else:
                o_ref = oc.attention(f["q"][q_rows], orc.k, orc.v)
                o_gpu = o_gpu[q_rows]
            err = rel_err(o_gpu, o_ref)
            worst = max(worst, err)
            assert err < TOL[cfg.dtype], f"frame {t}: attention error {err:.3e}"
        orc.update(f["r"], f["a"])
        assert cache.size(0) == orc.n == min((t + 1) * cfg.M, cfg.B)
        if t % cache_every == 0 or t == cfg.T - 1:
            compare_cache(cache, orc, kv=(t % (4 * cache_every) == 0 or t == cfg.T - 1))
        if log:
            print(f"[{log}] frame {t} ok", flush=True)
    assert cache.status(0) == 0
    cache.close()
    return worst


def test_cfg0_tiny_f32_full_stream():
    worst = run_stream(synth.preset(0))
    print("cfg0 worst attention err/RMS:", worst)


def test_bf16_ragged_small():
    # 200 queries (1.6 query blocks), 900 slots at steady state (7 tiles + tail of 4), odd head count,
    # residual width that is not a power of two
    cfg = synth.preset(1, M=200, H=3, C=200, B=700, T=9, n_special=3)
    worst = run_stream(cfg)
    print("ragged worst attention err/RMS:", worst)


def _hard_values(kind):
    """Q/K/V regimes that stress the attention kernel's running reference and half-precision
    weights; every array is rounded to the run dtype like the generator's own."""
    def fn(cfg, t, f):
        j = (t * cfg.M + np.arange(cfg.M, dtype=np.float32))[:, None, None]      # global token index
        ones = np.ones((cfg.M, cfg.H, cfg.d), np.float32)
        if kind == "peaky":                     # logit std 16: nearly one-hot rows
            f["q"] = f["q"] * 4.0; f["k"] = f["k"] * 4.0
        elif kind == "rising":                  # the maximum grows by ~0.9 (log2) per slot: a rescale in every tile
            f["k"] = ones * (j / 100.0); f["q"] = ones * 1.0
        elif kind == "falling":                 # the first slot dominates, later weights underflow
            f["k"] = ones * (-j / 100.0); f["q"] = ones * 1.0
        elif kind == "constant":                # uniform weights over the whole cache
            f["k"] = ones * 0.5
        elif kind == "zero_q":
            f["q"] = np.zeros_like(f["q"])
        elif kind == "big_v":
            f["v"] = f["v"] * 300.0
        elif kind == "tiny_v":
            f["v"] = f["v"] * 1e-3
        elif kind == "outlier_key":             # one key per frame carries most of every row's mass
            f["q"] = np.abs(f["q"]); f["k"][7] = 3.0
        elif kind == "all_low":                 # every logit near -40 nats: far below the zero rows behind the
            f["q"] = ones * 1.0                 # cache's end, which must not pull the reference up (the softmax
            f["k"] = ones * -5.0 + f["k"] * 0.25   # is shift-invariant); the resident count is no multiple of 128
        for x in "qkv":
            f[x] = synth.quantise(np.ascontiguousarray(f[x], dtype=np.float32), cfg.dtype)
    return fn


@pytest.mark.parametrize("kind", ["peaky", "rising", "falling", "constant", "zero_q", "big_v", "tiny_v", "outlier_key",
                                  "all_low"])
def test_attention_hard_value_distributions(kind):
    # 6 frames of 200 tokens under a budget that keeps everything: 1200 slots = 9 tiles + a tail,
    # every frame's output compared
    cfg = synth.preset(1, M=200, H=2, C=64, B=2000, T=6, n_special=2)
    worst = run_stream(cfg, qkv_fn=_hard_values(kind))
    print(f"{kind}: worst attention err/RMS {worst:.3e}")


# (2100, 2500) has 17 query blocks: more than the merge pass's table of records holds, so the pass
# lists each item's records itself; the last two have an even number of heads and three or five
# query blocks, so workgroups pass from items whose two halves share one head's tiles to the mixed
# item of the odd last block and back, several pieces each
@pytest.mark.parametrize("M,B,H,C", [(1, 64, 1, 64), (37, 74, 2, 1024), (130, 1000, 5, 4096), (128, 256, 16, 8),
                                     (2100, 2500, 2, 64), (300, 6000, 4, 64), (520, 3000, 2, 128)])
def test_bf16_odd_shapes(M, B, H, C):
    cfg = synth.preset(1, M=M, H=H, C=C, B=B, T=max(6, 2 * B // M + 3) if M > 1 else 70, n_special=min(M - 1, 2))
    run_stream(cfg)


def test_f32_shapes_with_eviction_and_ties():
    cfg = synth.preset(3, M=70, H=2, C=96, B=300, T=14, n_special=2, dtype="f32")
    run_stream(cfg)


def test_ties_bf16_stream():
    cfg = synth.preset(3, M=300, H=2, C=1024, B=2000, T=30, n_special=5)
    run_stream(cfg, attn_frames={0, 7, 29})


def test_cfg4_shape_budget_sweep_and_full_cache_equality():
    for budget in (4096, 8192):
        cfg = synth.preset(4, B=budget, T=budget // 1041 + 4)
        run_stream(cfg, attn_frames={0, budget // 1041 - 1, budget // 1041, cfg.T - 1}, cache_every=2)
    # budget >= everything seen: equals uncompressed causal streaming attention
    cfg = synth.preset(4, B=8 * 1041, T=8)
    torch = _torch()
    cache = make_cache(cfg, L=1)
    out = cache.new_output()[0]
    ks, vs = [], []
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t)
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        ks.append(f["k"]); vs.append(f["v"])
        if t in (0, 3, 7):
            ref = oc.attention(f["q"], np.concatenate(ks), np.concatenate(vs))
            assert rel_err(out.float().cpu().numpy().astype(np.float64), ref) < TOL["bf16"]
    e = cache.export(0)
    assert np.array_equal(e["ids"], np.arange(cfg.T * cfg.M))
    assert np.array_equal(e["k"], stored_v(np.concatenate(ks), "bf16"))
    assert np.array_equal(e["v"], stored_v(np.concatenate(vs), "bf16"))
    cache.close()


@pytest.mark.parametrize("budget", [32768, 65536])
def test_cfg4_large_budgets_attention_full_size(budget):
    """The two largest budgets of the 518x392 sweep at full size (up to 66 577 resident keys, 521
    slot tiles): sampled query rows against the oracle while the cache still holds the whole stream
    (budget >= total: the result must equal uncompressed causal streaming attention, Eq. 2 over the
    concatenated frames, which the test builds itself from the frames it fed), on the frames around
    the first eviction, and 50 frames into eviction; kept ids, scores and flags on the way."""
    torch = _torch()
    cfg = synth.preset(4, B=budget)
    fill = budget // cfg.M                       # frames that fit entirely: 31 (32 271 tokens), 62 (64 542)
    T = fill + 52
    cache = make_cache(cfg, L=1)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    out = cache.new_output()[0]
    rows = np.unique(np.concatenate([np.random.default_rng(4).choice(cfg.M, size=40, replace=False), [0, 127, 128, 1040]]))
    under = {0, fill // 2, fill - 1}
    check = under | {fill, fill + 1, fill + 50}
    ks, vs = [], []
    worst = 0.0
    for t in range(T):
        f = synth.frame_inputs(cfg, 0, t)
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        orc.append(f["k"], f["v"])
        if t < fill:
            ks.append(f["k"]); vs.append(f["v"])
        if t in check:
            o_gpu = out.float().cpu().numpy().astype(np.float64)[rows]
            if t in under:                       # nothing has been evicted: the whole stream so far
                assert cache.size(0) == (t + 1) * cfg.M
                o_ref = oc.attention(f["q"][rows], np.concatenate(ks), np.concatenate(vs))
            else:
                o_ref = oc.attention(f["q"][rows], orc.k, orc.v)
            err = rel_err(o_gpu, o_ref)
            worst = max(worst, err)
            assert err < TOL["bf16"], f"B={budget} frame {t}: attention error {err:.3e}"
        orc.update(f["r"], f["a"])
        if t == fill - 1:
            e = cache.export(0)
            assert np.array_equal(e["ids"], np.arange(fill * cfg.M))
            assert np.array_equal(e["k"], stored_v(np.concatenate(ks), "bf16"))
            assert np.array_equal(e["v"], stored_v(np.concatenate(vs), "bf16"))
            ks, vs = [], []
        if t in check or t == T - 1:
            compare_cache(cache, orc, kv=(t == T - 1))
        if t % 10 == 0:
            print(f"[cfg4 B={budget}] frame {t} ok", flush=True)
    assert cache.status(0) == 0
    print(f"cfg4 B={budget}: worst sampled attention err/RMS {worst:.3e}")
    cache.close()


def test_cfg2_24_layers_kept_ids_deep_into_eviction():
    """The 24-layer workload, all layers per call, 100 frames past the first eviction: kept ids,
    slot layout, scores and flags of six layers after every evicting frame.  Three residual
    streams are spread over the layers (layer l gets stream l mod 3); the cache policy of the
    stored-score mode depends on residual rows and anchor bits only, so three oracles on a
    one-element K/V cover all layers and the device side reuses one frame's Q/K/V."""
    torch = _torch()
    cfg = synth.preset(2)
    L, kinds = cfg.L, 3
    T = cfg.B // cfg.M + 1 + 100
    cache = make_cache(cfg)
    orcs = [oc.OracleCache(cfg.M, 1, 1, cfg.B) for _ in range(kinds)]
    out = cache.new_output()
    layer_kind = (torch.arange(L) % kinds).cuda()
    f0 = [synth.frame_inputs(cfg, k, 0, want=("q", "k", "v")) for k in range(kinds)]
    q, k, v = (dev(np.stack([f[x] for f in f0]), cfg).index_select(0, layer_kind).contiguous() for x in "qkv")
    zk = np.zeros((cfg.M, 1, 1), np.float32)
    check_layers = (0, 1, 2, 9, 16, 23)
    for t in range(T):
        fs = [synth.frame_inputs(cfg, kk, t, want=("r", "a")) for kk in range(kinds)]
        r = dev(np.stack([f["r"] for f in fs]), cfg).index_select(0, layer_kind).contiguous()
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda().index_select(0, layer_kind).contiguous()
        cache.step(q, k, v, r, a, out)
        for kk in range(kinds):
            orcs[kk].append(zk, zk)
            orcs[kk].update(fs[kk]["r"], fs[kk]["a"])
        if (t + 1) * cfg.M > cfg.B or t % 6 == 0:
            for l in check_layers:
                o = orcs[l % kinds]
                n = cache.size(l)
                assert n == o.n
                ids = np.zeros(n, np.uint32); ss = np.zeros(n, np.float32); flags = np.zeros(n, np.uint8)
                B.ovggt_cache_export(cache.h, l, ids, None, None, ss, flags, cache.stream)
                assert np.array_equal(ids, o.gid), f"frame {t} layer {l}: kept ids / layout differ"
                assert np.array_equal(ss.view(np.uint32), o.ss.view(np.uint32)), f"frame {t} layer {l}: scores differ"
                assert np.array_equal(flags, o.flag), f"frame {t} layer {l}: flags differ"
        if t % 10 == 0:
            print(f"[cfg2 deep] frame {t} ok", flush=True)
    assert all(cache.status(l) == 0 for l in range(L))
    cache.close()


def test_values_beyond_the_half_range_saturate_and_set_status():
    """bf16 handles cache K and V as IEEE half: elements beyond +-65504 (bf16 reaches 3e38) are
    saturated, the status word reports it, export returns the saturated image, and attention
    runs on that image."""
    torch = _torch()
    cfg = synth.preset(1, M=130, H=2, C=64, B=600, T=3, n_special=2)
    cache = make_cache(cfg, L=1)
    out = cache.new_output()[0]
    ks, vs = [], []
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t)
        if t == 1:
            f["k"][3, 0, 5] = 7.0e4; f["k"][4, 1, 0] = -1.0e30; f["k"][5, 1, 63] = 65536.0
            f["v"][6, 0, 1] = 3.0e38; f["v"][7, 1, 2] = -65536.0; f["v"][8, 0, 0] = 65280.0   # the last one fits
            f["k"] = synth.quantise(f["k"], "bf16"); f["v"] = synth.quantise(f["v"], "bf16")
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        ks.append(f["k"]); vs.append(f["v"])
        st = cache.status(0)                       # reads and clears
        assert st == (B.OVGGT_STATUS_VRANGE if t == 1 else 0), (t, st)
        kc, vc = oc.cached_half(np.concatenate(ks)), oc.cached_half(np.concatenate(vs))
        ref = oc.attention(f["q"], kc, vc)
        assert rel_err(out.float().cpu().numpy().astype(np.float64), ref) < TOL["bf16"], t
    e = cache.export(0)
    kc, vc = oc.cached_half(np.concatenate(ks)), oc.cached_half(np.concatenate(vs))
    assert np.abs(kc).max() == 65504.0 and np.abs(vc).max() == 65504.0 and vc[130 + 8, 0, 0] == 65280.0
    assert np.array_equal(e["k"], synth.quantise(kc, "bf16"))
    assert np.array_equal(e["v"], synth.quantise(vc, "bf16"))
    cache.close()


def test_scaled_query_beyond_the_half_range_is_clamped():
    """A query element whose product with scale*log2(e) leaves the half range is clamped to
    +-65504, so the output stays finite and equals attention with the clamped query."""
    torch = _torch()
    cfg = synth.preset(1, M=130, H=2, C=64, B=600, T=2, n_special=2)
    cache = make_cache(cfg, L=1)
    out = cache.new_output()[0]
    c = (1.0 / 8.0) * 1.4426950408889634
    ks, vs = [], []
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t)
        f["k"] = synth.quantise(f["k"] * 2.0 ** -10, "bf16")       # keeps the clamped logits apart by a few units
        f["q"][5, 0, 3] = 1.0e6; f["q"][9, 1, 60] = -3.0e7
        f["q"] = synth.quantise(f["q"], "bf16")
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        ks.append(f["k"]); vs.append(f["v"])
        o = out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(o).all()
        q_eff = np.clip(f["q"].astype(np.float64), -65504.0 / c, 65504.0 / c)
        ref = oc.attention(q_eff, np.concatenate(ks), np.concatenate(vs))
        assert rel_err(o, ref) < TOL["bf16"], t
    assert cache.status(0) == 0
    cache.close()


def test_cfg1_shapes_warmup_boundary():
    """Full-size layer (M=1374, 16x64, B=16384): frames around the first eviction."""
    cfg = synth.preset(1, T=14)
    rows = np.random.default_rng(0).choice(cfg.M, size=96, replace=False)
    rows = np.unique(np.concatenate([rows, [0, 127, 128, 1279, 1280, 1373]]))
    worst = run_stream(cfg, attn_frames={0, 1, 10, 11, 12, 13}, q_rows=rows, cache_every=1, log="cfg1")
    print("cfg1 worst sampled attention err/RMS:", worst)


def test_cfg3_full_budget_sampled():
    """The long-stream workload's layer (B=32768, heavy-tailed scores with exact duplicates): the
    frames around the first eviction at full size, attention checked on sampled query rows."""
    cfg = synth.preset(3, T=27)
    rows = np.random.default_rng(1).choice(cfg.M, size=64, replace=False)
    rows = np.unique(np.concatenate([rows, [0, 1373]]))
    worst = run_stream(cfg, attn_frames={23, 24, 26}, q_rows=rows, cache_every=4, log="cfg3")
    print("cfg3 worst sampled attention err/RMS:", worst)


@pytest.mark.parametrize("preset,budget,evicting_frames", [(1, 16384, 300), (3, 32768, 500), (4, 65536, 250)])
def test_full_size_streams_kept_ids_deep_into_eviction(preset, budget, evicting_frames):
    """The two largest caches of the workload list at full size, well past the first eviction:
    kept ids, slot layout, scores and flags bit-exact after every frame.  The cache policy of the
    stored-score mode depends on residual rows and anchor bits only, so the oracle runs on a
    one-element K/V (its attention is not used here) and the device side reuses one frame's
    Q/K/V; the other full-size tests cover attention and the K/V moves."""
    torch = _torch()
    cfg = synth.preset(preset, B=budget)
    T = budget // cfg.M + 1 + evicting_frames
    cache = make_cache(cfg, L=1)
    orc = oc.OracleCache(cfg.M, 1, 1, cfg.B)
    out = cache.new_output()[0]
    f0 = synth.frame_inputs(cfg, 0, 0, want=("q", "k", "v"))
    q, k, v = (dev(f0[x], cfg) for x in "qkv")
    zk = np.zeros((cfg.M, 1, 1), np.float32)
    for t in range(T):
        f = synth.frame_inputs(cfg, 0, t, want=("r", "a"))
        cache.step(q, k, v, dev(f["r"], cfg), torch.from_numpy(f["a"]).to("cuda:0"), out, layer=0)
        orc.append(zk, zk)
        orc.update(f["r"], f["a"])
        n = cache.size(0)
        assert n == orc.n == min((t + 1) * cfg.M, cfg.B)
        if t * cfg.M >= cfg.B - cfg.M or t % 8 == 0:           # every evicting frame, some of the warm-up
            ids = np.zeros(n, np.uint32); ss = np.zeros(n, np.float32); flags = np.zeros(n, np.uint8)
            B.ovggt_cache_export(cache.h, 0, ids, None, None, ss, flags, cache.stream)
            assert np.array_equal(ids, orc.gid), f"frame {t}: kept ids / layout differ"
            assert np.array_equal(ss.view(np.uint32), orc.ss.view(np.uint32)), f"frame {t}: scores differ"
            assert np.array_equal(flags, orc.flag), f"frame {t}: flags differ"
        if t % 10 == 0:
            print(f"[full-size preset {preset}] frame {t} ok", flush=True)
    assert cache.status(0) == 0
    cache.close()


def test_cfg2_full_size_24_layers_batched_sampled():
    """The 24-layer workload in the launch shape the benchmark times (all layers per call, 192 head
    pairs dealt out to the XCDs round by round).  Three distinct input streams are spread over the
    layers (layer l gets stream l mod 3), so three oracles cover all layers; kept ids, scores and
    flags of six layers and sampled attention rows of six layers are checked around the first
    eviction."""
    torch = _torch()
    cfg = synth.preset(2, T=13)
    L, kinds = cfg.L, 3
    cache = make_cache(cfg)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B) for _ in range(kinds)]
    out = cache.new_output()
    rows = np.unique(np.concatenate([np.random.default_rng(2).choice(cfg.M, size=24, replace=False), [0, 1373]]))
    rows_t = torch.from_numpy(rows).cuda()
    check_layers = (0, 1, 2, 10, 17, 23)
    layer_kind = (torch.arange(L) % kinds).cuda()
    worst = 0.0
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, k, t) for k in range(kinds)]
        # three uploads per tensor, spread over the 24 layers on the device
        pack = lambda key: dev(np.stack([f[key] for f in fs]), cfg).index_select(0, layer_kind).contiguous()
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda().index_select(0, layer_kind).contiguous()
        cache.step(pack("q"), pack("k"), pack("v"), pack("r"), a, out)
        for k in range(kinds):
            orcs[k].append(fs[k]["k"], fs[k]["v"])
        if t in (0, 10, 11, 12):
            for l in check_layers:
                o_gpu = out[l].index_select(0, rows_t).float().cpu().numpy().astype(np.float64)
                o_ref = oc.attention(fs[l % kinds]["q"][rows], orcs[l % kinds].k, orcs[l % kinds].v)
                err = rel_err(o_gpu, o_ref)
                worst = max(worst, err)
                assert err < TOL["bf16"], (t, l, err)
        for k in range(kinds):
            orcs[k].update(fs[k]["r"], fs[k]["a"])
        if t >= 10:
            for l in check_layers:
                compare_cache(cache, orcs[l % kinds], layer=l, kv=(t == cfg.T - 1 and l in (0, 23)))
        print(f"[cfg2] frame {t} ok", flush=True)
    assert all(cache.status(l) == 0 for l in range(L))
    assert all(cache.size(l) == cfg.B for l in range(L))
    print("cfg2 worst sampled attention err/RMS:", worst)
    cache.close()


def test_worst_case_compaction_rising_scores():
    cfg = synth.preset(1, M=300, H=4, B=1500, T=12, n_special=5)
    torch = _torch()
    cache = make_cache(cfg, L=1)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    out = cache.new_output()[0]
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t, want=("q", "k", "v", "a"))
        r = synth.rising_resid(cfg, 0, t)
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(r, cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        orc.step(f["q"], f["k"], f["v"], r, f["a"], attend=False)
        dst, src = cache.last_moves(0)
        if t >= 5:
            assert len(dst) == cfg.M              # every new token survives: M entries move per frame
        compare_cache(cache, orc)
    cache.close()


@pytest.mark.parametrize("shape", [
    dict(M=150, H=2, C=256, B=400, T=7, L=3),          # 3 head pairs: one chunk per workgroup
    dict(M=300, H=8, C=64, B=5000, T=5, L=4),          # 16 head pairs: two rounds per XCD, tile segments
    dict(M=130, H=16, C=64, B=300, T=4, L=3),          # 24 head pairs: three rounds, short caches
    dict(M=600, H=16, C=64, B=1000, T=4, L=8),         # 64 head pairs x 5 query blocks: whole items per workgroup for a
                                                       # round, the 8 left over per XCD cut into 4-tile chunks (5 pieces each)
])
def test_batched_layers_match_per_layer_oracle(shape):
    cfg = synth.preset(2, n_special=5, **shape)
    torch = _torch()
    cache = make_cache(cfg)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B) for _ in range(cfg.L)]
    out = cache.new_output()
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, l, t) for l in range(cfg.L)]
        stack = lambda key: dev(np.stack([f[key] for f in fs]), cfg)
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda()
        cache.step(stack("q"), stack("k"), stack("v"), stack("r"), a, out)      # layer = all
        o = out.float().cpu().numpy().astype(np.float64)
        for l in range(cfg.L):
            ref = orcs[l].step(fs[l]["q"], fs[l]["k"], fs[l]["v"], fs[l]["r"], fs[l]["a"])
            assert rel_err(o[l], ref) < TOL["bf16"], (t, l)
            compare_cache(cache, orcs[l], layer=l)
    cache.close()


def test_compaction_carried_by_the_next_append_equals_the_stand_alone_kernel():
    """The same stream through three handles: A is exported after every frame (the export applies
    the outstanding compaction with the stand-alone kernel), B is never touched between frames (every
    compaction rides along with the next frame's append), C is flushed explicitly on odd frames.
    Outputs of every frame and the final caches must be identical, and equal to the oracle's."""
    torch = _torch()
    cfg = synth.preset(1, M=300, H=4, B=1500, T=16, n_special=5)
    caches = [make_cache(cfg, L=1) for _ in range(3)]
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    outs = [c.new_output()[0] for c in caches]
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t)
        if t >= 6:
            f["r"] = synth.rising_resid(cfg, 0, t)            # many movers per frame
        q, k, v, r = (dev(f[x], cfg) for x in "qkvr")
        a = torch.from_numpy(f["a"]).to("cuda:0")
        for c, o in zip(caches, outs):
            c.step(q, k, v, r, a, o, layer=0)
        orc.step(f["q"], f["k"], f["v"], f["r"], f["a"])
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), f"frame {t}: outputs differ"
        compare_cache(caches[0], orc)
        if t % 2 == 1:
            caches[2].flush(0)
    for c in caches:
        compare_cache(c, orc)
        assert c.status(0) == 0
        c.close()


def test_compaction_outstanding_in_some_layers_only():
    """Three layers stepped together; between frames one layer is flushed, another one is given a
    late anchor (which applies its compaction first), the third keeps its compaction outstanding:
    the next batched call has to cope with the mix."""
    torch = _torch()
    cfg = synth.preset(1, M=200, H=2, C=256, B=900, T=12, n_special=3, L=3)
    cache = make_cache(cfg)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B) for _ in range(cfg.L)]
    out = cache.new_output()
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, l, t) for l in range(cfg.L)]
        pack = lambda key: dev(np.stack([f[key] for f in fs]), cfg)
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda()
        cache.step(pack("q"), pack("k"), pack("v"), pack("r"), a, out)
        for l in range(cfg.L):
            orcs[l].step(fs[l]["q"], fs[l]["k"], fs[l]["v"], fs[l]["r"], fs[l]["a"])
        if t >= 5:
            cache.flush(0)
            if t % 3 == 0:                                    # protect what is left of frame t-2 in layer 1
                cache.set_protect(t - 2, None, True, layer=1)
                orcs[1].set_protect(t - 2, None, True)
    for l in range(cfg.L):
        compare_cache(cache, orcs[l], layer=l)
        assert cache.status(l) == 0
    cache.close()


def test_per_layer_calls_are_independent():
    cfg = synth.preset(2, M=64, H=1, C=64, B=128, T=5, L=2, n_special=1)
    torch = _torch()
    cache = make_cache(cfg)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B) for _ in range(2)]
    out = cache.new_output()[0]
    for t in range(cfg.T):                        # layer 1 runs one frame behind layer 0
        for l, tt in ((0, t), (1, t - 1)):
            if tt < 0:
                continue
            f = synth.frame_inputs(cfg, l, tt)
            cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                       torch.from_numpy(f["a"]).cuda(), out, layer=l)
            ref = orcs[l].step(f["q"], f["k"], f["v"], f["r"], f["a"])
            assert rel_err(out.float().cpu().numpy().astype(np.float64), ref) < TOL["bf16"]
            compare_cache(cache, orcs[l], layer=l)
    with pytest.raises(B.OvggtError) as e:        # layers out of step: a batched call is refused
        cache.global_attn(out, out, out, out)
    assert e.value.code == B.OVGGT_ERR_STATE
    cache.close()


def test_call_order_and_argument_errors():
    cfg = synth.preset(0)
    torch = _torch()
    cache = make_cache(cfg)
    f = synth.frame_inputs(cfg, 0, 0)
    q, k, v, r = (dev(f[x], cfg) for x in "qkvr")
    out = cache.new_output()[0]
    for call in (lambda: cache.score_select(r, None, 0), lambda: cache.compact(0)):
        with pytest.raises(B.OvggtError) as e:
            call()
        assert e.value.code == B.OVGGT_ERR_STATE
    with pytest.raises(B.OvggtError) as e:
        cache.global_attn(q, k, v, out, layer=5)
    assert e.value.code == B.OVGGT_ERR_ARG
    with pytest.raises(B.OvggtError) as e:
        B.ovggt_global_attn(cache.h, 0, q.data_ptr() + 4, k, v, out, cache.stream)
    assert e.value.code == B.OVGGT_ERR_ARG
    assert cache.size(0) == 0
    cache.global_attn(q, k, v, out, 0)
    for call in (lambda: cache.global_attn(q, k, v, out, 0), lambda: cache.compact(0)):
        with pytest.raises(B.OvggtError) as e:
            call()
        assert e.value.code == B.OVGGT_ERR_STATE
    assert cache.size(0) == cfg.M
    cache.score_select(r, None, 0)
    with pytest.raises(B.OvggtError):
        cache.score_select(r, None, 0)
    cache.compact(0)
    assert cache.size(0) == cfg.M and cache.frames(0) == 1
    cache.close()


def test_protected_set_larger_than_budget_sets_status():
    cfg = synth.preset(0, B=100, T=3)
    torch = _torch()
    cache = make_cache(cfg)
    out = cache.new_output()[0]
    ones = torch.ones(cfg.M, dtype=torch.uint8, device="cuda:0")
    for t in range(2):                               # 130 protected tokens, budget 100
        f = synth.frame_inputs(cfg, 0, t)
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg), ones, out, layer=0)
    assert cache.status(0) & B.OVGGT_STATUS_BUDGET
    assert cache.status(0) == 0                      # reading clears it
    assert cache.size(0) == cfg.B
    cache.close()


def test_import_export_and_crafted_scores():
    """Selection on hand-made cache contents: NaN ranks lowest, ties go to the
    older id, k = 0 evicts every evictable entry."""
    cfg = synth.preset(0, M=8, B=16, H=1, C=64, T=1, dtype="f32", n_special=1)
    rng = np.random.default_rng(3)
    cache = make_cache(cfg)
    n = 16
    ids = rng.permutation(80)[:n].astype(np.uint32)           # 10 frames already seen
    ss = rng.choice(np.array([0.0, 1.0, 1.0, 2.0, 5.0], np.float32), size=n)
    ss[3] = np.nan
    flags = (rng.random(n) < 0.25).astype(np.uint8)
    k = rng.standard_normal((n, 1, 64)).astype(np.float32); v = rng.standard_normal((n, 1, 64)).astype(np.float32)
    cache.import_(0, 10, ids, k, v, ss, flags)
    e = cache.export(0)
    assert np.array_equal(e["ids"], ids) and np.array_equal(e["k"], k) and np.array_equal(e["flags"], flags)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    orc.k, orc.v, orc.gid, orc.ss, orc.flag, orc.t = k.copy(), v.copy(), ids.copy(), ss.copy(), flags.copy(), 10
    torch = _torch()
    f = synth.frame_inputs(cfg, 0, 10)
    f["r"][2] = f["r"][5]                                      # an exact tie among the new tokens
    out = cache.new_output()[0]
    cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
               torch.from_numpy(f["a"]).cuda(), out, layer=0)
    ref = orc.step(f["q"], f["k"], f["v"], f["r"], f["a"])
    assert rel_err(out.cpu().numpy().astype(np.float64), ref) < TOL["f32"]
    e = cache.export(0)
    assert np.array_equal(e["ids"], orc.gid)
    assert np.array_equal(np.isnan(e["ss"]), np.isnan(orc.ss))
    assert cache.status(0) & B.OVGGT_STATUS_NONFINITE
    cache.close()


@pytest.mark.parametrize("regime,M,Bq", [(r, 256, 12000) for r in (
    "spread", "few_ties", "many_ties", "one_bin", "all_equal", "whole_bin", "two_levels_equal", "protected_low")] + [
    ("spread", 1041, 65536), ("many_ties", 1041, 65536), ("one_bin", 1041, 65536), ("protected_low", 1374, 32768)])
def test_selection_threshold_regimes(regime, M, Bq):
    """Hand-made score populations around the eviction threshold, one per branch of the
    selection: a threshold among distinct keys, among a few or among hundreds of equal scores
    (ids decide), every key within one leading-bits bin, all scores equal, a threshold on a bin
    boundary, keys that agree in their 22 leading bits, and low scores that are protected; also
    at the cache sizes of the largest workloads."""
    H, d, C = 1, 64, 64
    cfg = synth.preset(0, M=M, B=Bq, H=H, C=C, T=1, dtype="f32", n_special=1)
    rng = np.random.default_rng(11)
    n = Bq
    frames_seen = (n + M - 1) // M + 3
    ids = rng.permutation(frames_seen * M)[:n].astype(np.uint32)
    flags = np.zeros(n, np.uint8)
    spread = np.exp(rng.standard_normal(n)).astype(np.float32) + np.float32(4.0)      # all above 4
    ss = spread.copy()
    low = rng.permutation(n)                                                          # slots that get the low keys
    ramp = lambda m: (1.0 + np.arange(m) / 4096.0).astype(np.float32)          # m distinct keys in [1, 1.5)
    if regime == "few_ties":          # M - 20 distinct low keys, then 40 equal ones: 20 of them go
        ss[low[:M - 20]] = ramp(M - 20)
        ss[low[M - 20:M + 20]] = np.float32(2.5)
    elif regime == "many_ties":       # 300 equal keys straddle the threshold
        ss[low[:M - 156]] = ramp(M - 156)
        ss[low[M - 156:M + 144]] = np.float32(2.5)
    elif regime == "one_bin":         # every cached key shares sign, exponent and three mantissa bits
        ss = (1.0 + rng.permutation(n) * 2.0 ** -20).astype(np.float32)
    elif regime == "all_equal":
        ss[:] = np.float32(3.0)
    elif regime == "whole_bin":       # exactly M keys in [1.5, 1.625), the rest from 4.0 up
        ss[low[:M]] = (1.5 + rng.random(M) * 0.12).astype(np.float32)
    elif regime == "two_levels_equal":  # 90 keys that differ only below bit 9 of the score word
        ss[low[:M - 56]] = ramp(M - 56)
        ss[low[M - 56:M + 34]] = (np.float32(2.5).view(np.uint32) + rng.permutation(90).astype(np.uint32)).view(np.float32)
    elif regime == "protected_low":   # 300 of the lowest keys are protected: they stay, others go
        ss[low[:M + 444]] = ramp(M + 444)
        flags[low[:300]] = 1
    k = rng.standard_normal((n, H, d)).astype(np.float32); v = rng.standard_normal((n, H, d)).astype(np.float32)
    cache = make_cache(cfg)
    cache.import_(0, frames_seen, ids, k, v, ss, flags)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    orc.k, orc.v, orc.gid, orc.ss, orc.flag, orc.t = k.copy(), v.copy(), ids.copy(), ss.copy(), flags.copy(), frames_seen
    torch = _torch()
    f = synth.frame_inputs(cfg, 0, frames_seen)
    r = np.zeros((M, C), np.float32)
    r[:, 0] = np.float32(100.0)                               # new tokens: ss = 10 000, all stay ...
    if regime == "all_equal":                                 # ... unless they tie with the cache: ss = 3 exactly
        r[:, 0] = np.float32(1.0); r[:, 1] = np.float32(1.0); r[:, 2] = np.float32(1.0)
    if regime == "spread":
        r[:, 0] = np.exp(rng.standard_normal(M)).astype(np.float32) + np.float32(2.0)
    f["r"] = r
    a = np.zeros(M, np.uint8)
    out = cache.new_output()[0]
    cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(r, cfg), torch.from_numpy(a).cuda(), out, layer=0)
    ref = orc.step(f["q"], f["k"], f["v"], r, a)
    assert rel_err(out.cpu().numpy().astype(np.float64), ref) < TOL["f32"]
    compare_cache(cache, orc)
    assert cache.status(0) == 0
    # a second frame on top of the compacted cache (layout and scores carry over)
    f2 = synth.frame_inputs(cfg, 0, frames_seen + 1)
    r2 = r.copy(); r2[:, 0] = (r[:, 0] * np.float32(0.5)) if regime == "spread" else r[:, 0]
    cache.step(dev(f2["q"], cfg), dev(f2["k"], cfg), dev(f2["v"], cfg), dev(r2, cfg), torch.from_numpy(a).cuda(), out, layer=0)
    orc.step(f2["q"], f2["k"], f2["v"], r2, a)
    compare_cache(cache, orc)
    cache.close()


def _random_population_case(seed, M=None, Bq=None):
    """One seeded cache population (frame size, budget, score distribution, ties, protected share
    all drawn at random), three frames of selection on top of it; True if ids, layout, scores and
    flags equal the oracle's after every frame (odd seeds) or after the last one (even seeds)."""
    torch = _torch()
    rng = np.random.default_rng(seed)
    M_ = int(rng.choice([1, 3, 16, 17, 64, 100, 256, 700, 1041, 1374, 2100]))
    B_ = max(M_, int(rng.choice([M_, M_ + 1, 2 * M_ + 5, 1000, 4096, 9000, 20000, 40000, 70000])))
    M, Bq = (M_, B_) if M is None else (M, Bq)
    H, d, C = 1, 64, 64
    n = Bq
    frames_seen = (n + M - 1) // M + 3
    ids = rng.permutation(frames_seen * M)[:n].astype(np.uint32)
    kind = rng.integers(0, 6)
    if kind == 0:       # log-normal, narrow to wide
        ss = np.exp(rng.standard_normal(n) * rng.choice([0.1, 1, 3])).astype(np.float32)
    elif kind == 1:     # a few dozen distinct values: ties everywhere
        ss = rng.choice(np.exp(rng.standard_normal(int(rng.integers(1, 40)))).astype(np.float32), size=n)
    elif kind == 2:     # one leading-bits bin, few to many distinct low-order patterns
        ss = (1.0 + rng.integers(0, int(rng.choice([4, 300, 1 << 20])), size=n) * 2.0 ** -22).astype(np.float32)
    elif kind == 3:
        ss = np.full(n, 2.0, np.float32)
    elif kind == 4:     # heavy tail with 5 % exact duplicates
        ss = (rng.pareto(1.5, n) + 1).astype(np.float32); ss[rng.random(n) < 0.05] = ss[0]
    else:               # any binade, subnormals included
        ss = np.abs(rng.standard_normal(n)).astype(np.float32) * np.float32(10.0 ** rng.integers(-30, 30))
    if rng.random() < 0.3:
        ss[rng.integers(0, n, size=min(n, 3))] = np.float32(0.0)
    if rng.random() < 0.2:
        ss[rng.integers(0, n, size=min(n, 3))] = np.float32(np.inf)
    flags = (rng.random(n) < rng.choice([0.0, 0.01, 0.3, 0.9])).astype(np.uint8)
    k = np.zeros((n, H, d), np.float32); v = np.zeros((n, H, d), np.float32)
    cache = B.Cache(1, H, d, M, C, Bq, "f32")
    cache.import_(0, frames_seen, ids, k, v, ss, flags)
    orc = oc.OracleCache(M, H, d, Bq)
    orc.k, orc.v, orc.gid, orc.ss, orc.flag, orc.t = k.copy(), v.copy(), ids.copy(), ss.copy(), flags.copy(), frames_seen
    out = cache.new_output()[0]
    z = torch.zeros((M, H, d), dtype=torch.float32, device="cuda:0")
    zk = np.zeros((M, H, d), np.float32)
    ok = True
    for step in range(3):
        mode = rng.integers(0, 4)
        r = np.zeros((M, C), np.float32)
        if mode == 0:
            r[:, 0] = np.exp(rng.standard_normal(M)).astype(np.float32)
        elif mode == 1:
            r[:, 0] = np.float32(1e3)
        elif mode == 2:     # ss = 2 or 3 exactly: ties with the all-equal populations
            r[:, 0] = np.sqrt(np.float32(2.0)); r[:, 1] = rng.choice([0.0, 1.0], size=M).astype(np.float32)
        else:
            r[:, :] = rng.standard_normal((M, C)).astype(np.float32) * 0.1
        a = (rng.random(M) < rng.choice([0.0, 0.05])).astype(np.uint8)
        if int(orc.flag.sum() + a.sum()) > Bq:
            a[:] = 0
        cache.step(z, z, z, B.to_device(r, "f32"), torch.from_numpy(a).cuda(), out, layer=0)
        orc.append(zk, zk); orc.update(r, a)
        if seed % 2 == 0 and step < 2:
            continue            # even seeds: no export between frames, so the appends carry the compactions
        nn = cache.size(0)
        gi = np.zeros(nn, np.uint32); gs = np.zeros(nn, np.float32); gf = np.zeros(nn, np.uint8)
        B.ovggt_cache_export(cache.h, 0, gi, None, None, gs, gf, cache.stream)
        ok = ok and nn == orc.n and np.array_equal(gi, orc.gid) and \
            np.array_equal(gs.view(np.uint32), orc.ss.view(np.uint32)) and np.array_equal(gf, orc.flag)
    cache.close()
    return ok


def test_selection_at_the_largest_cache_the_library_accepts():
    """B + M = 131 072 slots (the limit the configuration check enforces), every score distribution."""
    bad = [seed for seed in range(12) if not _random_population_case(seed, M=2048, Bq=131072 - 2048)]
    assert not bad, f"selection differs from the oracle for seeds {bad}"
    cfg = B.make_config(1, 1, 64, 2048, 64, 131072 - 2047, "f32")          # one slot more: rejected
    with pytest.raises(B.OvggtError):
        B.ovggt_cache_query_bytes(cfg)


def test_selection_random_populations():
    """200 seeded random populations (sizes 1 .. 72 100 slots, six score distributions, zeros,
    infinities, up to 90 % protected), three selections each.  The same generator was run once over
    6 000 seeds when the selection was rewritten: no difference."""
    bad = [seed for seed in range(200) if not _random_population_case(seed)]
    assert not bad, f"selection differs from the oracle for seeds {bad}"


@pytest.mark.parametrize("dtype,ph,pw,ns,H,C,B_,alpha", [
    ("bf16", 9, 13, 5, 2, 256, 500, 0.5),       # budget not a multiple of the frame, eviction from frame 4 on
    ("f32", 6, 7, 2, 2, 96, 130, 0.25),
    ("bf16", 1, 40, 0, 1, 64, 100, 1.0),        # one-row map, no aux tokens, pure convolution
    ("bf16", 37, 37, 5, 4, 1024, 4200, 0.5),    # the paper's patch grid (518 px / 14) at a small budget
])
def test_activation_smoothing_matches_oracle(dtype, ph, pw, ns, H, C, B_, alpha):
    M = ns + ph * pw
    cfg = synth.preset(1, M=M, H=H, C=C, B=B_, T=2 * (B_ // M) + 5, n_special=ns, dtype=dtype)
    sm = (alpha, ph, pw, ns, synth.gaussian_kernel3(1.0))
    run_stream(cfg, smooth=sm, attn_frames={0, cfg.T - 1})


def test_activation_smoothing_batched_layers_and_bad_configs():
    torch = _torch()
    ph, pw, ns = 8, 10, 3
    cfg = synth.preset(1, M=ns + ph * pw, H=2, C=128, B=300, T=8, n_special=ns, L=3)
    sm = (0.5, ph, pw, ns, synth.gaussian_kernel3(0.8))
    cache = make_cache(cfg, smooth=sm)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, smooth=sm) for _ in range(cfg.L)]
    out = cache.new_output()
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, l, t) for l in range(cfg.L)]
        q, k, v, r = (dev(np.stack([f[x] for f in fs]), cfg) for x in "qkvr")
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda()
        cache.step(q, k, v, r, a, out)                                         # layer = all
        for l, (f, o) in enumerate(zip(fs, orcs)):
            o.append(f["k"], f["v"]); o.update(f["r"], f["a"])
            compare_cache(cache, o, layer=l, kv=(t == cfg.T - 1))
    cache.close()
    g = synth.gaussian_kernel3(1.0)
    for bad in [(0.5, 8, 10, 2, g), (1.5, 8, 10, 3, g), (-0.1, 8, 10, 3, g), (0.5, 0, 83, 0, g), (float("nan"), 8, 10, 3, g),
                (0.5, 8, 10, 3, np.full((3, 3), np.nan, np.float32))]:
        with pytest.raises(B.OvggtError):
            make_cache(cfg, smooth=bad)


@pytest.mark.parametrize("M,H,C,B_,beta,ns", [
    (50, 2, 64, 170, 0.5, 2),          # two elements per lane, budget not a multiple of the frame
    (33, 1, 64, 100, 0.3, 1),          # one head: one element per lane
    (40, 3, 128, 200, 0.5, 2),         # 192-wide keys: the tree's zero padding is live
    (70, 5, 64, 300, 0.7, 3),          # 320-wide keys padded to 512
    (200, 16, 256, 900, 0.5, 5),       # the paper's 16 x 64 keys, several centroid chunks
    (64, 16, 64, 128, 0.0, 0),         # beta = 0: new tokens all rank 0, no anchors at all
    (64, 4, 64, 128, 1.0, 4),          # beta = 1: history all ranks 0
])
def test_hybrid_scoring_matches_oracle(M, H, C, B_, beta, ns):
    cfg = synth.preset(1, M=M, H=H, C=C, B=B_, T=2 * (B_ // M) + 6, n_special=ns)
    run_stream(cfg, hybrid_beta=beta, attn_frames={0, cfg.T - 1})


def test_hybrid_scoring_with_smoothing_and_batched_layers():
    torch = _torch()
    ph, pw, ns = 6, 9, 2
    cfg = synth.preset(1, M=ns + ph * pw, H=4, C=128, B=210, T=9, n_special=ns, L=3)
    sm = (0.5, ph, pw, ns, synth.gaussian_kernel3(1.0))
    cache = make_cache(cfg, smooth=sm, hybrid_beta=0.5)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, smooth=sm, hybrid_beta=0.5) for _ in range(cfg.L)]
    out = cache.new_output()
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, l, t) for l in range(cfg.L)]
        q, k, v, r = (dev(np.stack([f[x] for f in fs]), cfg) for x in "qkvr")
        a = torch.from_numpy(np.stack([f["a"] for f in fs])).cuda()
        cache.step(q, k, v, r, a, out)                                         # layer = all
        for l, (f, o) in enumerate(zip(fs, orcs)):
            o.append(f["k"], f["v"]); o.update(f["r"], f["a"])
            compare_cache(cache, o, layer=l, kv=(t == cfg.T - 1))
    assert all(cache.status(l) == 0 for l in range(cfg.L))
    cache.close()


def test_hybrid_scoring_resumes_from_an_imported_cache():
    """The running centroid sum is rebuilt on import: a stream continued from an exported
    mid-stream state matches the oracle continued from the same state."""
    torch = _torch()
    cfg = synth.preset(1, M=60, H=3, C=64, B=200, T=12, n_special=2)
    a = make_cache(cfg, L=1, hybrid_beta=0.4)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, hybrid_beta=0.4)
    out = a.new_output()[0]

    def feed(cache, t):
        f = synth.frame_inputs(cfg, 0, t)
        cache.step(dev(f["q"], cfg), dev(f["k"], cfg), dev(f["v"], cfg), dev(f["r"], cfg),
                   torch.from_numpy(f["a"]).cuda(), out, layer=0)
        return f

    for t in range(6):
        f = feed(a, t)
        orc.append(f["k"], f["v"]); orc.update(f["r"], f["a"])
    compare_cache(a, orc)
    e = a.export(0)
    # the exported bf16 values are the state both sides continue from (a half below 2^-14 need not
    # survive the trip through bf16, so the oracle takes the exported keys, not its own)
    orc.k, orc.v = e["k"].copy(), e["v"].copy()
    bits = lambda x: (np.ascontiguousarray(x).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    b = make_cache(cfg, L=1, hybrid_beta=0.4)
    b.import_(0, 6, e["ids"], bits(e["k"]), bits(e["v"]), e["ss"], e["flags"])
    for t in range(6, cfg.T):
        f = feed(b, t)
        orc.append(f["k"], f["v"]); orc.update(f["r"], f["a"])
        compare_cache(b, orc)
    assert b.status(0) == 0
    a.close(); b.close()


def test_hybrid_scoring_full_width_stream():
    # the benchmark layer's shape at a reduced budget: 1374 tokens of 16 x 64 keys per frame
    cfg = synth.preset(1, B=4096, T=8)
    run_stream(cfg, hybrid_beta=0.5, attn_frames={cfg.T - 1}, cache_every=2)


def _dap_stream(cfg, policy_args, hybrid_beta=None, layers=1, camera=None):
    """A stream whose anchors are registered and demoted by the library's host policy; the oracle
    follows its own policy object, and both caches are compared after every frame.  `camera`: also
    run a one-token-per-frame cache (the camera head's) whose tokens are protected and released in
    step with the anchors."""
    torch = _torch()
    cache = make_cache(cfg, L=layers, hybrid_beta=hybrid_beta)
    orcs = [oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, hybrid_beta=hybrid_beta) for _ in range(layers)]
    dap = B.ovggt_dap_create(*policy_args)
    pol = oc.DapPolicy(*policy_args)
    out = cache.new_output()
    mask_host = np.zeros(cfg.M, np.uint8)
    if camera is not None:
        ccfg = camera
        cam = make_cache(ccfg, L=1, hybrid_beta=hybrid_beta)
        cam_orc = oc.OracleCache(1, ccfg.H, ccfg.d, ccfg.B, hybrid_beta=hybrid_beta)
        cam_out = cam.new_output()[0]
    events = 0
    for t in range(cfg.T):
        fs = [synth.frame_inputs(cfg, l, t) for l in range(layers)]
        a0 = np.zeros(cfg.M, np.uint8)
        if t == 0:
            a0[:] = 1                                            # the global initial anchor
        q, k, v, r = (dev(np.stack([f[x] for f in fs]), cfg) for x in "qkvr")
        a = torch.from_numpy(np.stack([a0] * layers)).cuda()
        cache.step(q, k, v, r, a, out)
        for f, o in zip(fs, orcs):
            o.append(f["k"], f["v"]); o.update(f["r"], a0)
        if camera is not None:
            cf = synth.frame_inputs(ccfg, 0, t)
            ca = np.array([1 if t == 0 else 0], np.uint8)
            cam.step(dev(cf["q"], ccfg), dev(cf["k"], ccfg), dev(cf["v"], ccfg), dev(cf["r"], ccfg),
                     torch.from_numpy(ca).cuda(), cam_out, layer=0)
            cam_orc.append(cf["k"], cf["v"]); cam_orc.update(cf["r"], ca)
        rho, conf = synth.coverage_and_confidence(cfg, t)
        reg, dem = B.ovggt_dap_step(dap, t, rho, conf, mask_host)
        m_ref, d_ref = pol.step(t, rho, conf)
        assert (reg == t) == (m_ref is not None) and dem == (-1 if d_ref is None else d_ref)
        if dem >= 0:
            cache.set_protect(dem, None, False)
            for o in orcs:
                o.set_protect(d_ref, None, False)
            if camera is not None:
                cam.set_protect(dem, None, False, layer=0); cam_orc.set_protect(d_ref, None, False)
        if reg >= 0:
            events += 1
            cache.set_protect(reg, torch.from_numpy(mask_host).cuda(), True)
            for o in orcs:
                o.set_protect(t, m_ref, True)
            if camera is not None:
                cam.set_protect(reg, None, True, layer=0); cam_orc.set_protect(t, None, True)
        for l, o in enumerate(orcs):
            compare_cache(cache, o, layer=l, kv=(t == cfg.T - 1))
        if camera is not None:
            compare_cache(cam, cam_orc, kv=(t == cfg.T - 1))
    assert events >= 3 and len(pol.active) == policy_args[0]
    assert all(cache.status(l) == 0 for l in range(layers))
    # Eq. 9 on the device's own flags
    per = int(np.ceil(policy_args[3] * policy_args[5]))
    assert int(cache.export(0)["flags"].sum()) <= cfg.M + policy_args[0] * per
    B.ovggt_dap_destroy(dap)
    cache.close()
    if camera is not None:
        cam.close()


def test_dynamic_anchors_stored_scores():
    cfg = synth.preset(1, M=2 + 8 * 9, H=2, C=128, B=400, T=40, n_special=2)
    _dap_stream(cfg, (2, 5, 0.7, 0.1, 2, 72))


def test_dynamic_anchors_hybrid_scoring_batched_layers():
    cfg = synth.preset(1, M=2 + 8 * 9, H=3, C=64, B=400, T=40, n_special=2)
    _dap_stream(cfg, (2, 5, 0.7, 0.1, 2, 72), hybrid_beta=0.5, layers=2)


def test_camera_head_cache_follows_the_anchors():
    """Supp. C: the camera head's cache holds one token per frame under the same policy (no
    smoothing); its token is protected and released together with the aggregator's anchor."""
    cfg = synth.preset(1, M=2 + 6 * 6, H=2, C=64, B=200, T=60, n_special=2)
    cam = synth.preset(1, M=1, H=16, C=256, B=16, T=60, n_special=1)
    _dap_stream(cfg, (3, 4, 0.8, 0.2, 2, 36), camera=cam)
    _dap_stream(cfg, (3, 4, 0.8, 0.2, 2, 36), hybrid_beta=0.5, camera=cam)


def test_set_protect_argument_and_state_errors():
    torch = _torch()
    cfg = synth.preset(1, M=16, H=1, C=64, B=64, T=3, n_special=1)
    cache = make_cache(cfg, L=2)
    out = cache.new_output()
    with pytest.raises(B.OvggtError) as e:
        cache.set_protect(0, None, True)                         # no frame seen yet
    assert e.value.code == B.OVGGT_ERR_ARG
    fs = [synth.frame_inputs(cfg, l, 0) for l in range(2)]
    q, k, v, r = (dev(np.stack([f[x] for f in fs]), cfg) for x in "qkvr")
    cache.global_attn(q, k, v, out)
    with pytest.raises(B.OvggtError) as e:
        cache.set_protect(0, None, True)                         # mid-frame
    assert e.value.code == B.OVGGT_ERR_STATE
    cache.score_select(r, None); cache.compact()
    cache.set_protect(0, None, True, layer=1)
    assert cache.export(0)["flags"].sum() == 0 and cache.export(1)["flags"].sum() == cfg.M
    with pytest.raises(B.OvggtError):
        cache.set_protect(1, None, True)                         # frame 1 has not been appended
    with pytest.raises(B.OvggtError):
        cache.set_protect(0, None, True, layer=5)
    cache.close()


def test_bf16_output_is_the_rounded_fp32_output():
    """out_dtype = bf16 stores RNE(bf16) of exactly the value the fp32-output run stores."""
    cfg = synth.preset(1, M=200, H=3, C=64, B=500, T=5, n_special=3)
    torch = _torch()
    c32 = make_cache(cfg, L=1)
    c16 = B.Cache(1, cfg.H, cfg.d, cfg.M, cfg.C, cfg.B, cfg.dtype, out_dtype="bf16")
    o32, o16 = c32.new_output()[0], c16.new_output()[0]
    assert o16.dtype == torch.bfloat16
    for t in range(cfg.T):
        f = synth.frame_inputs(cfg, 0, t)
        args = [dev(f[x], cfg) for x in "qkvr"] + [torch.from_numpy(f["a"]).cuda()]
        c32.step(*args, o32, layer=0)
        c16.step(*args, o16, layer=0)
        assert torch.equal(o32.to(torch.bfloat16), o16), t
    c32.close(); c16.close()


def test_captured_step_replayed_from_a_hip_graph_matches_the_oracle():
    """One steady-state step (append with the carried moves, attention, merge, score/select) is
    captured into a HIP graph and replayed for 20 further frames, the inputs copied into the captured
    buffers before each replay: every replay's attention output against the oracle, and the cache
    (kept ids, layout, scores, flags, K, V) bit-exact at the end.  No kernel argument depends on the
    frame: the token ids come from device memory."""
    torch = _torch()
    cfg = synth.preset(1, M=300, H=4, C=256, B=1500, T=32, n_special=5)
    cache = make_cache(cfg, L=1)
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    out = cache.new_output()[0]
    eager = 9                                             # 5 frames fill the cache, 4 more evict
    f = synth.frame_inputs(cfg, 0, 0)
    fixed = [dev(f[x], cfg) for x in "qkvr"] + [torch.from_numpy(f["a"]).cuda()]

    def load(t):
        f = synth.frame_inputs(cfg, 0, t)
        for dst, x in zip(fixed[:4], "qkvr"):
            dst.copy_(dev(f[x], cfg))
        fixed[4].copy_(torch.from_numpy(f["a"]).cuda())
        return f

    def check(t, f):
        ref = orc.step(f["q"], f["k"], f["v"], f["r"], f["a"])
        torch.cuda.synchronize()
        err = rel_err(out.float().cpu().numpy().astype(np.float64), ref)
        assert err < TOL["bf16"], f"frame {t}: attention error {err:.3e}"

    for t in range(eager):
        f = load(t)
        cache.step(*fixed, out, layer=0)
        check(t, f)
    with pytest.raises(B.OvggtError):
        B.ovggt_cache_advance(cache.h, 0, 0)
    g = torch.cuda.CUDAGraph()
    f = load(eager)                                       # the inputs of the first replay are in place before the capture
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        cache.step(*fixed, out, layer=0)                  # enqueues nothing; counts as frame `eager` on the host
    assert cache.frames(0) == eager + 1
    for i in range(21):
        t = eager + i
        if i > 0:
            f = load(t)
            cache.advance(1, layer=0)
        g.replay()
        check(t, f)
        assert cache.frames(0) == t + 1 and cache.size(0) == cfg.B
        print(f"[graph] replay {i} (frame {t}) ok", flush=True)
    compare_cache(cache, orc)                             # applies the outstanding compaction with the stand-alone kernel
    with pytest.raises(B.OvggtError) as e:                # the handle left the captured state: a replay is refused
        cache.advance(1, layer=0)
    assert e.value.code == B.OVGGT_ERR_STATE
    t = eager + 21                                        # eager steps continue from where the replays stopped
    f = load(t)
    cache.step(*fixed, out, layer=0)
    check(t, f)
    compare_cache(cache, orc)
    assert cache.status(0) == 0
    cache.close()


def test_mfma_loop_helper_runs_and_rejects_bad_arguments():
    """The measurement helper behind bench.py's MFMA-loop figure (a library of its own): it runs, and
    rejects bad arguments.  Rates are reported by the benchmark, not asserted here."""
    from paper_2603_05959_amd import measure
    torch = _torch()
    sink = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    cst = measure.ovggt_measure_mfma_loop(sink, 512, False, 2000, stream)
    rnd = measure.ovggt_measure_mfma_loop(sink, 512, True, 2000, stream)
    assert np.isfinite([cst, rnd]).all() and cst > 0 and rnd > 0
    assert float(sink.abs().sum()) == 0.0
    for bad in ((None, 512, True, 100), (sink, 0, True, 100), (sink, 512, True, 0)):
        with pytest.raises(RuntimeError):
            measure.ovggt_measure_mfma_loop(*bad, stream)
