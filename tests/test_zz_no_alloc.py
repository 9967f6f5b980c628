"""The entry point for callers that cannot allocate (ovggt_global_attn_static_ws): same results as
ovggt_global_attn, with the attention's partial records in the library's own device array."""
import numpy as np
import pytest

from oracle import ovggt_oracle as oc
from paper_2603_05959_amd import binding as B
from paper_2603_05959_amd import synth

pytestmark = pytest.mark.gpu


def _stream_both_ways(cfg, frames):
    """The same frames through two handles, one per entry point; returns the last frame's inputs and
    the reference output of the oracle for it."""
    import torch
    caches = [B.Cache(1, cfg.H, cfg.d, cfg.M, cfg.C, cfg.B, cfg.dtype) for _ in range(2)]
    outs = [c.new_output()[0] for c in caches]
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B)
    for t in range(frames):
        f = synth.frame_inputs(cfg, 0, t)
        q, k, v, r = (B.to_device(f[x], cfg.dtype) for x in "qkvr")
        a = torch.from_numpy(f["a"]).cuda()
        B.ovggt_global_attn(caches[0].h, 0, q, k, v, outs[0], caches[0].stream)
        B.ovggt_global_attn_static_ws(caches[1].h, 0, q, k, v, outs[1], caches[1].stream)
        for c in caches:
            c.score_select(r, a, layer=0)
            c.compact(layer=0)
        ref = orc.step(f["q"], f["k"], f["v"], f["r"], f["a"])
        torch.cuda.synchronize()
        o0, o1 = (o.float().cpu().numpy().astype(np.float64) for o in outs)
        rms = np.sqrt((ref ** 2).mean())
        assert np.abs(o1 - ref).max() / rms < 2e-2, (cfg.name, t)
        assert np.array_equal(o0, o1), (cfg.name, t, "the two entry points run the same plan on the same kernels")
    e0, e1 = caches[0].export(0), caches[1].export(0)
    for key in ("ids", "k", "v", "ss", "flags"):
        assert np.array_equal(e0[key], e1[key]), key
    assert np.array_equal(e1["ids"], orc.gid)
    for c in caches:
        assert c.status(0) == 0
        c.close()


def test_static_workspace_entry_point_matches_the_regular_one_twice_in_a_row():
    # two calls in a row share the library's array: a larger launch (11 tiles, several pieces per query
    # block) and then a smaller one (2 tiles), each compared with ovggt_global_attn and the oracle
    _stream_both_ways(synth.preset(1, M=300, H=4, C=128, B=1100, T=6, n_special=3), 6)
    _stream_both_ways(synth.preset(1, M=70, H=2, C=64, B=200, T=5, n_special=1), 5)


def test_static_workspace_entry_point_rejects_launches_beyond_its_array():
    import torch
    cfg = synth.preset(2, M=130, H=16, C=64, B=300, T=1, L=2, n_special=2)      # 32 (layer, head) pairs per batched call
    cache = B.Cache(cfg.L, cfg.H, cfg.d, cfg.M, cfg.C, cfg.B, cfg.dtype)
    out = cache.new_output()
    fs = [synth.frame_inputs(cfg, l, 0) for l in range(cfg.L)]
    q, k, v = (B.to_device(np.stack([f[x] for f in fs]), cfg.dtype) for x in "qkv")
    with pytest.raises(B.OvggtError) as e:
        B.ovggt_global_attn_static_ws(cache.h, B.OVGGT_ALL_LAYERS, q, k, v, out, cache.stream)
    assert e.value.code == B.OVGGT_ERR_TOO_LARGE and "static workspace" in str(e.value)
    assert cache.size(0) == 0                                                   # nothing changed
    B.ovggt_global_attn_static_ws(cache.h, 0, q[0], k[0], v[0], out[0], cache.stream)   # one layer of 16 heads fits
    torch.cuda.synchronize()
    assert cache.size(0) == cfg.M and cache.size(1) == 0
    cache.close()
