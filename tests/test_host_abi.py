"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-side validation works without a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2603_05959_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _built():
    from paper_2603_05959_amd import measure
    if not os.path.exists(B.LIB_PATH) or not os.path.exists(measure.LIB_PATH):
        from paper_2603_05959_amd import build
        build.build(verbose=False)


def test_header_symbols_are_exported():
    _built()
    hdr = open(os.path.join(ROOT, "include", "ovggt.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ovggt_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    # the measurement helper is a library of its own with a header of its own
    from paper_2603_05959_amd import measure
    hdr = open(os.path.join(ROOT, "include", "ovggt_measure.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared_m = set(re.findall(r"\b(ovggt_[a-z_]+)\s*\(", hdr))
    assert declared_m == set(measure.EXPORTS) and not (declared_m & declared)
    for name in declared_m:
        assert hasattr(measure.lib(), name), name
        assert not hasattr(lib, name), name


def test_query_bytes_and_config_validation():
    _built()
    cfg = B.make_config(1, 16, 64, 1374, 1024, 16384, "bf16")
    kv, meta, ws = B.ovggt_cache_query_bytes(cfg)
    cap = (16384 + 1374 + 127) // 128 * 128
    assert kv == 2 * 16 * cap * 64 * 2                 # 4 KiB per token per layer: the paper's 2*N_h*d elements in bf16
    assert meta >= cap * 9 and ws > 0 and kv % 256 == 0 and meta % 256 == 0 and ws % 256 == 0
    kv24, meta24, _ = B.ovggt_cache_query_bytes(B.make_config(24, 16, 64, 1374, 1024, 16384, "bf16"))
    assert kv24 == 24 * kv and meta24 == 24 * meta
    bad = [dict(head_dim=128), dict(budget=100), dict(n_layers=0), dict(resid_dim=0), dict(resid_dim=5000),
           dict(dtype=7), dict(score_mode=2), dict(score_mode=1, dtype="f32"), dict(score_mode=1, hybrid_beta=1.5),
           dict(score_mode=1, hybrid_beta=-0.5), dict(score_mode=1, n_heads=65), dict(softmax_scale=-1.0), dict(budget=131072), dict(out_dtype=3),
           dict(dtype="f32", out_dtype="bf16")]
    for kw in bad:
        args = dict(n_layers=1, n_heads=16, head_dim=64, tokens_per_frame=1374, resid_dim=1024, budget=16384,
                    dtype="bf16", score_mode=0, softmax_scale=0.0, out_dtype="f32")
        args.update(kw)
        with pytest.raises(B.OvggtError) as e:
            B.ovggt_cache_query_bytes(B.make_config(**args))
        assert e.value.code == B.OVGGT_ERR_ARG
    B.ovggt_cache_query_bytes(B.make_config(1, 16, 64, 1374, 1024, 16384, "bf16", score_mode=1, hybrid_beta=0.5))


def test_null_and_misaligned_arguments_rejected_before_any_launch():
    _built()
    lib = B.lib()
    cfg = B.make_config(1, 2, 64, 65, 128, 256, "f32")
    h = C.c_void_p()
    assert lib.ovggt_cache_init(C.byref(h), C.byref(cfg), None, None, None, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_cache_init(C.byref(h), C.byref(cfg), 0x1001, 0x2000, 0x3000, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_cache_init(None, C.byref(cfg), 0x1000, 0x2000, 0x3000, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_global_attn(None, 0, None, None, None, None, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_score_select(None, 0, None, None, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_cache_compact(None, 0, None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_cache_destroy(None) == B.OVGGT_ERR_ARG
    assert lib.ovggt_cache_advance(None, 0, 1) == B.OVGGT_ERR_ARG
    assert "memory" in B.strerror(B.OVGGT_ERR_NOMEM)
    assert B.strerror(0) == "ok" and "order" in B.strerror(B.OVGGT_ERR_STATE)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_05959_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(import|from)\s+oracle|oracle[/.]\w", src), f


def test_dap_policy_follows_the_oracle_schedule():
    """The host-side registration rule (no device work) against the oracle's on random inputs."""
    from oracle import ovggt_oracle as oc
    rng = np.random.default_rng(5)
    for k_max, gap, tau, eta, ns, npch in [(3, 100, 0.5, 0.05, 5, 1036), (1, 1, 0.9, 1.0, 0, 7), (2, 3, 0.3, 0.34, 1, 50)]:
        h = B.ovggt_dap_create(k_max, gap, tau, eta, ns, npch)
        pol = oc.DapPolicy(k_max, gap, tau, eta, ns, npch)
        mask = np.zeros(ns + npch, np.uint8)
        for t in range(12 * gap + 5):
            rho = float(rng.random())
            conf = rng.integers(0, 5, npch).astype(np.float32) if t % 2 else rng.random(npch).astype(np.float32)
            reg, dem = B.ovggt_dap_step(h, t, rho, conf, mask)
            m_ref, d_ref = pol.step(t, rho, conf)
            assert (reg == t) == (m_ref is not None) and (reg in (t, -1))
            assert dem == (-1 if d_ref is None else d_ref)
            if m_ref is not None:
                assert np.array_equal(mask, m_ref)
            assert B.ovggt_dap_active(h) == pol.active
        with pytest.raises(B.OvggtError):
            B.ovggt_dap_step(h, 3, 0.0, conf, mask)                  # frames must advance
        B.ovggt_dap_destroy(h)
    for bad in [(0, 100, 0.5, 0.05, 5, 10), (3, 0, 0.5, 0.05, 5, 10), (3, 100, 0.5, 0.0, 5, 10), (3, 100, 0.5, 1.5, 5, 10),
                (3, 100, float("nan"), 0.05, 5, 10), (3, 100, 0.5, 0.05, -1, 10), (3, 100, 0.5, 0.05, 5, 0)]:
        with pytest.raises(B.OvggtError):
            B.ovggt_dap_create(*bad)


def test_attention_plans_cover_every_tile_once():
    """Host-side walk of the attention launch plan over many shapes: every (head, query block, key
    tile) exactly once, pieces within the records a workgroup owns; where chunks are balanced by
    estimated cost, the busiest workgroup stays close to the mean."""
    shapes = [(1374, 16, 16384, 1), (1374, 16, 16384, 24), (1374, 16, 32768, 1), (1041, 16, 4096, 1),
              (1041, 16, 65536, 1), (200, 3, 700, 1), (1, 1, 64, 1), (37, 2, 74, 1), (130, 5, 1000, 1),
              (128, 16, 256, 1), (300, 8, 5000, 4), (130, 16, 300, 3), (150, 2, 400, 3), (1, 16, 188, 1),
              (500, 4, 3000, 2), (129, 1, 100000, 1), (2000, 32, 9000, 1), (64, 64, 640, 2), (600, 16, 1000, 8),
              (1041, 16, 8192, 24), (4096, 16, 4096, 1), (520, 2, 9000, 16)]
    for M, H, Bud, L in shapes:
        cfg = B.make_config(L, H, 64, M, 64, max(Bud, M), "bf16")
        for n_total in sorted({M, min(2 * M, Bud + M), (Bud + M) // 2, Bud + M - 1, Bud + M}):
            for n_wgs in (256, 64, 304):
                st = B.ovggt_attn_plan_stats(cfg, L, n_total, n_wgs)        # raises if inconsistent
                assert st["tiles_max"] >= st["tiles_min"] >= 0 and st["pieces_max"] >= 1
                if st["balanced"] and st["tiles_min"] > 30:
                    assert st["cost_max"] <= 1.12 * st["cost_mean"] + 1, (M, H, Bud, L, n_total, n_wgs, st)
    st = B.ovggt_attn_plan_stats(B.make_config(1, 16, 64, 1374, 1024, 16384, "bf16"), 1, 17758, 256)
    assert st["balanced"] == 1 and st["segments"] == 3 and st["pieces_max"] <= 2
    # 24 layers: 264 items per XCD over 32 workgroups = 8 rounds of whole items and one round of cut ones
    cfg24 = B.make_config(24, 16, 64, 1374, 1024, 16384, "bf16")
    st = B.ovggt_attn_plan_stats(cfg24, 24, 17758, 256)
    assert st["rounds"] == 9 and st["segments"] == 1 and st["tiles_max"] - st["tiles_min"] <= 8
    assert B.ovggt_cache_query_bytes(cfg24)[2] == B.ovggt_cache_query_bytes(B.make_config(1, 16, 64, 1374, 1024, 16384, "bf16"))[2]
    # items whose two halves of the workgroup share one head's tiles: all block pairs of every head when
    # the launch has an even number of heads (the odd eleventh block of two heads makes a mixed item)
    assert st["shared_items"] == 192 * 10
    assert B.ovggt_attn_plan_stats(B.make_config(1, 16, 64, 1374, 1024, 16384, "bf16"), 1, 17758, 256)["shared_items"] == 80
    assert B.ovggt_attn_plan_stats(B.make_config(1, 5, 64, 130, 64, 1000, "bf16"), 1, 1130, 256)["shared_items"] == 0
    assert B.ovggt_attn_plan_stats(B.make_config(1, 2, 64, 256, 64, 1000, "bf16"), 1, 1256, 256)["shared_items"] == 2
    assert B.ovggt_attn_plan_stats(B.make_config(1, 2, 64, 100, 64, 1000, "bf16"), 1, 1100, 256)["shared_items"] == 0
    print(st)
