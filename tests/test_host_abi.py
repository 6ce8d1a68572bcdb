"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
validates configurations on the host, and its host-side arithmetic (memory accounting, K
layout offsets) matches the paper's printed numbers and the binding's permutation."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_2512_00504_amd as P
from paper_2512_00504_amd.state import k_cache_to_rows, k_rows_to_cache

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden(name):
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split(":")
                out[k.strip()] = float(v)
    return out


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", name)).read()
                     for name in sorted(os.listdir(os.path.join(ROOT, "include"))) if name.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gkv_[a-z_0-9]+)\s*\(", header))
    assert {"gkv_attend_decode", "gkv_score_window", "gkv_global_update", "gkv_select_topk",
            "gkv_compact"} <= declared
    lib = ctypes.CDLL(P.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in gkv.h but not exported"
    assert declared == set(P.EXPORTS)


def _cfg(**kw):
    base = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, head_dim=64, budget=64, window=8,
                interval=16, capacity=96, dtype="f32")
    base.update(kw)
    return P.make_config(**base)


def test_create_validates_configuration():
    ctx = P.Context(_cfg())
    assert ctx.workspace_bytes() > 0
    ctx.close()
    bad = [dict(window=17),                 # w > s
           dict(window=8, budget=8),        # w >= b
           dict(n_q_heads=7),               # h_q % h_kv
           dict(alpha=1.5), dict(alpha=float("nan")),
           dict(dtype=3), dict(combine=5),
           dict(capacity=64),               # < b + s
           dict(capacity=100),              # not a multiple of 32
           dict(head_dim=62), dict(head_dim=512)]
    for kw in bad:
        with pytest.raises(P.GkvError):
            P.Context(_cfg(**kw))
    lib = P.load_library()
    assert lib.gkv_create(None, None) == 1
    assert lib.gkv_status_string(6) == b"cache capacity exceeded"


def test_create_rejects_shapes_whose_kernels_would_not_fit_lds():
    # the plain attend kernel keeps 4 x float[capacity + 1 + d] in LDS: 66,576 bytes at capacity
    # 4096, d = 64, over the 64 KiB a workgroup gets; 4000 rows fit
    with pytest.raises(P.GkvError) as e:
        P.Context(_cfg(budget=2048, interval=128, capacity=4096))
    assert e.value.status == 2
    P.Context(_cfg(budget=2048, interval=128, capacity=4000)).close()
    with pytest.raises(P.GkvError) as e:       # bf16 too: "force_generic" may select the same kernel
        P.Context(_cfg(budget=2048, interval=128, capacity=4096, dtype="bf16", head_dim=128, n_q_heads=14))
    assert e.value.status == 2


def test_split_count_raised_after_sizing_the_workspace_is_refused():
    cfg = _cfg(dtype="bf16", head_dim=128, n_q_heads=14, budget=512, window=16, interval=128, capacity=640)
    ctx = P.Context(cfg)
    lib = P.load_library()
    small = ctx.workspace_bytes()                       # sized without split-K partials
    fake = ctypes.c_void_p(4096)                        # never dereferenced: the call fails before any launch
    ctx.set_param("attend_splits", 3)
    rc = lib.gkv_attend_decode(ctx.h, fake, fake, fake, fake, fake, fake, 0, fake, fake, 0, fake, fake, None)
    assert rc == 3
    assert ctx.workspace_bytes() > small                # sizing again covers the partials
    ctx.close()


def test_calls_reject_null_pointers_without_a_gpu():
    ctx = P.Context(_cfg())
    lib = P.load_library()
    n = ctypes.c_void_p(None)
    assert lib.gkv_attend_decode(ctx.h, n, n, n, n, n, n, 0, n, n, 0, n, n, n) == 1
    assert lib.gkv_score_window(ctx.h, n, n, n, 0, 0, n, n, n) == 1
    assert lib.gkv_global_update(ctx.h, n, n, n, 0, 0, n, n) == 1
    assert lib.gkv_select_topk(ctx.h, n, n, 0, 0, n, n, n) == 1
    assert lib.gkv_compact(ctx.h, n, n, n, n, n, n, n, 0, n, n) == 1
    assert lib.gkv_evict(ctx.h, n, n, n, n, n, n, 0, 0, n, n, n, n, n) == 1
    assert lib.gkv_set_param(ctx.h, b"no_such_knob", 1) == 1


def test_memory_accounting_reproduces_the_papers_appendix():
    g = _golden("memory_analysis.txt")
    GB = float(2 ** 30)
    # the paper's example: 28 layers, 2 KV heads, d = 128, bf16
    one = P.make_config(28, 1, 28, 2, 128, 512, 16, 128, 640, "bf16")
    kv, _ = P.cache_bytes(one, 16384)
    assert round(kv / GB, 2) == g["full_kv_per_sequence_gb"]
    full = P.make_config(28, 128, 28, 2, 128, 512, 16, 128, 640, "bf16")
    kv_full, _ = P.cache_bytes(full, 16384)
    assert round(kv_full / GB) == g["full_kv_batch128_gb"]
    for b in (512, 1024, 2048):
        cfg = P.make_config(28, 128, 28, 2, 128, b, 16, 128, b + 128, "bf16")
        kv, sc = P.cache_bytes(cfg, b + 128, 2)
        assert kv / GB == pytest.approx(g[f"compressed_kv_gb_b{b}"], abs=0.011)
        # savings: exact values are 96.09 / 92.97 / 86.72 %, printed to one decimal
        assert 100 * (1 - kv / kv_full) == pytest.approx(g[f"saving_percent_b{b}"], abs=0.08)
        kv_b, sc_b = P.cache_bytes(cfg, b, 2)
        assert sc_b / kv_b == pytest.approx((b - 16) / (b * 128 * 2))
        assert sc_b / kv_b == pytest.approx(g["score_fraction_approx"], rel=0.04)


def test_k_offset_matches_the_layout_permutation():
    for dtype, tdt, idt in (("bf16", torch.bfloat16, torch.int16), ("f32", torch.float32, torch.int32)):
        cfg = _cfg(dtype=dtype, head_dim=64, capacity=96)
        ids = torch.arange(96 * 64, dtype=torch.int32).reshape(96, 64).to(idt)      # 6144 ids fit in int16
        for n_tiled in (0, 32, 96):
            cache = k_rows_to_cache(ids.view(tdt), n_tiled)
            flat = cache.view(idt).reshape(-1)
            for (r, c) in ((0, 0), (1, 0), (15, 63), (16, 0), (17, 9), (31, 8), (32, 0), (40, 7), (40, 8), (95, 63)):
                off = P.k_offset(cfg, r, c, n_tiled)
                assert int(flat[off]) == r * 64 + c, (dtype, n_tiled, r, c)
            assert torch.equal(k_cache_to_rows(cache, n_tiled).view(idt), ids)
    # row 17, channel 9 of a bf16 d=64 block: tile 1 (1024) + chunk 1 (128) + row 1 (8) + 1
    assert P.k_offset(_cfg(dtype="bf16"), 17, 9, 32) == 1024 + 128 + 8 + 1
    assert P.k_offset(_cfg(dtype="bf16"), 17, 9, 16) == 17 * 64 + 9
    assert P.k_offset(_cfg(), -1, 0, 0) == -1 and P.k_offset(_cfg(), 0, 64, 0) == -1


def test_benchmark_refuses_more_than_one_gpu():
    # one GPU is all this build measures: asking for more ends with a message, before any GPU work
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "--gpus must be 1" in (res.stdout + res.stderr)
