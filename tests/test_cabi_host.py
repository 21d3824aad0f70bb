"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and its
host-side argument checks return the documented error codes (no compute calls here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2511_21699_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    text = open(os.path.join(ROOT, "include", "cacheback.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(cb_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_header():
    assert C.sizeof(B.CbConfig) == 12 * 4
    assert C.sizeof(B.CbKvLayer) == 40


def _kv(cap=100, paged=False):
    return B.CbKvLayer(0x1000, 0x2000, cap, 0x3000 if paged else None, 8 if paged else 0, 0)


def test_workspace_bytes_and_bad_configs():
    good = B.make_config(32, 8, 128, "bf16", "bf16", 1, 128, 8, 32000)
    # bf16 / head_dim 128: room for the MFMA kernel's bf16 partials at 64 splits (4,224 bytes per 16-row tile and
    # split), not for the scalar kernel's fp32 ones at that split count
    assert 128 * 32 // 16 * 64 * 4224 < B.workspace_bytes(good) < 128 * 32 * 64 * 132 * 4
    scalar = B.make_config(32, 8, 128, "f32", "f32", 1, 128, 8, 32000)
    assert B.workspace_bytes(scalar) > 128 * 32 * 64 * 132 * 4
    for bad in (B.make_config(32, 5, 128, "bf16", "bf16", 1, 64, 6, 100),
                B.make_config(32, 8, 96, "bf16", "bf16", 1, 64, 6, 100),
                B.make_config(32, 8, 128, "bf16", "bf16", 1, 257, 6, 100),
                B.make_config(32, 8, 128, "bf16", "bf16", 65, 64, 6, 100),
                B.make_config(32, 8, 128, "bf16", "bf16", 1, 64, 6, 0)):
        with pytest.raises(B.CbError) as e:
            B.workspace_bytes(bad)
        assert e.value.code == B.CB_EINVAL


def test_tree_and_capacity_checks():
    cfg = B.make_config(4, 2, 64, "f32", "f32", 2, 8, 3, 100)
    ok = dict(kv_len=[10, 20], node_offsets=[0, 3, 7], parent=[-1, 0, 1, -1, 0, 0, 2])
    assert B.check_verify_args(cfg, 2, _kv(), **ok)[0] == B.CB_OK
    cases = [
        (dict(ok, parent=[0, 0, 1, -1, 0, 0, 2]), B.CB_ETREE),        # root parent not -1
        (dict(ok, parent=[-1, 0, 2, -1, 0, 0, 2]), B.CB_ETREE),       # parent[i] == i
        (dict(ok, parent=[-1, 0, 1, -1, 0, 0, -1]), B.CB_ETREE),      # negative parent below the root
        (dict(ok, node_offsets=[0, 3, 12], parent=[-1, 0, 1] + [-1] + [0] * 8), B.CB_ECAP),   # > max_nodes
        (dict(ok, kv_len=[10, 98]), B.CB_ECAP),                       # prefix + nodes beyond the cache
        (dict(ok, kv_len=[-1, 20]), B.CB_EINVAL),
        (dict(ok, node_offsets=[1, 3, 7]), B.CB_EINVAL),
        (dict(ok, node_offsets=[0, 0, 7]), B.CB_EINVAL),              # a sequence without a root
    ]
    for args, code in cases:
        rc, text = B.check_verify_args(cfg, 2, _kv(), **args)
        assert rc == code and text, (args, rc, text)
    deep = dict(kv_len=[1], node_offsets=[0, 5], parent=[-1, 0, 1, 2, 3])      # depth 4 > max_depth 3
    assert B.check_verify_args(cfg, 1, _kv(), **deep)[0] == B.CB_ETREE
    assert B.check_verify_args(cfg, 3, _kv(), **ok)[0] == B.CB_EINVAL          # batch > max_batch
    pcfg = B.make_config(4, 2, 64, "f32", "f32", 2, 8, 3, 100, block_size=16)
    assert B.check_verify_args(pcfg, 2, _kv(paged=True), **ok)[0] == B.CB_OK   # 8 blocks x 16 = 128 slots
    assert B.check_verify_args(pcfg, 2, _kv(paged=True), **dict(ok, kv_len=[10, 125]))[0] == B.CB_ECAP
    assert B.check_verify_args(pcfg, 2, _kv(paged=False), **ok)[0] == B.CB_EINVAL


def test_init_without_device_fails_cleanly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = B.load()
    cfg = B.make_config(4, 2, 64, "f32", "f32", 1, 8, 3, 100)
    ctx = C.c_void_p()
    rc = lib.cb_init(C.byref(cfg), 0x10000, 1 << 30, C.byref(ctx))
    assert rc == B.CB_EHIP and not ctx.value and lib.cb_last_error(None)


def _plan_invariants(cfg, kv_len, offs, plan, g):
    n = np.diff(offs)
    lens = np.asarray(kv_len) + n
    assert plan["chunk"] % 32 == 0 and plan["chunk"] >= 32
    assert plan["nsplit"] >= 1
    cap = cfg.max_splits if cfg.max_splits > 0 else 64
    assert plan["nsplit"] <= cap
    # the splits cover the longest sequence exactly once, with no empty trailing split
    assert plan["nsplit"] * plan["chunk"] >= lens.max()
    assert (plan["nsplit"] - 1) * plan["chunk"] < lens.max()
    if plan["impl"] == 2:
        assert plan["tile_rows"] in (64, 128, 256)
        assert plan["tile_rows"] >= min(256, n.max() * g) or plan["tile_rows"] == 256
        tiles = -(-(n * g) // plan["tile_rows"]) * cfg.num_kv_heads
    else:
        assert plan["tile_rows"] == 1
        tiles = n * cfg.num_q_heads
    assert plan["workgroups"] == int((tiles * -(-lens // plan["chunk"])).sum())


def test_attention_plan_invariants_on_the_paper_shapes_and_random_batches():
    # the five workload shapes: (Hq, Hkv, D, dtype, kv_len, node counts, block)
    shapes = [(8, 8, 64, "f32", [256], [15], 0), (32, 32, 128, "bf16", [2048], [64], 0),
              (32, 8, 128, "bf16", [8192], [128], 0), (40, 40, 128, "bf16", [65536], [256], 0)]
    for Hq, Hkv, D, dt, kv, n, blk in shapes:
        cfg = B.make_config(Hq, Hkv, D, dt, dt, len(kv), max(n), 8, 1000, blk)
        offs = np.concatenate([[0], np.cumsum(n)])
        plan = B.plan_attention(cfg, kv, offs)
        _plan_invariants(cfg, kv, offs, plan, Hq // Hkv)
        assert plan["impl"] == (2 if (dt == "bf16" and D == 128) else 1)
    # the 7B-shaped step fills the chip's 256 compute units in one round
    cfg = B.make_config(32, 32, 128, "bf16", "bf16", 1, 64, 8, 32000)
    plan = B.plan_attention(cfg, [2048], [0, 64])
    assert 218 <= plan["workgroups"] <= 256 and plan["tile_rows"] == 64
    rng = np.random.default_rng(7)
    for _ in range(200):
        Bn = int(rng.integers(1, 17))
        Hkv = int(rng.choice([1, 2, 8, 32]))
        g = int(rng.choice([1, 4, 8]))
        n = rng.integers(1, 97, Bn)
        kv = rng.integers(0, 20000, Bn)
        ms = int(rng.choice([0, 1, 3, 16, 200]))
        cfg = B.make_config(Hkv * g, Hkv, 128, "bf16", "bf16", Bn, 96, 8, 1000, 16, ms)
        offs = np.concatenate([[0], np.cumsum(n)])
        _plan_invariants(cfg, kv, offs, B.plan_attention(cfg, kv, offs), g)
        forced = int(rng.integers(1, 40))
        p = B.plan_attention(cfg, kv, offs, forced)
        _plan_invariants(cfg, kv, offs, p, g)
        assert p["nsplit"] <= forced


def test_attention_plan_rejects_bad_shapes():
    cfg = B.make_config(8, 8, 128, "bf16", "bf16", 2, 8, 3, 100)
    for kv, offs in (([5], [1, 4]), ([5], [0, 0]), ([5], [0, 9]), ([-1], [0, 3]), ([1, 2, 3], [0, 1, 2, 3])):
        with pytest.raises(B.CbError):
            B.plan_attention(cfg, kv, offs)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so (before it touches torch or the library)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_no_alloc_entry_point_checks_its_arguments_on_the_host():
    """cb_tree_attention_noalloc rejects bad arguments, and shapes whose scratch need exceeds the library's
    fixed device array, before it touches a device (so this runs without a GPU; nothing is launched)."""
    L = B.load()
    i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))

    def call(cfg, kv, kv_len, offs, q=0x10000, out=0x20000, par=0x30000):
        a, b = i32(kv_len), i32(offs)
        rc = L.cb_tree_attention_noalloc(C.byref(cfg), None, len(a), q, C.byref(kv), ip(a), ip(b), par, out)
        return rc, L.cb_last_error(None).decode()

    ragged = B.make_config(32, 32, 128, "bf16", "bf16", 16, 96, 8, 32000, 16, 72)
    kv = B.CbKvLayer(0x1000, 0x2000, 20000, 0x3000, 1100, 0)
    lens = [16000] + [600] * 15
    offs = np.arange(17) * 96
    # one long sequence among short ones: the planner spreads it over several splits, and the partial states
    # of 1536 nodes x 32 heads then take about 13 MB per split -- beyond the library's 32 MiB
    plan = B.plan_attention(ragged, lens, offs)
    assert plan["nsplit"] >= 4, plan
    rc, text = call(ragged, kv, lens, offs)
    assert rc == B.CB_ECAP and "scratch" in text, (rc, text)
    assert call(ragged, kv, lens, offs, q=0)[0] == B.CB_EINVAL       # null pointer
    assert call(ragged, kv, lens, offs, out=0x20004)[0] == B.CB_EINVAL   # misaligned
    assert call(ragged, kv, lens[:1] + [-5] + lens[2:], offs)[0] == B.CB_EINVAL
    assert call(ragged, kv, [17590] * 16, offs)[0] == B.CB_ECAP      # prefix + nodes beyond the block table
    bad = B.make_config(32, 5, 128, "bf16", "bf16", 1, 64, 6, 100)
    assert call(bad, kv, [10], [0, 4])[0] == B.CB_EINVAL
