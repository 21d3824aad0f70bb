"""Shared driver for the GPU parity tests: run the HIP library through its C ABI on a workload and
compare every output with the CPU oracle on the same inputs."""
from __future__ import annotations

import numpy as np

from oracle import cb_oracle as O
from paper_2511_21699_amd import binding as B
from paper_2511_21699_amd import workloads as W

# Tolerances of the attention output against the float64 oracle:
#   |gpu - ref| <= atol + rtol * |ref| elementwise, and, because the synthetic outputs can be far
#   smaller than atol, also max|gpu - ref| <= rel_to_max * max|ref| (a scale-free bound).
TOL = {"bf16": dict(atol=2e-2, rtol=1e-2, rel_to_max=2e-2), "f32": dict(atol=1e-5, rtol=1e-5, rel_to_max=1e-5)}


def check_attention(case, got_f64: np.ndarray, ref: np.ndarray, what: str = ""):
    tol = TOL[case.dtype]
    err = np.abs(got_f64 - ref)
    bound = tol["atol"] + tol["rtol"] * np.abs(ref)
    worst = float((err / bound).max())
    assert (err <= bound).all(), f"{what}: attention outside atol/rtol (worst ratio {worst:.3g}, max err {err.max():.3g})"
    scale_free = float(err.max() / np.abs(ref).max())
    assert scale_free <= tol["rel_to_max"], f"{what}: max|err|/max|ref| = {scale_free:.3g}"
    return scale_free


def sample_rows(case, count: int, seed: int = 0) -> np.ndarray:
    """Random (sequence, head, node) triples, always including each sequence's root and last node."""
    rng = np.random.default_rng(seed)
    rows = []
    for b in range(case.B):
        n = int(case.node_offsets[b + 1] - case.node_offsets[b])
        rows += [(b, 0, 0), (b, case.Hq - 1, n - 1)]
    while len(rows) < count:
        b = int(rng.integers(case.B))
        n = int(case.node_offsets[b + 1] - case.node_offsets[b])
        rows.append((b, int(rng.integers(case.Hq)), int(rng.integers(n))))
    return np.asarray(rows, dtype=np.int32)


def structured_rows(case, per_tile: int = 1) -> np.ndarray:
    """(sequence, head, node) triples that put `per_tile` rows into every 16-row tile of every kv head of
    every sequence -- the unit a wavefront of the MFMA kernel owns -- at a row position that walks through
    the tile with the tile and head numbers.  The kernel's rows of one kv head are node * g + (head % g);
    every workgroup row tile (64, 128 or 256 rows) and every wave inside it is a union of such 16-row
    tiles, and every row attends to the whole prefix, i.e. takes a contribution from every split."""
    g = case.Hq // case.Hkv
    rows = []
    for b in range(case.B):
        n = int(case.node_offsets[b + 1] - case.node_offsets[b])
        m = n * g
        for hk in range(case.Hkv):
            for t in range((m + 15) // 16):
                for j in range(per_tile):
                    r = t * 16 + (t + hk + 5 * j + 3 * b) % 16
                    r = min(r, m - 1)
                    rows.append((b, hk * g + r % g, r // g))
    return np.asarray(sorted(set(rows)), dtype=np.int32)


def run_case(case, rows=None, layout=B.CB_LAYOUT_TOKEN_MAJOR, options=None, max_splits=0, compact=True,
             threads=16, what="", expect_status=0):
    """Full parity run.  ``rows`` = None checks every attention row, else the sampled triples."""
    import torch
    print(f"[case] {what or case.name} dtype={case.dtype} B={case.B} Hq={case.Hq} Hkv={case.Hkv} D={case.D} "
          f"kv_len={case.kv_len[:4].tolist()} nodes={np.diff(case.node_offsets)[:4].tolist()} layout={layout} "
          f"options={options}", flush=True)
    dc = B.DeviceCase(case, layout=layout)
    ver = B.Verifier(B.config_for_case(case, max_splits=max_splits))
    for k, v in (options or {}).items():
        ver.set_option(k, v)
    try:
        out, acc_len, acc_tok = ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent,
                                                case.tokens, dc.logits)
        torch.cuda.synchronize()
        status = ver.device_status()
        assert status & 3 == 0                   # bits 0-1: tree problems; bits 4 and 5 only report how a merge went
        assert status & expect_status == expect_status, f"{what}: device status {status}, expected bits {expect_status}"
        # ---- argmax / acceptance: bit-exact
        a_ref, res = O.verify(case)
        a_gpu = ver.get_argmax(case.total_nodes)
        assert np.array_equal(a_gpu, a_ref), f"{what}: argmax differs at rows {np.flatnonzero(a_gpu != a_ref)[:8]}"
        path_gpu = ver.get_path(case.B)
        for b, (L, path, toks) in enumerate(res):
            assert acc_len[b] == L, f"{what}: accepted_len[{b}] {acc_len[b]} != {L}"
            assert acc_tok[b, :L + 1].tolist() == toks.tolist() and (acc_tok[b, L + 1:] == -1).all()
            assert path_gpu[b, :L + 1].tolist() == path.tolist() and (path_gpu[b, L + 1:] == -1).all()
        # ---- attention: tolerance against the float64 oracle
        got = W.to_f64(B.to_host(out, case.dtype), case.dtype)
        if rows is None:
            ref = O.attention(case, threads=threads)
            sf = check_attention(case, got, ref, what)
        else:
            ref = O.attention_rows(case, rows, threads=threads)
            sel = np.stack([got[case.node_offsets[b] + i, h] for b, h, i in rows])
            sf = check_attention(case, sel, ref, what)
        # ---- compaction: byte-exact against the oracle's copy
        if compact:
            new_len = ver.compact_kv([dc.kv], case.B)
            torch.cuda.synchronize()
            k_ref, v_ref = case.k.copy(), case.v.copy()
            for b, (L, path, toks) in enumerate(res):
                assert O.compact(case, k_ref, v_ref, b, path) == new_len[b]
            k_gpu, v_gpu = B.to_host(dc.k, case.dtype), B.to_host(dc.v, case.dtype)
            if layout == B.CB_LAYOUT_HEAD_MAJOR:
                k_gpu, v_gpu = k_gpu.swapaxes(1, 2), v_gpu.swapaxes(1, 2)
            assert np.array_equal(k_gpu.view(np.uint8 if False else k_gpu.dtype), k_ref), f"{what}: compacted K differs"
            assert np.array_equal(v_gpu, v_ref), f"{what}: compacted V differs"
        return dict(scale_free_err=sf, accepted=[int(x) for x in acc_len])
    finally:
        ver.close()
