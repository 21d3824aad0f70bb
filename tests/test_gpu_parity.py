"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs.  Integer results (argmax, accepted length/tokens/path, compacted K/V bytes) must be
bit-exact; attention must be within the tolerances in gpu_harness.TOL."""
import numpy as np
import pytest

from paper_2511_21699_amd import binding as B
from paper_2511_21699_amd import workloads as W
from tests.gpu_harness import check_attention, run_case, sample_rows, structured_rows

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- sizes the oracle finishes whole
def test_config1_tiny_fp32_full():
    for off in range(4):
        r = run_case(W.make_config(1, seed_offset=off), what=f"cfg1 seed+{off}")
    assert r["scale_free_err"] < 1e-5


@pytest.mark.parametrize("impl", [1, 2])
def test_config2_7b_shape_full(impl):
    run_case(W.make_config(2), options={"attn_impl": impl}, what=f"cfg2 impl={impl}")


@pytest.mark.parametrize("impl", [1, 2])
def test_config2_peaked_softmax(impl):
    # queries scaled so the softmax concentrates: outputs are O(1) and the tolerance bites
    run_case(W.make_config(2, peaked=True, S=700), options={"attn_impl": impl}, what=f"cfg2 peaked impl={impl}")


@pytest.mark.parametrize("impl", [1, 2])
def test_config3_gqa_reduced_prefix(impl):
    run_case(W.make_config(3, S=1500), options={"attn_impl": impl}, what=f"cfg3 S=1500 impl={impl}")
    run_case(W.make_config(3, S=777, peaked=True), options={"attn_impl": impl}, what=f"cfg3 S=777 peaked impl={impl}")


@pytest.mark.parametrize("impl", [1, 2])
def test_config4_ragged_paged_reduced(impl):
    run_case(W.make_config(4, B=5, S=(100, 1500), Hq=8, Hkv=8), options={"attn_impl": impl},
             what=f"cfg4 reduced impl={impl}")


@pytest.mark.parametrize("impl", [1, 2])
def test_config5_long_reduced(impl):
    run_case(W.make_config(5, S=3000, Hq=8, Hkv=8, V=128256, N=256), options={"attn_impl": impl},
             what=f"cfg5 reduced impl={impl}")


# ---------------------------------------------------------------- full sizes, sampled rows
# (rows in every 16-row tile of every kv head -- every workgroup row tile and every wave of it -- and
# each of them attends to the whole prefix, so every split, the first, the last and the one that
# reaches the tree, contributes to every checked row)
def test_config3_gqa_full_size_sampled():
    case = W.make_config(3)
    rows = structured_rows(case, per_tile=2)
    assert len(rows) >= 512
    run_case(case, rows=rows, what="cfg3 full")


def test_config4_ragged_full_size_sampled():
    case = W.make_config(4)
    rows = structured_rows(case)[::4]          # every fourth (tile, head) pair: still every sequence, head and tile index
    rows = np.concatenate([rows, sample_rows(case, 64)])
    assert len(rows) >= 512
    run_case(case, rows=rows, max_splits=72, what="cfg4 full")


def test_config5_long_full_size_sampled():
    case = W.make_config(5)
    rows = structured_rows(case)
    assert len(rows) >= 512
    run_case(case, rows=rows, what="cfg5 full")


# ---------------------------------------------------------------- edge cases
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_single_node_tree_and_empty_prefix(dtype, D):
    run_case(W.custom_case(31, dtype, 2, 4, 2, D, 300, [0, 5], [[-1], [-1]]), what="single node")
    run_case(W.custom_case(32, dtype, 1, 4, 4, D, 300, [0], [W.chain_tree(9)]), what="empty prefix chain")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_max_nodes_chain_and_star(dtype):
    run_case(W.custom_case(33, dtype, 1, 2, 2, 128, 500, [131], [W.chain_tree(256)], p_match=0.97), what="chain 256")
    run_case(W.custom_case(34, dtype, 1, 2, 1, 128, 500, [77], [W.star_tree(256)]), what="star 256")


@pytest.mark.parametrize("S", [1, 31, 32, 33, 255, 257, 1023])
def test_ragged_prefix_lengths_around_tile_edges(S):
    rng = np.random.default_rng(S)
    par = W.random_tree(rng, 70, 4, 7, False)[0]
    run_case(W.custom_case(40 + S, "bf16", 1, 4, 2, 128, 1000, [S], [par], q_scale=3.0), what=f"S={S}")


@pytest.mark.parametrize("merge", ["cooperative", "last_arrival", "merge_kernel", "gave_up"])
@pytest.mark.parametrize("splits", [1, 2, 5, 13])
def test_split_counts_agree_with_the_oracle(splits, merge):
    """Every way the splits of a tile can be merged: cooperatively by the tile's workgroups (the default when
    the grid fits the machine in one round), by the last workgroup to finish, by the separate merge kernel,
    and cooperatively with a spin limit of zero -- every workgroup but the one that completes a tile gives up
    at once and leaves its slice to that one (status bit 32 says that it happened)."""
    rng = np.random.default_rng(5)
    par = W.random_tree(rng, 64, 4, 6, False)[0]
    case = W.custom_case(50, "bf16", 1, 8, 8, 128, 1000, [1000], [par], q_scale=2.0)
    opts = {"cooperative": {}, "last_arrival": {"coop_merge": 0}, "merge_kernel": {"external_merge": 1},
            "gave_up": {"merge_spin_limit": 0}}[merge]
    run_case(case, options=dict(opts, splits=splits), what=f"splits={splits} merge={merge}",
             expect_status=32 if (merge == "gave_up" and splits > 1) else 0)


@pytest.mark.parametrize("splits", [2, 3, 7])
def test_ragged_batch_with_forced_splits(splits):
    # several sequences of unequal length are launched longest first within every XCD, and by default
    # with as few splits as spread the longest one (often a single one): here the splits, and with
    # them the tiles' merges and the workgroups that find no keys, are forced
    case = W.make_config(4, B=6, S=(200, 3000), V=2048)
    run_case(case, options={"splits": splits}, what=f"ragged batch, {splits} splits")
    run_case(case, options={"splits": splits, "fuse_logits": 0, "coop_merge": 0}, what=f"ragged batch, {splits} splits, separate launches")


@pytest.mark.parametrize("opts", [{}, {"coop_merge": 0}, {"fuse_logits": 0}, {"fuse_logits": 0, "coop_merge": 0}])
def test_merge_across_xcds(opts):
    """15 workgroups (3 kv heads x 5 splits) cannot be renumbered into whole tiles per XCD, so the splits of a
    tile run on different XCDs and the merge must read the partials past its own L2: the device status word
    reports that branch (bit 16), and the results are the oracle's -- for the cooperative merge, the
    last-arrival merge, and the one-launch verification's acceptance behind either."""
    rng = np.random.default_rng(15)
    par = W.random_tree(rng, 12, 3, 4, False)[0]          # 12 logits items for 15 workgroups: small enough for one launch
    case = W.custom_case(55, "bf16", 1, 3, 3, 128, 8000, [1100], [par], q_scale=2.0, p_match=0.8)
    run_case(case, options=dict(opts, splits=5), what=f"cross-XCD merge {opts}", expect_status=16)


@pytest.mark.parametrize("layout", [B.CB_LAYOUT_TOKEN_MAJOR, B.CB_LAYOUT_HEAD_MAJOR])
@pytest.mark.parametrize("paged", [False, True])
def test_cache_layouts(layout, paged):
    rng = np.random.default_rng(6)
    pars = [W.random_tree(rng, n, 3, 6, False)[0] for n in (40, 17, 64)]
    case = W.custom_case(60, "bf16", 3, 8, 2, 128, 2000, [300, 45, 1000], pars, paged=paged)
    run_case(case, layout=layout, what=f"layout={layout} paged={paged}")


def test_argmax_ties_and_odd_vocab():
    # coarse logits: the row maximum repeats many times; vocabulary not a multiple of the vector width
    rng = np.random.default_rng(7)
    par = W.random_tree(rng, 50, 4, 6, False)[0]
    for dtype in ("bf16", "f32"):
        case = W.custom_case(70, dtype, 1, 2, 2, 64, 33333, [10], [par])
        x = np.round(rng.standard_normal(case.logits.shape, dtype=np.float32) * 2) / 2
        x[3, :] = -0.0; x[3, 9000] = 0.0
        x[4, :] = 1.5
        x[5, -1] = 9.0
        x[6, [8191, 8192]] = 9.0
        case.logits = W.f32_to_bf16_bits(x) if dtype == "bf16" else x
        run_case(case, what=f"ties {dtype}")


def test_non_ancestor_keys_do_not_leak_on_gpu():
    """Changing K/V of nodes that are not ancestors of node i leaves node i's output bit-identical."""
    import torch
    rng = np.random.default_rng(8)
    par = W.random_tree(rng, 64, 4, 6, False)[0]
    case = W.custom_case(80, "bf16", 1, 4, 4, 128, 100, [500], [par], q_scale=2.0)
    target = 37
    anc, x = set(), target
    while x >= 0:
        anc.add(x); x = int(par[x])
    outs = []
    for poke in (False, True):
        c2 = case
        if poke:
            k, v = case.k.copy(), case.v.copy()
            for a in range(64):
                if a not in anc:
                    k[0, 500 + a] = W.f32_to_bf16_bits(np.full(k.shape[2:], 30.0, dtype=np.float32))
                    v[0, 500 + a] = W.f32_to_bf16_bits(np.full(v.shape[2:], -7.0, dtype=np.float32))
            import copy
            c2 = copy.copy(case); c2.k, c2.v = k, v
        dc = B.DeviceCase(c2)
        ver = B.Verifier(B.config_for_case(c2))
        out, _, _ = ver.verify_tree(dc.q, dc.kv, c2.kv_len, c2.node_offsets, c2.parent, c2.tokens, dc.logits)
        outs.append(B.to_host(out, "bf16")[target].copy())
        ver.close()
    assert np.array_equal(outs[0], outs[1])


def test_multi_layer_compaction_and_device_form():
    """cb_verify_tree_device leaves its results on the device; cb_compact_kv moves several layers at once."""
    import torch
    from oracle import cb_oracle as O
    rng = np.random.default_rng(9)
    pars = [W.chain_tree(30), W.random_tree(rng, 48, 3, 6, False)[0]]
    case = W.custom_case(90, "bf16", 2, 4, 2, 128, 64, [37, 120], pars, paged=True, p_match=0.9)
    dc = B.DeviceCase(case)
    layers_k = [dc.k] + [torch.randn_like(dc.k) for _ in range(2)]
    layers_v = [dc.v] + [torch.randn_like(dc.v) for _ in range(2)]
    before = [(B.to_host(k, "bf16").copy(), B.to_host(v, "bf16").copy()) for k, v in zip(layers_k, layers_v)]
    ver = B.Verifier(B.config_for_case(case))
    d_par = torch.from_numpy(case.parent).cuda(); d_tok = torch.from_numpy(case.tokens).cuda()
    out = torch.empty_like(dc.q)
    d_len = torch.zeros(2, dtype=torch.int32, device="cuda")
    d_acc = torch.zeros(2, case.max_depth + 1, dtype=torch.int32, device="cuda")
    ver.verify_tree_device(dc.q, dc.kv, case.kv_len, case.node_offsets, d_par, d_tok, dc.logits, out, d_len, d_acc)
    new_len = ver.compact_kv([B.kv_layer(k, v, dc.block_table, paged=True) for k, v in zip(layers_k, layers_v)], 2)
    torch.cuda.synchronize()
    a_ref, res = O.verify(case)
    assert d_len.cpu().tolist() == [r[0] for r in res] and max(r[0] for r in res) >= 3
    for b, (L, path, toks) in enumerate(res):
        assert d_acc[b, :L + 1].cpu().tolist() == toks.tolist()
        assert new_len[b] == case.kv_len[b] + L + 1
    import copy
    for (k0, v0), kg, vg in zip(before, layers_k, layers_v):
        c2 = copy.copy(case); c2.k, c2.v = k0, v0
        for b, (L, path, toks) in enumerate(res):
            O.compact(c2, k0, v0, b, path)
        assert np.array_equal(B.to_host(kg, "bf16"), k0) and np.array_equal(B.to_host(vg, "bf16"), v0)
    ver.close()


def test_error_paths_leave_outputs_alone():
    import torch
    case = W.custom_case(95, "f32", 1, 2, 2, 64, 50, [10], [W.chain_tree(5)])
    dc = B.DeviceCase(case)
    ver = B.Verifier(B.config_for_case(case))
    with pytest.raises(B.CbError) as e:
        ver.compact_kv([dc.kv], 1)
    assert e.value.code == B.CB_ESTATE
    bad = case.parent.copy(); bad[3] = 3
    with pytest.raises(B.CbError) as e:
        ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, bad, case.tokens, dc.logits)
    assert e.value.code == B.CB_ETREE
    with pytest.raises(B.CbError) as e:
        ver.verify_tree(dc.q, dc.kv, [10 + 100], case.node_offsets, case.parent, case.tokens, dc.logits)
    assert e.value.code == B.CB_ECAP
    ver.close()


@pytest.mark.parametrize("S", [700, 2048])
def test_hip_graph_replays_match_eager_steps(S):
    """The benchmark replays captured steps: every replay of verify + compact must leave exactly what
    the same steps leave when launched eagerly (compaction rewrites tree slots, so the state evolves).
    S = 2048 is the benchmark's own workload and launch configuration (device-resident tree, one-launch
    verification + compaction in a HIP graph); its first replay is also checked against the oracle."""
    import torch
    from oracle import cb_oracle as O
    case = W.make_config(2, S=S)
    cfg = B.config_for_case(case)
    results = {}
    for mode in ("eager", "graph"):
        dc = B.DeviceCase(case)
        ver = B.Verifier(cfg)
        d_par = torch.from_numpy(case.parent).cuda(); d_tok = torch.from_numpy(case.tokens).cuda()
        out = torch.zeros_like(dc.q)
        d_len = torch.zeros(1, dtype=torch.int32, device="cuda")
        d_acc = torch.zeros(1, case.max_depth + 1, dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        step = ver.bind_step(dc.q, dc.kv, case.kv_len, case.node_offsets, d_par, d_tok, dc.logits, out, d_len, d_acc,
                             [dc.kv], stream=side)
        snaps = []
        if mode == "graph":
            with torch.cuda.stream(side):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    step()
        for rep in range(3):
            with torch.cuda.stream(side):
                if mode == "graph":
                    graph.replay()
                else:
                    step()
            side.synchronize()
            # eager work of the program's own between the replays
            scratch = (dc.logits.float().sum() + out.float().abs().sum()).item()
            assert np.isfinite(scratch)
            snaps.append((B.to_host(out, "bf16").copy(), B.to_host(dc.k, "bf16").copy(), B.to_host(dc.v, "bf16").copy(),
                          d_len.cpu().numpy().copy(), d_acc.cpu().numpy().copy()))
        results[mode] = snaps
        ver.close()
    for rep in range(3):
        for a, b in zip(results["eager"][rep], results["graph"][rep]):
            assert np.array_equal(a, b), f"replay {rep} differs from the eager step"
    assert results["eager"][0][3][0] >= 0
    if S == 2048:
        out0, k0, v0, len0, acc0 = results["graph"][0]
        a_ref, res = O.verify(case)
        L, path, toks = res[0]
        assert len0[0] == L and acc0[0, :L + 1].tolist() == toks.tolist()
        rows = sample_rows(case, 64, seed=3)
        ref = O.attention_rows(case, rows)
        got = W.to_f64(out0, "bf16")
        check_attention(case, np.stack([got[case.node_offsets[b] + i, h] for b, h, i in rows]), ref, "graph replay, full size")
        k_ref, v_ref = case.k.copy(), case.v.copy()
        O.compact(case, k_ref, v_ref, 0, path)
        assert np.array_equal(k0, k_ref) and np.array_equal(v0, v_ref)


def test_one_graph_of_different_cases_through_one_workspace():
    """Three different verification steps -- different trees, prefix lengths, queries, logits -- captured
    back to back into one HIP graph through ONE context, so they share the workspace (split partials, merge
    and scan tickets, argmax partials), replayed three times with eager work between the replays.  Every
    step of every replay is checked against the oracle: a stale partial, or a ticket that one step left
    behind for the next, would show here.  The caches evolve (each step compacts its accepted path), and the
    oracle's copies evolve with them."""
    import copy
    import torch
    from oracle import cb_oracle as O
    rng = np.random.default_rng(41)
    cases = [W.make_config(2),
             W.custom_case(411, "bf16", 1, 32, 32, 128, 32000, [1500], [W.random_tree(rng, 40, 4, 6, False)[0]], p_match=0.8),
             W.custom_case(412, "bf16", 1, 32, 32, 128, 32000, [333], [W.random_tree(rng, 64, 3, 6, False)[0]], q_scale=2.0, p_match=0.7)]
    depth = max(c.max_depth for c in cases)
    cfg = B.make_config(32, 32, 128, "bf16", "bf16", 1, 64, depth, 32000)
    ver = B.Verifier(cfg)
    side = torch.cuda.Stream()
    dcs = [B.DeviceCase(c) for c in cases]
    pars = [torch.from_numpy(c.parent).cuda() for c in cases]
    toks = [torch.from_numpy(c.tokens).cuda() for c in cases]
    outs = [torch.zeros_like(dc.q) for dc in dcs]
    lens = [torch.zeros(1, dtype=torch.int32, device="cuda") for _ in cases]
    accs = [torch.zeros(1, depth + 1, dtype=torch.int32, device="cuda") for _ in cases]
    steps = [ver.bind_step(dc.q, dc.kv, c.kv_len, c.node_offsets, pars[i], toks[i], dc.logits, outs[i], lens[i], accs[i],
                           [dc.kv], stream=side) for i, (c, dc) in enumerate(zip(cases, dcs))]
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for st in steps:
                st()
    refs = [copy.copy(c) for c in cases]
    for r in refs:
        r.k, r.v = r.k.copy(), r.v.copy()
    for rep in range(3):
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        scratch = sum(float(o.float().abs().sum()) for o in outs)     # eager work of the program's own between replays
        assert np.isfinite(scratch)
        for i, (c, ref) in enumerate(zip(cases, refs)):
            print(f"[case] shared-workspace graph: replay {rep} step {i}", flush=True)
            a_ref, res = O.verify(ref)
            L, path, tk = res[0]
            assert int(lens[i].item()) == L, f"replay {rep} step {i}: accepted_len"
            assert accs[i][0, :L + 1].cpu().tolist() == tk.tolist(), f"replay {rep} step {i}: accepted tokens"
            check_attention(ref, W.to_f64(B.to_host(outs[i], "bf16"), "bf16"), O.attention(ref), f"replay {rep} step {i}")
            O.compact(ref, ref.k, ref.v, 0, path)
            assert np.array_equal(B.to_host(dcs[i].k, "bf16"), ref.k) and np.array_equal(B.to_host(dcs[i].v, "bf16"), ref.v), \
                f"replay {rep} step {i}: compacted cache"
    assert ver.device_status() & 3 == 0
    ver.close()


@pytest.mark.parametrize("shape", ["7b", "ragged", "odd_vocab", "single_nodes", "many_splits"])
def test_one_launch_verification_matches_separate_launches(shape):
    """Small calls run attention, logits scan and acceptance as one launch; the same call with that
    switched off uses three.  Both must give the oracle's results, and identical bits to each other."""
    import torch
    rng = np.random.default_rng(11)
    opts, rows = {}, None
    if shape == "7b":
        case = W.make_config(2)
        rows = sample_rows(case, 96)
    elif shape == "ragged":       # short sequences leave whole splits without keys: those workgroups only scan logits
        pars = [W.random_tree(rng, n, 4, 6, False)[0] for n in (64, 3, 33, 1)]
        case = W.custom_case(111, "bf16", 4, 8, 8, 128, 20000, [1500, 10, 400, 0], pars, paged=True)
        opts = {"splits": 12}     # 12 x 8 heads x 4 sequences workgroups for 101 rows x 3 chunks
    elif shape == "odd_vocab":    # rows that are not 16-byte aligned and a ragged last chunk
        case = W.custom_case(112, "bf16", 1, 16, 16, 128, 8193 + 6, [900], [W.random_tree(rng, 40, 4, 6, False)[0]])
        opts = {"splits": 6}
    elif shape == "many_splits":  # so many partials per tile that a separate merge kernel follows the launch
        case = W.custom_case(114, "bf16", 1, 8, 8, 128, 1000, [6000], [W.random_tree(rng, 64, 4, 6, False)[0]], q_scale=2.0)
        opts = {"splits": 24}
    else:
        case = W.custom_case(113, "bf16", 3, 32, 8, 128, 300, [2000, 1, 77], [[-1], [-1], [-1]])
    run_case(case, rows=rows, options=opts, what=f"one launch {shape}")
    run_case(case, rows=rows, options=dict(opts, fuse_logits=0), what=f"separate launches {shape}")
    dc = B.DeviceCase(case)
    got = []
    for fuse in (1, 0):
        ver = B.Verifier(B.config_for_case(case))
        for k, v in dict(opts, fuse_logits=fuse).items():
            ver.set_option(k, v)
        out, acc_len, acc_tok = ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent, case.tokens, dc.logits)
        torch.cuda.synchronize()
        assert ver.last_launch_info()["fused"] == bool(fuse), ver.last_launch_info()
        got.append((B.to_host(out, "bf16").copy(), acc_len.copy(), acc_tok.copy(), ver.get_argmax(case.total_nodes), ver.get_path(case.B)))
        ver.close()
    for x, y in zip(got[0], got[1]):
        assert np.array_equal(x, y)


def test_large_calls_keep_separate_launches():
    case = W.make_config(3, S=600)            # 128 nodes x 4 query heads per kv head: two row tiles per wave
    dc = B.DeviceCase(case)
    ver = B.Verifier(B.config_for_case(case))
    ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent, case.tokens, dc.logits)
    assert ver.last_launch_info()["fused"] is False and ver.last_launch_info()["impl"] == 2
    ver.close()


@pytest.mark.parametrize("kind", ["mfma", "scalar"])
def test_model_step_of_several_layers(kind):
    """cb_tree_attention_device for the lower layers, cb_verify_tree_device on the last, one cb_compact_kv
    over all layers: every layer's attention against the oracle, the acceptance, and every layer's cache."""
    import copy
    import torch
    from oracle import cb_oracle as O
    rng = np.random.default_rng(21)
    pars = [W.random_tree(rng, 40, 3, 6, False)[0], W.chain_tree(12)]
    if kind == "mfma":
        case = W.custom_case(121, "bf16", 2, 8, 4, 128, 700, [900, 130], pars, paged=True, p_match=0.8)
    else:
        case = W.custom_case(122, "f32", 2, 4, 2, 64, 700, [300, 50], pars, p_match=0.8)
    nl = 3
    layers = []
    for i in range(nl):
        c = copy.copy(case)
        if i:
            sub = W.custom_case(130 + i, case.dtype, 2, case.Hq, case.Hkv, case.D, 16, case.kv_len, pars, paged=case.block_size > 0)
            c.q, c.k, c.v = sub.q, sub.k, sub.v
            if case.block_size:
                assert sub.k.shape == case.k.shape
        layers.append(c)
    dcs = [B.DeviceCase(c) for c in layers]
    for dc in dcs[1:]:
        dc.block_table = dcs[0].block_table            # the layers share one geometry
    kvs = [B.kv_layer(dc.k, dc.v, dcs[0].block_table, paged=case.block_size > 0) for dc in dcs]
    for c in layers[1:]:
        c.block_table = case.block_table
    ver = B.Verifier(B.config_for_case(case))
    d_par = torch.from_numpy(case.parent).cuda(); d_tok = torch.from_numpy(case.tokens).cuda()
    outs = [torch.zeros_like(dc.q) for dc in dcs]
    d_len = torch.zeros(2, dtype=torch.int32, device="cuda")
    d_acc = torch.zeros(2, case.max_depth + 1, dtype=torch.int32, device="cuda")
    step = ver.bind_model_step([dc.q for dc in dcs], kvs, case.kv_len, case.node_offsets, d_par, d_tok, dcs[-1].logits,
                               outs, d_len, d_acc)
    # the same step captured as one HIP graph (what `bench.py --layers` replays) on copies of the caches:
    # after one replay it must have left exactly what the eager step leaves
    dcs2 = [B.DeviceCase(c) for c in layers]
    kvs2 = [B.kv_layer(dc.k, dc.v, dcs[0].block_table, paged=case.block_size > 0) for dc in dcs2]
    outs2 = [torch.zeros_like(dc.q) for dc in dcs2]
    d_len2 = torch.zeros(2, dtype=torch.int32, device="cuda")
    d_acc2 = torch.zeros(2, case.max_depth + 1, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    step2 = ver.bind_model_step([dc.q for dc in dcs2], kvs2, case.kv_len, case.node_offsets, d_par, d_tok, dcs2[-1].logits,
                                outs2, d_len2, d_acc2, stream=side)
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step2()
    step()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.replay()
    side.synchronize()
    assert torch.equal(d_len, d_len2) and torch.equal(d_acc, d_acc2)
    for o1, o2, a, b2 in zip(outs, outs2, dcs, dcs2):
        assert torch.equal(o1, o2) and torch.equal(a.k, b2.k) and torch.equal(a.v, b2.v), "graph replay of the model step differs from the eager step"
    assert ver.device_status() & 3 == 0
    a_ref, res = O.verify(layers[-1])
    assert d_len.cpu().tolist() == [r[0] for r in res]
    for b, (L, path, toks) in enumerate(res):
        assert d_acc[b, :L + 1].cpu().tolist() == toks.tolist()
    for c, dc, out in zip(layers, dcs, outs):
        got = W.to_f64(B.to_host(out, case.dtype), case.dtype)
        check_attention(c, got, O.attention(c), "model step layer")
        k_ref, v_ref = c.k.copy(), c.v.copy()
        for b, (L, path, toks) in enumerate(res):
            O.compact(c, k_ref, v_ref, b, path)
        assert np.array_equal(B.to_host(dc.k, case.dtype), k_ref) and np.array_equal(B.to_host(dc.v, case.dtype), v_ref)
    ver.close()


@pytest.mark.parametrize("qkv,lg", [("bf16", "f32"), ("f32", "bf16")])
def test_logits_dtype_independent_of_the_cache_dtype(qkv, lg):
    """The configuration names the two element types separately; acceptance must be bit-exact for either mix."""
    import torch
    from oracle import cb_oracle as O
    rng = np.random.default_rng(31)
    par = W.random_tree(rng, 50, 4, 6, False)[0]
    case = W.custom_case(141, qkv, 1, 8, 8, 128, 9001, [800], [par], p_match=0.8)
    other = W.custom_case(142, lg, 1, 8, 8, 128, 9001, [800], [par], p_match=0.8)      # logits and tokens of the other type
    dc = B.DeviceCase(case)
    d_logits = B.to_device(other.logits, lg)
    cfg = B.make_config(8, 8, 128, qkv, lg, 1, 50, case.max_depth, 9001)
    ver = B.Verifier(cfg)
    out, acc_len, acc_tok = ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent, other.tokens, d_logits)
    torch.cuda.synchronize()
    a = O.argmax(other.logits, lg)
    assert np.array_equal(ver.get_argmax(50), a)
    L, path, toks = O.accept(case.parent, other.tokens, a)
    assert acc_len[0] == L and acc_tok[0, :L + 1].tolist() == toks.tolist() and L >= 1
    check_attention(case, W.to_f64(B.to_host(out, qkv), qkv), O.attention(case), f"qkv {qkv} logits {lg}")
    ver.close()
