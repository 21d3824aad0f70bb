"""Pins for the CPU oracle: each oracle function is checked against something that is not the
oracle -- brute force, a library routine on a special case, a closed form, or the paper's worked
example (tests/golden/fig2_example.json)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import cb_oracle as O
from paper_2511_21699_amd import workloads as W
from tests import helpers as H

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_case(seed, dtype="f32", paged=False, Hq=4, Hkv=2, D=16, B=2, q_scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    parents = [W.random_tree(rng, int(rng.integers(3, 12)), 3, 4, False)[0] for _ in range(B)]
    kv_len = rng.integers(0, 40, size=B)
    return W.custom_case(seed, dtype, B, Hq, Hkv, D, 50, kv_len, parents, paged=paged, q_scale=q_scale)


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_tree_attention_equals_causal_attention_along_each_path(dtype, paged, seed):
    case = small_case(seed, dtype, paged, q_scale=3.0)
    want = H.per_path_attention(case)
    got = O.attention(case)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_tiny_config_against_brute_force():
    case = W.make_config(1, S=40)
    np.testing.assert_allclose(O.attention(case), H.per_path_attention(case), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (6, 2)])
def test_chain_tree_is_library_causal_attention(Hq, Hkv):
    S, N, D = 37, 9, 32
    case = W.custom_case(11, "f32", 1, Hq, Hkv, D, 20, [S], [W.chain_tree(N)], q_scale=2.0)
    got = O.attention(case)
    k = torch.from_numpy(case.k[0, :S + N].astype(np.float64)).permute(1, 0, 2)          # [Hkv, T, D]
    v = torch.from_numpy(case.v[0, :S + N].astype(np.float64)).permute(1, 0, 2)
    k = k.repeat_interleave(Hq // Hkv, dim=0)
    v = v.repeat_interleave(Hq // Hkv, dim=0)
    q = torch.zeros(Hq, S + N, D, dtype=torch.float64)
    q[:, S:] = torch.from_numpy(case.q.astype(np.float64)).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
    np.testing.assert_allclose(got, ref[:, S:].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_star_tree_is_independent_single_token_decodes():
    S, N, D, H = 20, 6, 16, 2
    case = W.custom_case(12, "f32", 1, H, H, D, 20, [S], [W.star_tree(N)], q_scale=2.0)
    got = O.attention(case)
    for i in range(N):
        slots = list(range(S)) + ([S] if i == 0 else [S, S + i])
        for h in range(H):
            k = torch.from_numpy(H_rows(case, "k", slots, h))
            v = torch.from_numpy(H_rows(case, "v", slots, h))
            q = torch.from_numpy(case.q[i, h].astype(np.float64))[None]
            ref = torch.nn.functional.scaled_dot_product_attention(q[None, None], k[None, None], v[None, None])[0, 0, 0]
            np.testing.assert_allclose(got[i, h], ref.numpy(), rtol=1e-10, atol=1e-12)


def H_rows(case, which, slots, h):
    return H.slot_rows(case, which, 0, slots, h)


def test_values_all_one_give_output_one():
    case = small_case(5)
    case.v[...] = 1.0
    np.testing.assert_allclose(O.attention(case), 1.0, rtol=0, atol=1e-15)


def test_equal_keys_give_mean_of_visible_values():
    case = small_case(6, B=1)
    case.k[...] = case.k[0, 0, 0][None, None, None, :]
    got = O.attention(case)
    S = int(case.kv_len[0])
    for i in range(len(case.parent)):
        anc, x = [], i
        while x >= 0:
            anc.append(x); x = int(case.parent[x])
        slots = list(range(S)) + [S + a for a in anc]
        for h in range(case.Hq):
            mean = H.slot_rows(case, "v", 0, slots, h // (case.Hq // case.Hkv)).mean(axis=0)
            np.testing.assert_allclose(got[i, h], mean, rtol=1e-12, atol=1e-14)


def test_non_ancestor_nodes_do_not_leak():
    case = small_case(7, B=1, q_scale=2.0)
    base = O.attention(case)
    S = int(case.kv_len[0])
    n = len(case.parent)
    for i in range(n):
        anc, x = set(), i
        while x >= 0:
            anc.add(x); x = int(case.parent[x])
        other = [a for a in range(n) if a not in anc]
        if not other:
            continue
        k2, v2 = case.k.copy(), case.v.copy()
        for a in other:
            k2[0, S + a] += 100.0
            v2[0, S + a] -= 50.0
        kk, vv = case.k, case.v
        case.k, case.v = k2, v2
        rows = np.array([(0, h, i) for h in range(case.Hq)], dtype=np.int32)
        got = O.attention_rows(case, rows)
        case.k, case.v = kk, vv
        assert np.array_equal(got, base[i])              # bit-identical: masked keys never enter
    # and an ancestor *does* matter
    k2 = case.k.copy(); k2[0, S] += 1.0
    case.k = k2
    assert not np.array_equal(O.attention(case)[n - 1], base[n - 1])


def test_block_shuffle_leaves_output_unchanged():
    case = small_case(8, paged=True)
    base = O.attention(case)
    rng = np.random.default_rng(0)
    nb = case.k.shape[0]
    perm = rng.permutation(nb)                           # new physical id of old block j is perm[j]
    k2, v2 = np.empty_like(case.k), np.empty_like(case.v)
    k2[perm], v2[perm] = case.k, case.v
    bt = case.block_table.copy()
    bt[bt >= 0] = perm[bt[bt >= 0]]
    case.k, case.v, case.block_table = k2, v2, bt
    assert np.array_equal(O.attention(case), base)


def test_gqa_equals_mha_with_repeated_kv_heads():
    case = small_case(9, Hq=6, Hkv=2)
    base = O.attention(case)
    case.k = np.repeat(case.k, 3, axis=2)
    case.v = np.repeat(case.v, 3, axis=2)
    case.Hkv = 6
    assert np.array_equal(O.attention(case), base)


def test_softmax_scale_is_applied_to_scores():
    case = small_case(10, B=1)
    a = O.attention(case, scale=0.5)
    case.q = (case.q * np.float32(2.0)).astype(np.float32)   # exact doubling
    b = O.attention(case, scale=0.25)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=0)
    # scale 0 => uniform weights over the visible keys
    c = O.attention(case, scale=0.0)
    S = int(case.kv_len[0])
    mean_root = H.slot_rows(case, "v", 0, list(range(S + 1)), 0).mean(axis=0)
    np.testing.assert_allclose(c[0, 0], mean_root, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ argmax
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_argmax_matches_numpy_first_occurrence(dtype):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((40, 5000), dtype=np.float32)
    x[20:] = np.round(x[20:] * 2) / 2                     # coarse values: the maximum repeats within a row
    lg = W.f32_to_bf16_bits(x) if dtype == "bf16" else x
    vals = W.bf16_bits_to_f32(lg) if dtype == "bf16" else lg
    got = O.argmax(lg, dtype)
    assert np.array_equal(got, np.argmax(vals, axis=1))
    ties = (vals == vals.max(axis=1, keepdims=True)).sum(axis=1)
    assert (ties[20:] > 1).any()


def test_argmax_constructed_ties_zero_signs_and_constant_rows():
    V = 1000
    x = np.full((6, V), -1.0, dtype=np.float32)
    x[0, [17, 400]] = 3.0            # two equal maxima -> the first
    x[1, [0, V - 1]] = 3.0           # first and last element
    x[2, V - 1] = 3.0                # only the last
    x[3, :] = -0.0; x[3, 5] = 0.0    # -0 and +0 compare equal -> index 0
    x[4, :] = 2.5                    # constant row -> 0
    x[5, 63] = 3.0; x[5, 64] = 3.0   # across a 64-lane boundary
    for dtype, lg in (("f32", x), ("bf16", W.f32_to_bf16_bits(x))):
        assert O.argmax(lg, dtype).tolist() == [17, 0, V - 1, 0, 0, 63]


def test_argmax_negative_values_in_bf16():
    x = -np.abs(np.random.default_rng(4).standard_normal((3, 777), dtype=np.float32)) - 1.0
    lg = W.f32_to_bf16_bits(x)
    assert np.array_equal(O.argmax(lg, "bf16"), np.argmax(W.bf16_bits_to_f32(lg), axis=1))


# ------------------------------------------------------------------ acceptance
def test_paper_figure2_example():
    with open(os.path.join(GOLDEN, "fig2_example.json")) as f:
        g = json.load(f)
    voc = g["vocab"]
    tok = [voc[w] for w in g["tree_tokens"]]
    a = [voc[g["generated_at_node"][w]] for w in g["tree_tokens"]]
    L, path, emitted = O.accept(g["tree_parent"], tok, a)
    assert L == g["expected_accepted_len"]
    assert path.tolist() == g["expected_path"]
    assert emitted.tolist() == [voc[w] for w in g["expected_tokens"]]


@pytest.mark.parametrize("seed", range(40))
def test_acceptance_equals_sequential_greedy_walk(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    parent, depth = W.random_tree(rng, n, 3, 6, False)
    V = 2 if seed % 2 else 4                               # tiny vocabularies: many matches; with 2 tokens siblings
                                                           # often carry the same one, so equal-depth ties occur
    tok = rng.integers(0, V, size=n)
    a = rng.integers(0, V, size=n)
    L, path, emitted = O.accept(parent, tok, a)
    L2, path2, emitted2 = H.sequential_greedy_accept(parent, tok, a)
    assert (L, path.tolist(), emitted.tolist()) == (L2, path2, emitted2)
    assert 0 <= L <= depth.max() and len(emitted) == L + 1    # 1 .. 1 + longest branch tokens per step
    assert path[0] == 0 and all(parent[path[j]] == path[j - 1] for j in range(1, L + 1))


def test_acceptance_is_lossless_against_token_by_token_decoding():
    """With a model whose next token is a function of the whole token sequence, the tokens emitted
    by verification equal plain greedy decoding of the same model, whatever the tree drafts."""
    def next_token(seq):
        return (sum((i + 1) * t for i, t in enumerate(seq)) * 2654435761 >> 7) % 5

    rng = np.random.default_rng(1)
    for trial in range(30):
        context = rng.integers(0, 5, size=6).tolist()
        n = int(rng.integers(2, 30))
        parent, _ = W.random_tree(rng, n, 4, 5, False)
        tok = rng.integers(0, 5, size=n)
        tok[0] = context[-1]
        a = np.empty(n, dtype=np.int64)
        for i in range(n):
            chain, x = [], i
            while x > 0:
                chain.append(int(tok[x])); x = int(parent[x])
            a[i] = next_token(context + chain[::-1])
        L, path, emitted = O.accept(parent, tok, a)
        seq = list(context)
        for t in emitted:
            assert t == next_token(seq)
            seq.append(int(t))


def test_single_node_tree_accepts_nothing_and_emits_one_token():
    L, path, emitted = O.accept([-1], [7], [3])
    assert (L, path.tolist(), emitted.tolist()) == (0, [0], [3])


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("paged", [False, True])
def test_compaction_moves_the_accepted_rows(paged):
    parent = W.chain_tree(40) if paged else np.array([-1, 0, 0, 1, 2, 2], dtype=np.int32)
    case = W.custom_case(21, "bf16", 1, 2, 2, 8, 10, [29], [parent], paged=paged)
    path = [0, 2, 5] if not paged else [0] + list(range(3, 40, 2))    # paged: long path across 16-token blocks
    S = int(case.kv_len[0])
    before_k = {a: H.slot_rows(case, "k", 0, [S + a], 1)[0] for a in path}
    before_v = {a: H.slot_rows(case, "v", 0, [S + a], 0)[0] for a in path}
    prefix_k = H.slot_rows(case, "k", 0, list(range(S + 1)), 0).copy()
    k, v = case.k.copy(), case.v.copy()
    new_len = O.compact(case, k, v, 0, path)
    assert new_len == S + len(path)
    case.k, case.v = k, v
    for j, a in enumerate(path):
        assert np.array_equal(H.slot_rows(case, "k", 0, [S + j], 1)[0], before_k[a])
        assert np.array_equal(H.slot_rows(case, "v", 0, [S + j], 0)[0], before_v[a])
    assert np.array_equal(H.slot_rows(case, "k", 0, list(range(S + 1)), 0), prefix_k)   # prefix and root untouched


def test_compaction_of_an_already_compact_path_changes_nothing():
    case = W.custom_case(22, "f32", 1, 2, 2, 8, 10, [5], [W.chain_tree(6)])
    k, v = case.k.copy(), case.v.copy()
    O.compact(case, k, v, 0, [0, 1, 2, 3])
    assert np.array_equal(k, case.k) and np.array_equal(v, case.v)


def test_compaction_source_slot_that_is_also_a_destination():
    # path [0,2,5]: slot S+2 is the source of step 1 and the destination of step 2
    case = W.custom_case(23, "f32", 1, 1, 1, 4, 10, [3], [np.array([-1, 0, 0, 1, 2, 2], dtype=np.int32)])
    k0 = case.k.copy()
    k, v = case.k.copy(), case.v.copy()
    O.compact(case, k, v, 0, [0, 2, 5])
    assert np.array_equal(k[0, 4], k0[0, 5]) and np.array_equal(k[0, 5], k0[0, 8])
