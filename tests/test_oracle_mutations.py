"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a
dropped term, an off-by-one, a swapped operand, a wrong tie rule ...), builds it, and checks that the
pin battery of test_oracle_pins fails on it.  The mistakes live in the copy only, on the CPU."""
import os
import subprocess

import pytest

from oracle import cb_oracle as O
from tests import test_oracle_pins as P

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "cb_oracle.c")

MUTATIONS = {
    "node does not see itself": ("for (int a = i, steps = 0;", "for (int a = par[i], steps = 0;"),
    "softmax scale dropped": ("      s *= scale;\n", ""),
    "kv head by modulo instead of group": ("int hk = h / g;", "int hk = h % Hkv;"),
    "values read from K": ("o[d] += w[t] * load_elem(v, dtype, vo + d);", "o[d] += w[t] * load_elem(k, dtype, vo + d);"),
    "no normalisation": ("for (int d = 0; d < D; d++) o[d] /= denom;", ""),
    "last prefix key missing": ("for (int j = 0; j < S; j++) vis[nvis++] = j;", "for (int j = 0; j + 1 < S; j++) vis[nvis++] = j;"),
    "query row of the wrong head": ("* Hq + h) * (int64_t)D;", "* Hq + (Hq - 1 - h)) * (int64_t)D;"),
    "argmax keeps the last maximum": ("if (x > best) { best = x; arg = (int32_t)t; }", "if (x >= best) { best = x; arg = (int32_t)t; }"),
    "argmax skips element zero tie": ("double best = load_elem(logits, dtype, base);", "double best = load_elem(logits, dtype, base) - 1e-30;"),
    "token compared with the node's own argmax": ("if (tok[x] != a[parent[x]]) ok = 0;", "if (tok[x] != a[x]) ok = 0;"),
    "later node wins equal depth": ("if (ok && depth > best_depth)", "if (ok && depth >= best_depth)"),
    "emits draft tokens instead of generated ones": ("tokens[j] = a[path[j]];", "tokens[j] = tok[path[j]];"),
    "only the direct parent is checked": ("for (int x = c; parent[x] >= 0; x = parent[x]) {\n      if (tok[x] != a[parent[x]]) ok = 0;\n      depth++;",
                                           "for (int x = c; parent[x] >= 0; x = parent[x]) {\n      if (x == c && tok[x] != a[parent[x]]) ok = 0;\n      depth++;"),
    "compaction destination off by one": ("int64_t dst = slot_index(seq, (int64_t)S + j,", "int64_t dst = slot_index(seq, (int64_t)S + j - 1,"),
    "compaction copies slot j instead of path[j]": ("int64_t src = slot_index(seq, (int64_t)S + path[j],", "int64_t src = slot_index(seq, (int64_t)S + j,"),
    "paged slot offset wrong": ("return ((blk * block_size + slot % block_size) * Hkv + h)", "return ((blk * block_size + (slot + 1) % block_size) * Hkv + h)"),
    "bf16 widened with the wrong shift": ("((const uint16_t *)base)[idx]) << 16;", "((const uint16_t *)base)[idx]) << 15;"),
}


def battery():
    """A compact run over the pins (same functions pytest collects, fixed parameters)."""
    P.test_tree_attention_equals_causal_attention_along_each_path("f32", False, 1)
    P.test_tree_attention_equals_causal_attention_along_each_path("bf16", True, 2)
    P.test_chain_tree_is_library_causal_attention(6, 2)
    P.test_star_tree_is_independent_single_token_decodes()
    P.test_equal_keys_give_mean_of_visible_values()
    P.test_values_all_one_give_output_one()
    P.test_softmax_scale_is_applied_to_scores()
    P.test_argmax_matches_numpy_first_occurrence("bf16")
    P.test_argmax_constructed_ties_zero_signs_and_constant_rows()
    P.test_paper_figure2_example()
    for seed in range(40):
        P.test_acceptance_equals_sequential_greedy_walk(seed)
    P.test_acceptance_is_lossless_against_token_by_token_decoding()
    P.test_compaction_moves_the_accepted_rows(False)
    P.test_compaction_moves_the_accepted_rows(True)
    P.test_compaction_source_slot_that_is_also_a_destination()


def test_battery_passes_on_the_real_oracle():
    battery()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"the oracle source changed: '{old}' should occur exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", str(so), str(src), "-lm"], check=True)
    monkeypatch.setattr(O, "_lib", O.load_library(str(so)))
    with pytest.raises(AssertionError):
        battery()
