"""Seeded random shapes through the whole path against the oracle: head counts and groupings, node
counts on both sides of the 64/128/256-row tile limits, prefix lengths around stage and split
boundaries, contiguous and paged caches in both layouts, forced split counts, vocabularies that are
not multiples of a vector or a chunk."""
import numpy as np
import pytest

from paper_2511_21699_amd import binding as B
from paper_2511_21699_amd import workloads as W
from tests.gpu_harness import run_case

pytestmark = pytest.mark.gpu


def _case(seed: int):
    rng = np.random.default_rng(9000 + seed)
    bf16 = rng.random() < 0.8
    dtype = "bf16" if bf16 else "f32"
    D = 128 if (bf16 and rng.random() < 0.85) else int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    g = int(rng.choice([1, 1, 2, 4, 7]))
    Bn = int(rng.choice([1, 1, 2, 3, 5]))
    lim = int(rng.choice([1, 8, 16, 17, 33, 64, 65, 100, 128, 129, 200, 256])) // (g if rng.random() < 0.5 else 1)
    lim = max(1, min(256, lim))
    ns = [int(rng.integers(max(1, lim // 2), lim + 1)) for _ in range(Bn)]
    ns[0] = lim
    pars = []
    for n in ns:
        kind = rng.random()
        if kind < 0.15:
            pars.append(W.chain_tree(n))
        elif kind < 0.3:
            pars.append(W.star_tree(n))
        else:
            mc, md = int(rng.integers(1, 6)), int(rng.integers(1, 12))
            if mc == 1 and md < n - 1 or mc > 1 and (mc ** (md + 1) - 1) // (mc - 1) < n:
                mc, md = 4, 12                           # (the draw could not hold n nodes)
            pars.append(W.random_tree(rng, n, mc, md, False)[0])
    edges = [0, 1, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257, 500, 777, 1024, 1500, 2100, 3001]
    kv = [int(rng.choice(edges)) + int(rng.integers(0, 3)) * int(rng.integers(0, 40)) for _ in range(Bn)]
    V = int(rng.choice([1, 7, 100, 1000, 8191, 8192, 8193, 20000]))
    paged = rng.random() < 0.4
    case = W.custom_case(9100 + seed, dtype, Bn, Hkv * g, Hkv, D, V, kv, pars, paged=paged,
                         q_scale=float(rng.choice([1.0, 3.0])), p_match=float(rng.choice([0.3, 0.7, 0.95])))
    opts = {}
    if rng.random() < 0.4:
        opts["splits"] = int(rng.choice([1, 2, 3, 7, 16, 30]))
    layout = B.CB_LAYOUT_HEAD_MAJOR if rng.random() < 0.3 else B.CB_LAYOUT_TOKEN_MAJOR
    return case, opts, layout


@pytest.mark.parametrize("seed", range(48))
def test_random_shape_matches_the_oracle(seed):
    case, opts, layout = _case(seed)
    run_case(case, options=opts, layout=layout, what=f"fuzz {seed}")
