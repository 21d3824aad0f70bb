"""The host-array form returns when the acceptance results have arrived, possibly before its launch
has ended.  These tests call it back to back without any synchronisation in between -- different trees
through one context, on one stream and on alternating streams, one launch and separate launches, one
sequence and several -- and compare every call's results with the CPU oracle; the attention output is
checked after a stream synchronisation."""
import numpy as np
import pytest

from oracle import cb_oracle as O
from paper_2511_21699_amd import binding as B
from paper_2511_21699_amd import workloads as W
from tests.gpu_harness import check_attention

pytestmark = pytest.mark.gpu


def _cases(multi: bool):
    if multi:   # several sequences per call: one arrival flag per sequence
        mk = lambda s: W.make_config(4, seed_offset=s, B=5, S=(300, 900), V=4096)
    else:
        mk = lambda s: W.make_config(2, seed_offset=s, S=1500, V=8192)
    return [mk(s) for s in range(3)]


def _expected(case):
    _, res = O.verify(case)
    return res


@pytest.mark.parametrize("options", [{}, {"full_sync": 1}, {"fuse_logits": 0}, {"attn_impl": 1}])
@pytest.mark.parametrize("multi", [False, True])
def test_back_to_back_host_calls_return_the_oracles_results(multi, options):
    import torch
    cases = _cases(multi)
    dcs = [B.DeviceCase(c) for c in cases]
    want = [_expected(c) for c in cases]
    c0 = cases[0]
    stride = max(c.max_depth for c in cases) + 1
    cfg = B.make_config(c0.Hq, c0.Hkv, c0.D, c0.dtype, c0.dtype, max(c.B for c in cases),
                        int(max(np.diff(c.node_offsets).max() for c in cases)), stride - 1, c0.V, c0.block_size)
    ver = B.Verifier(cfg)
    for k, v in options.items():
        ver.set_option(k, v)
    outs = [torch.zeros_like(dc.q) for dc in dcs]
    try:
        for it in range(30):
            j = (it * 2 + it // 3) % len(cases)           # an irregular order, repeats included
            print(f"[host form] multi={multi} options={options} call {it} case {j}", flush=True)
            case, dc = cases[j], dcs[j]
            _, acc_len, acc_tok = ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent, case.tokens,
                                                  dc.logits, attn_out=outs[j])
            for b, (L, path, toks) in enumerate(want[j]):
                assert acc_len[b] == L, f"call {it}: accepted_len[{b}] {acc_len[b]} != {L}"
                assert acc_tok[b, :L + 1].tolist() == toks.tolist() and (acc_tok[b, L + 1:] == -1).all()
        torch.cuda.synchronize()
        for j, case in enumerate(cases):
            got = W.to_f64(B.to_host(outs[j], case.dtype), case.dtype)
            check_attention(case, got, O.attention(case, threads=16), f"case {j}")
        assert ver.device_status() & 3 == 0
    finally:
        ver.close()


def test_alternating_streams_are_ordered_by_the_library():
    import torch
    cases = _cases(False)
    dcs = [B.DeviceCase(c) for c in cases]
    want = [_expected(c) for c in cases]
    c0 = cases[0]
    cfg = B.make_config(c0.Hq, c0.Hkv, c0.D, c0.dtype, c0.dtype, 1, int(np.diff(c0.node_offsets).max()),
                        max(c.max_depth for c in cases), c0.V)
    ver = B.Verifier(cfg)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]       # default priority
    outs = [torch.zeros_like(dc.q) for dc in dcs]
    torch.cuda.synchronize()
    try:
        for it in range(24):
            j = it % len(cases)
            print(f"[host form] streams: call {it} case {j} stream {it % 2}", flush=True)
            case, dc = cases[j], dcs[j]
            _, acc_len, acc_tok = ver.verify_tree(dc.q, dc.kv, case.kv_len, case.node_offsets, case.parent, case.tokens,
                                                  dc.logits, attn_out=outs[j], stream=streams[it % 2])
            L, path, toks = want[j][0]
            assert acc_len[0] == L and acc_tok[0, :L + 1].tolist() == toks.tolist()
        torch.cuda.synchronize()
        for j, case in enumerate(cases):
            got = W.to_f64(B.to_host(outs[j], case.dtype), case.dtype)
            check_attention(case, got, O.attention(case, threads=16), f"case {j}")
    finally:
        ver.close()
