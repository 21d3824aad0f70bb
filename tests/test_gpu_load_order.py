"""The MFMA attention kernel covers register loads and LDS-DMA loads with counted vmcnt waits of its
own, which is only right if the two kinds are counted off in the order they were requested.  The
library's probe (cb_probe_load_order, cacheback.h) checks that on the device the tests run on."""
import pytest

pytestmark = pytest.mark.gpu


def test_loads_are_counted_off_in_request_order():
    import torch
    from paper_2511_21699_amd import binding as B
    workgroups, iters = 512, 32
    n = workgroups * iters * 4096 + 256
    i = torch.arange(n, dtype=torch.int64, device="cuda")
    cold = ((i * 2654435761 + 12345) & 0xFFFFFFFF).to(torch.int64)
    cold = torch.where(cold >= 2 ** 31, cold - 2 ** 32, cold).to(torch.int32)   # the same 32 bits, as int32
    del i
    hot = torch.zeros(1024, dtype=torch.int32, device="cuda")
    res = torch.zeros(8, dtype=torch.int32, device="cuda")
    for _ in range(3):
        B.probe_load_order(cold, hot, workgroups, iters, res)
    torch.cuda.synchronize()
    r = res.cpu().tolist()
    reads = 3 * workgroups * iters * 64
    assert r[1] == 0 and r[3] == 0 and r[5] == 0, f"values wrong even after a full wait: {r}"
    assert r[0] == 0, f"a register load was not back although only younger LDS-DMA requests could be in flight: {r[0]} of {reads}"
    assert r[2] == 0, f"an LDS-DMA load was not back although only younger register loads could be in flight: {r[2]} of {reads}"
    assert r[4] > reads // 2, f"the control (no wait) saw the loaded value {reads - r[4]} times of {reads}: the probe cannot tell"


def test_probe_rejects_short_buffers():
    import torch
    from paper_2511_21699_amd import binding as B
    cold = torch.zeros(4096, dtype=torch.int32, device="cuda")
    hot = torch.zeros(1024, dtype=torch.int32, device="cuda")
    res = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.CbError):
        B.probe_load_order(cold, hot, 2, 2, res)
    with pytest.raises(B.CbError):
        B.probe_load_order(torch.zeros(2 * 2 * 4096 + 256, dtype=torch.int32, device="cuda"), hot[:100], 2, 2, res)


def test_stream_read_probe_runs_and_checks_its_arguments():
    import torch
    from paper_2511_21699_amd import binding as B
    buf = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    sink = torch.zeros(256, dtype=torch.int32, device="cuda")
    B.probe_stream_read(buf, buf.numel() * 4, sink)
    B.probe_stream_read(buf, 4096 + 16, sink)             # a ragged number of 16-byte pieces per thread
    torch.cuda.synchronize()
    with pytest.raises(B.CbError):
        B.probe_stream_read(buf, 100, sink)                # not a multiple of 16
    with pytest.raises(B.CbError):
        B.probe_stream_read(buf[1:], 1024, sink)           # not 16-byte aligned
