"""The benchmark's yardstick kernel (cb_probe_stream_read: a bare streaming read) runs and checks its arguments."""
import pytest

pytestmark = pytest.mark.gpu


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
