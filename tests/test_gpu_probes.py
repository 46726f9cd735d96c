"""The measurement aids of the C ABI (plain read stream, exponential rate, block-scoring instruction mix) run,
return, and leave their sinks alone (they store only on a value that cannot occur)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probes_run_and_leave_their_sinks_alone():
    from paper_2601_18383_amd import binding as B
    dev = torch.device("cuda:0")
    sink_u = torch.zeros(4, dtype=torch.int32, device=dev)
    sink_f = torch.zeros(4, dtype=torch.float32, device=dev)
    buf = torch.arange(1 << 20, dtype=torch.int32, device=dev)
    B.dynts_probe_read_stream(buf, 256, sink_u, magic=0x12345678)
    B.dynts_probe_exp_rate(64, 10, sink_f)
    for what in (1, 2, 3):
        B.dynts_probe_issue_mix(64, 10, what, sink_f)
    torch.cuda.synchronize()
    assert int(sink_u.abs().sum()) == 0
    assert float(sink_f.abs().sum()) == 0.0
