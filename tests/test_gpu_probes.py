"""The measurement aids of the library run and do what their description says (needs the GPU)."""
import pytest
import torch

import paper_2604_17709_amd as dn

pytestmark = pytest.mark.gpu


def test_mfma_probe_counts_its_products():
    ones = torch.ones(4096, dtype=torch.bfloat16, device="cuda")          # 8192 bytes of 1.0
    sink = torch.zeros(dn.PROBE_SINK_BYTES // 4, dtype=torch.float32, device="cuda")
    n = 10
    flops = dn.deinfer_probe_mfma_bf16(ones, n, sink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == 2.0 * 32 * 32 * 16 * 8 * n * 4 * cus
    # every element of every accumulator block is 16 * n; a lane sums 8 blocks x 16 elements
    got = sink[: cus * 256]
    assert torch.all(got == 8 * 16 * 16.0 * n)
    assert torch.all(sink[cus * 256:] == 0)


def test_stream_read_probe_leaves_its_input_alone():
    buf = torch.randint(0, 256, (8 << 20,), dtype=torch.uint8, device="cuda")
    ref = buf.clone()
    sink = torch.zeros(dn.PROBE_SINK_BYTES, dtype=torch.uint8, device="cuda")
    dn.deinfer_probe_stream_read(buf, buf.numel(), sink)
    dn.deinfer_probe_stream_read(buf[4096:], 1024, sink)                 # one piece, one workgroup
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)
    with pytest.raises(dn.DeinferError):
        dn.deinfer_probe_stream_read(buf, 1000, sink)
