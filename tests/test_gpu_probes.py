"""The ceiling probes of include/qqq_tuning.h run to completion on small inputs and reject what they
document as unsupported.  They compute nothing that is checked: what they are for is their duration,
which bench.py --ceilings reads; this test keeps them launchable."""
import pytest
import torch

from paper_2406_09904_amd import binding as qqq

pytestmark = pytest.mark.gpu


def test_stream_read_and_mfma_probes_launch():
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    buf = torch.ones((1 << 20,), dtype=torch.uint8, device="cuda")
    qqq.probe_stream_read(buf, 1 << 20, 64, sink)
    a = torch.randint(-8, 8, (4 * 4 * 512 * 16,), dtype=torch.int8, device="cuda")
    b = torch.randint(-8, 8, (2 * 2 * 512 * 16,), dtype=torch.int8, device="cuda")
    qqq.probe_mfma_i8(a, b, 4, 8, sink)
    torch.cuda.synchronize()
    assert int(sink[0].item()) == 0


@pytest.mark.parametrize("parts", [0, 4, 1, 5, 6, 8, 7, 15, 16, 31])
def test_prefill_loop_probe_launches_every_supported_combination(parts):
    wgs, region = 4, 2 * qqq.PROBE_LOOP_STAGE
    src = torch.randint(0, 256, (wgs * region,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    qqq.probe_prefill_loop(src, region, 5, parts, wgs, sink)
    torch.cuda.synchronize()
    assert int(sink[0].item()) == 0


def test_prefill_loop_probe_rejects_unsupported_arguments():
    src = torch.zeros((2 * qqq.PROBE_LOOP_STAGE,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    with pytest.raises(qqq.QQQError):
        qqq.probe_prefill_loop(src, 2 * qqq.PROBE_LOOP_STAGE, 5, 2, 1, sink)       # W_READS without CONVERT
    with pytest.raises(qqq.QQQError):
        qqq.probe_prefill_loop(src, qqq.PROBE_LOOP_STAGE + 16, 5, 0, 1, sink)      # region not a stage multiple
    with pytest.raises(qqq.QQQError):
        qqq.probe_prefill_loop(src, 2 * qqq.PROBE_LOOP_STAGE, 0, 0, 1, sink)       # no steps
    with pytest.raises(ValueError):
        qqq.probe_prefill_loop(src, 2 * qqq.PROBE_LOOP_STAGE, 5, 0, 2, sink)       # src too small for 2 workgroups
