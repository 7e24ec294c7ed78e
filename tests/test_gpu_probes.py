"""The library's two benchmark diagnostics: the bandwidth probe leaves memory as documented and the
clock probe ends by itself with plausible counts."""
import numpy as np
import pytest

import paper_2605_11744_amd as sa

pytestmark = pytest.mark.gpu


def test_bandwidth_probe_modes_touch_memory_as_documented():
    import torch
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")        # 4 MiB + a ragged tail below
    ref = buf.clone()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    nbytes = buf.numel() * 4 - 48                                        # not a multiple of a workgroup's span
    sa.segattn_bandwidth_probe(buf, nbytes, 0, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)                                         # a read changes nothing
    sa.segattn_bandwidth_probe(buf, nbytes, 1, sink)
    torch.cuda.synchronize()
    flipped = (ref.view(torch.int32).cpu().numpy().view(np.uint32) ^ np.uint32(0x80008000))
    got = buf.cpu().numpy().view(np.uint32)
    pieces = nbytes // 16
    want = ref.cpu().numpy().view(np.uint32).copy()
    want[0:4 * pieces:4] = flipped[0:4 * pieces:4]                       # first dword of every 16-byte piece
    assert np.array_equal(got, want)
    sa.segattn_bandwidth_probe(buf, nbytes, 1, sink)                     # a second pass restores the buffer
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)


def test_clock_probe_ends_by_itself_and_reports_a_plausible_clock():
    import torch
    counts = torch.zeros(2 * sa.SEGATTN_CLOCK_PROBE_WAVES, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    khz = sa.segattn_clock_probe(2000, counts)                           # two milliseconds
    torch.cuda.synchronize()
    c = counts.cpu().numpy().reshape(-1, 2)
    assert khz > 0
    want_ticks = 2000 * khz // 1000
    assert (c[:, 1] >= want_ticks).all() and (c[:, 1] < 2 * want_ticks).all()
    mhz = c[:, 0] / c[:, 1] * khz / 1e3
    assert ((mhz > 50.0) & (mhz < 3000.0)).all(), mhz
    for bad in (0, 10_000_001):
        with pytest.raises(sa.SegattnError) as e:
            sa.segattn_clock_probe(bad, counts)
        assert e.value.status == sa.SEGATTN_EINVAL


def test_mfma_probe_runs_and_reports_its_work():
    import torch
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    flops = sa.segattn_mfma_probe(1000, sink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == 2 * cus * 4 * 1000 * 8 * 2 * 32 * 32 * 16
    assert sa.segattn_mfma_probe(500, sink, operands=1) == flops // 2
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0                                 # the sink is never written
    with pytest.raises(sa.SegattnError):
        sa.segattn_mfma_probe(500, sink, operands=2)
    for bad in (0, 10_000_001):
        with pytest.raises(sa.SegattnError) as e:
            sa.segattn_mfma_probe(bad, sink)
        assert e.value.status == sa.SEGATTN_EINVAL
