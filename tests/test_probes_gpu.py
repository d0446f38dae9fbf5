"""The two measurement aids of the library run, report what they launched and reject bad arguments.
They produce no result to compare with the oracle: bench.py times them to get the practical HBM and
matrix-pipe ceilings it prints next to the data-sheet peaks.
"""
import pytest
import torch

from paper_2505_11076_amd import binding as B

import gpu_util as G

pytestmark = pytest.mark.gpu


def test_read_probe_runs_and_rejects_short_or_unaligned_buffers():
    G.say("start read probe")
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.dbf_probe_read(buf.data_ptr(), buf.numel(), sink.data_ptr(), 0)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0  # all-zero input never hits the sink value
    with pytest.raises(B.DbfError):
        B.dbf_probe_read(buf.data_ptr(), 1000, 0, 0)
    with pytest.raises(B.DbfError):
        B.dbf_probe_read(buf.data_ptr() + 4, 1 << 19, 0, 0)


@pytest.mark.parametrize("wide", [False, True])
@pytest.mark.parametrize("ands", [False, True])
def test_matrix_pipe_probe_runs_and_counts_its_operations(wide, ands):
    G.say("start mfma probe wide=%s ands=%s" % (wide, ands))
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ops = B.dbf_probe_mfma(wide, ands, 2, 10, sink.data_ptr(), 0)
    torch.cuda.synchronize()
    # 32 x 16*16*64 or 8 x 32*32*32 multiply-adds (2 operations each) per wavefront and iteration,
    # 4 wavefronts per workgroup, 2 workgroups per compute unit
    macs = 8 * 32 * 32 * 32 if wide else 32 * 16 * 16 * 64
    assert ops == 2.0 * macs * 10 * 4 * 2 * cus
    for bad in ((0, 10), (5, 10), (2, 0)):
        with pytest.raises(B.DbfError):
            B.dbf_probe_mfma(wide, ands, bad[0], bad[1], 0, 0)
