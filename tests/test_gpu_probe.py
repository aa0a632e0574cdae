"""The ceiling probes of the benchmark run, report the work they perform, and leave their buffer's data alone
(read and matrix kinds) or fill it (write kind)."""
import pytest
import torch

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_ceiling_probes_run_and_report_work():
    from paper_2603_05168_amd import probe as s
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    buf = torch.zeros(8 << 20, dtype=torch.uint8, device=DEV)
    buf[256:] = 7
    for kind, per in ((s.SBN_CEIL_SMFMAC_I8, 2 * 32 * 32 * 64), (s.SBN_CEIL_MFMA_I8, 2 * 32 * 32 * 32),
                      (s.SBN_CEIL_MFMA_BF16, 2 * 32 * 32 * 16)):
        work = s.sbn_ceiling_probe(kind, buf, 3)
        assert work == per * 16 * 3 * 4 * 2 * cus
    assert s.sbn_ceiling_probe(s.SBN_CEIL_LDS_READ, buf, 5) == 16 * 16 * 256 * 5 * 2 * cus
    work = s.sbn_ceiling_probe(s.SBN_CEIL_HBM_READ, buf, 1)
    torch.cuda.synchronize()
    assert 0 < work <= buf.numel() - 256 and work > buf.numel() - 256 - 16 * 8 * cus
    assert int(buf[256:].min()) == 7 and int(buf[256:].max()) == 7 and int(buf[:256].max()) == 0
    work_w = s.sbn_ceiling_probe(s.SBN_CEIL_HBM_WRITE, buf, 1)
    torch.cuda.synchronize()
    assert work_w == work
    assert int(buf[:256].max()) == 0                       # the first 256 bytes stay out of the stream
    written = buf[256:256 + int(work_w)].view(torch.int32).view(-1, 4)
    assert bool((written[:, 2] == 3).all()) and bool((written[:, 3] == 4).all())
