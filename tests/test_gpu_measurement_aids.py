"""The measurement-aid kernels of the library (mpa_ceiling_launch) on the GPU: every kind launches,
reports the work it is documented to do, completes, and leaves the caller's data alone."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mpa():
    import paper_2503_13737_amd as m
    m.load()
    return m


def test_every_ceiling_kind_runs_and_reports_its_work(mpa):
    import torch
    nbytes = 256 << 20
    buf = torch.full((nbytes,), 3, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    per_pass = 4096 * 256 * 8 * 16                       # whole passes of the read kernel's grid
    assert mpa.ceiling_launch(mpa.MPA_CEIL_STREAM_READ, buf, nbytes, 0, sink) == nbytes // per_pass * per_pass
    waves = 4096 * 4
    assert mpa.ceiling_launch(mpa.MPA_CEIL_RANDOM_4K, buf, nbytes, 4, sink) == waves * 5 * 4096
    assert mpa.ceiling_launch(mpa.MPA_CEIL_RANDOM_16K, buf, nbytes, 2, sink) == waves * 3 * 16384
    flops = 1024 * 4 * 10 * 4 * 2 * 32 * 32 * 16
    assert mpa.ceiling_launch(mpa.MPA_CEIL_MFMA_BF16, None, 0, 10, sink) == flops
    assert mpa.ceiling_launch(mpa.MPA_CEIL_MFMA_BF16_NOISY, None, 0, 10, sink) == flops
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    assert int(buf[:4096].min().item()) == 3 and int(buf[-4096:].max().item()) == 3
    with pytest.raises(mpa.MpaError):
        mpa.ceiling_launch(mpa.MPA_CEIL_RANDOM_4K, buf, nbytes, 3, sink)     # odd chunk count
