"""The measurement aids of the library on the GPU: the MFMA-only loop, the issue probe and the clock sample run to the end
and report plausible figures (they carry no method arithmetic: nothing here is compared with the oracle)."""
import pytest
import torch

import paper_2503_20313_amd as tl
from tests.gpu_util import dev, make_ctx

pytestmark = pytest.mark.gpu


def test_mfma_peak_probe_counts_its_work_and_samples_the_clock():
    ctx = make_ctx(world_size=1, rank=0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_thr = cus * 512
    opnd = torch.randn((n_thr, 48), device=dev(), dtype=torch.float32).to(torch.bfloat16).contiguous()
    sink = torch.zeros(n_thr, dtype=torch.float32, device=dev())
    clk = torch.zeros(2, dtype=torch.int64, device=dev())
    flop = tl.tl_mfma_peak_probe(ctx, opnd, opnd.numel() * 2, 200, sink, clk)
    torch.cuda.synchronize()
    assert flop == cus * 8 * 200 * 8 * 32768
    cyc, ticks = clk.cpu().tolist()
    assert cyc >= 200 * 8 * 32 and ticks > 0                     # a wave cannot issue its matrix instructions faster than one per 32 cycles
    assert 300.0 < cyc / ticks * 100.0 < 3000.0                 # a shader clock in MHz
    assert torch.isfinite(sink).all()
    with pytest.raises(tl.TileLinkError):
        tl.tl_mfma_peak_probe(ctx, opnd, 1024, 200, sink, clk)    # operand buffer too small
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("with_mfma", [1, 0])
def test_issue_probe_every_mode(with_mfma):
    ctx = make_ctx(world_size=1, rank=0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(1 + cus * 512, dtype=torch.float32, device=dev())
    clk = torch.zeros(2, dtype=torch.int64, device=dev())
    for mode in range(5):
        slots = tl.tl_issue_probe(ctx, with_mfma, mode, 100, sink, clk)
        torch.cuda.synchronize()
        assert slots == 800
        cyc, ticks = clk.cpu().tolist()
        assert cyc > 0 and ticks >= 0
        if with_mfma:
            assert cyc >= 800 * 32
        assert torch.isfinite(sink).all()
    with pytest.raises(tl.TileLinkError):
        tl.tl_issue_probe(ctx, 1, 7, 100, sink, clk)
    tl.tl_ctx_destroy(ctx)
