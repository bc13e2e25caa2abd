"""The MFMA ceiling probe of the library runs and reports plausible numbers."""
import pytest

pytestmark = pytest.mark.gpu


def test_mfma_ceiling_runs_and_reports():
    import torch
    from paper_2410_09397_amd import attn
    clock, flops = attn.attn_mfma_ceiling(2000)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == 2 * cus * 4 * 8 * 2000 * 2.0 * 32 * 32 * 16
    assert 0.5 < float(clock.item()) < 3.0   # GHz
    with pytest.raises(attn.AttnError):
        attn.attn_mfma_ceiling(0)
    for operands in (1, 2, 3, 4):  # zero operands; B operand from LDS; plus vector arithmetic; tile-loop skeleton
        clock, f2 = attn.attn_mfma_ceiling(500, operands)
        torch.cuda.synchronize()
        assert f2 == flops / 4 and 0.5 < float(clock.item()) < 3.0
    with pytest.raises(attn.AttnError):
        attn.attn_mfma_ceiling(10, 5)
