"""GPU: the measurement probes run, write finite values, and refuse the instruction counts they have no kernel for."""
import pytest

from paper_2505_19342_amd import binding as B

pytestmark = pytest.mark.gpu


def test_probes_run_and_check_their_arguments():
    import torch
    out = torch.full((4 * 512,), float("nan"), dtype=torch.float32, device="cuda:0")
    B.astra_probe_mfma_bf16(out, 4, 10)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    for nv in (0, 2, 4, 8, 16):
        for use_exp in (False, True):
            out.fill_(float("nan"))
            B.astra_probe_mfma_valu_bf16(out, 4, 10, nv, use_exp)
            torch.cuda.synchronize()
            assert torch.isfinite(out).all()
    with pytest.raises(B.AstraError):
        B.astra_probe_mfma_valu_bf16(out, 4, 10, 3, False)
    with pytest.raises(B.AstraError):
        B.astra_probe_mfma_valu_bf16(out, 0, 10, 4, False)
