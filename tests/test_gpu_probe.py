"""GPU: the matrix-core probe runs, writes finite values and checks its arguments."""
import pytest

from paper_2505_19342_amd import binding as B

pytestmark = pytest.mark.gpu


def test_probe_runs_and_checks_its_arguments():
    import torch
    out = torch.full((4 * 512,), float("nan"), dtype=torch.float32, device="cuda:0")
    B.astra_probe_mfma_bf16(out, 4, 10)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    with pytest.raises(B.AstraError):
        B.astra_probe_mfma_bf16(out, 0, 10)
