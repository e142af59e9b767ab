"""The wave-wide scans and reductions of the kernels (DPP row shifts and broadcasts) against sums computed on the host."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def test_wave_scans_and_reductions_agree_with_the_host(dgn):
    import torch
    buf = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    assert dgn.dgn_selftest_wave_ops(buf, buf.numel()) == 0
    # argument errors are reported, not acted on
    assert dgn.dgn_selftest_wave_ops(buf, 1024) < 0
