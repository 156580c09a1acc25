"""The measurement aids run: the register-only matrix-instruction loop and the stage-shaped loop of the prefill
linear (each piece alone and together) launch, finish and give the same checksums twice."""
import pytest
import torch

from paper_2209_01188_amd import binding
from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_mfma_loop_runs_and_reports_its_operation_count():
    out = torch.zeros(8 * 256, dtype=torch.int32, device=DEV)
    for kind in (0, 1):
        ops = binding.petals_bench_mfma(kind, 1, 10, 8, out)
        torch.cuda.synchronize()
        assert ops == 8 * 4 * 10 * 262144


@pytest.mark.parametrize("parts", [1, 2, 3, 4, 5, 6, 7])
def test_stage_loop_runs_with_every_combination_of_its_pieces(parts):
    stages, regions, wgs = 6, 2, 24
    g = torch.Generator(device=DEV)
    g.manual_seed(parts)
    src = torch.randint(0, 256, (regions * stages * 32 * 1024,), dtype=torch.uint8, device=DEV, generator=g)
    sums = []
    for _ in range(2):
        out = torch.zeros(wgs * 512, dtype=torch.int32, device=DEV)
        binding.petals_bench_stage(parts, stages, regions, wgs, src, out)
        torch.cuda.synchronize()
        sums.append(out.clone())
    assert torch.equal(sums[0], sums[1])
    if parts & 4:                      # products of random bytes: the checksums are not all zero
        assert int((sums[0] != 0).sum()) > 0
    with pytest.raises(binding.PetalsError):
        binding.petals_bench_stage(parts, stages, regions + 1, wgs, src, out)      # source too small for 3 regions
