"""The library's MFMA rate probe (a measurement aid) does the work it reports: with every operand equal to 1 each
8-pass instruction adds 16 to every accumulator element, so the value a lane writes counts the instructions."""
import pytest
import torch

from paper_2510_08431_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("f16", [0, 1])
def test_rate_probe_counts_its_instructions(f16):
    cus = torch.cuda.get_device_properties(DEV).multi_processor_count
    dt = torch.float16 if f16 else torch.bfloat16
    ones = torch.ones(8 * 256 * 8, dtype=dt, device=DEV)
    out = torch.full((256 * cus,), -1.0, dtype=torch.float32, device=DEV)
    iters = 10
    flops = binding.attn_jvp_mfma_rate_probe(ones, out, f16, iters)
    torch.cuda.synchronize()
    # per lane: 4 chains x 16 accumulator elements, each grown by 16 per instruction, 4 * iters instructions per chain
    assert torch.all(out == 4 * 16 * 16 * 4 * iters)
    assert flops == 32768.0 * 16 * iters * 4 * cus
    zeros = torch.zeros_like(ones)
    binding.attn_jvp_mfma_rate_probe(zeros, out, f16, iters)
    torch.cuda.synchronize()
    assert torch.all(out == 0)
    with pytest.raises(binding.AttnJvpError):
        binding.attn_jvp_mfma_rate_probe(ones, out, f16, 0)
