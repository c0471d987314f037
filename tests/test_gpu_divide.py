"""The reciprocal-based quotient of the bf16 merge + quantize kernel against the hardware's IEEE divide, on the GPU,
for every one of the 2^23 significands a scale can have (three exponents each) and, per scale, every decision point of
the quantizer with five units in the last place to either side (l4q_check_fast_divide)."""
import pytest

pytestmark = pytest.mark.gpu


def test_fast_quotient_equals_ieee_divide_for_every_scale_significand():
    import torch
    from paper_2402_04902_amd import binding
    counts = torch.zeros(4, dtype=torch.int64, device="cuda:0")
    step = 1 << 21
    for first in range(0, 1 << 23, step):
        print("significands", first, "..", first + step - 1, flush=True)
        binding.l4q_check_fast_divide(first, step, counts)
        torch.cuda.synchronize()
    wrong_r, wrong_q, compared = (int(v) for v in counts[:3].cpu())
    print("reciprocals wrong:", wrong_r, "quotients wrong:", wrong_q, "of", compared, flush=True)
    assert compared == (1 << 23) * 3 * (256 + 14) * 11
    assert wrong_r == 0 and wrong_q == 0
