"""The entry point that allocates nothing (abs_average_bf16_static) against abs_average_bf16 with a caller's
scratch buffer: bit-equal results on two calls in a row, the second on a smaller block; sizes beyond the static
buffer are refused."""
import numpy as np
import pytest

from oracle import abs_oracle as O

pytestmark = pytest.mark.gpu


def test_static_mean_buffer_average_equals_the_scratch_argument_average():
    import torch
    import paper_2406_13936_amd as A
    gen = torch.Generator(device="cuda").manual_seed(11)
    # both blocks are large enough for the two-pass form (the one that stages the mean), ragged against the block size
    for M, n in ((8, (6 << 20) + 8 * 37), (8, (4 << 20) + 8 * 11)):
        p_ref = (torch.randn((M, n), generator=gen, device="cuda", dtype=torch.float32) / 8).to(torch.bfloat16)
        p_new = p_ref.clone()
        before = p_ref[:, :4096].double().cpu().numpy()
        scratch = torch.full((n,), float("nan"), device="cuda", dtype=torch.bfloat16)
        A.average_bf16(p_ref, scratch)
        A.average_bf16_static(p_new)
        torch.cuda.synchronize()
        assert torch.equal(p_ref.view(torch.int16), p_new.view(torch.int16)), (M, n)
        # and against the oracle's mean (fp32 summation may differ from fp64 in the last bf16 digit on exact ties)
        want = O.bf16_round(O.average(before)[0])
        got = p_new[3, :4096].double().cpu().numpy()
        assert (got != want).mean() < 2e-3 and np.abs(got - want).max() <= 2 ** -7 * np.abs(want).max()
    small = torch.ones((3, 64), device="cuda", dtype=torch.bfloat16)       # one-pass form: no staging at all
    small[1] = 4.0
    A.average_bf16_static(small)
    assert torch.all(small == 2.0)
    with pytest.raises(A.AbsError, match="static mean buffer"):
        A.average_bf16_static(torch.zeros((2, (16 << 20) + 8), device="cuda", dtype=torch.bfloat16))
