"""The error bound the GPU tests use for a 16-bit grad_x, checked on the CPU against the
arithmetic it describes: contributions rounded once to the 16-bit type, then a running sum
that is rounded after every addition, in any order.  With n additions the result stays within
(n + 1) * ulp * sum|c| of the exact sum, ulp = 2^-8 (bfloat16) or 2^-10 (fp16), and a bound
of a fraction of that would be violated -- the tolerance is neither vacuous nor too tight."""
import numpy as np
import pytest
import torch

ULP = {torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -10}


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_running_sum_bound(dtype):
    rng = np.random.default_rng(0)
    worst = 0.0
    for n in (1, 2, 3, 10, 50, 200, 1000):
        for trial in range(20):
            c = rng.standard_normal((n, 256)) * rng.choice([1e-2, 1.0, 30.0])
            exact = c.sum(0)
            mag = np.abs(c).sum(0)
            s = torch.zeros(256, dtype=dtype)
            for i in rng.permutation(n):
                s = s + torch.from_numpy(c[i]).to(dtype)          # rounds the term, then the sum
            err = np.abs(s.to(torch.float64).numpy() - exact)
            bound = (n + 1) * ULP[dtype] * mag
            assert (err <= bound).all(), (n, trial)
            worst = max(worst, float((err / bound).max()))
    assert worst > 0.02          # the bound is within a factor of 50 of what really happens
