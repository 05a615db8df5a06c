"""Seeded random sweep over graph shapes, table types and widths, batch sizes, fanouts and hop
counts: every case goes through the same element-by-element comparison with the oracle as the
hand-picked cases (IDs bit-exact, means and gradients within the documented tolerances, replay
bitwise, holes in replayed IDs).  It exists to reach combinations of kernel instantiations,
launch shapes and ragged tails that nobody thought of listing."""
import numpy as np
import pytest
import torch

from parity_util import to_f64
from test_gpu_parity import ragged_graph, run_case
from test_gpu_three_hop import three_hop_case
from test_gpu_weighted import _run as weighted_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("chunk", range(6))
def test_random_configurations(fsa, orc, chunk):
    rng = np.random.default_rng(1000 + chunk)
    for c in range(10):
        n = int(rng.integers(50, 4000))
        indptr, indices = ragged_graph(n, seed=int(rng.integers(1 << 30)), max_deg=int(rng.choice([3, 12, 40, 90, 300])),
                                       hub_deg=int(rng.integers(100, 6000)), wide=bool(rng.integers(2)))
        dt = [torch.float32, torch.bfloat16, torch.float16][int(rng.integers(3))]
        D = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 100, 128, 130, 256, 300, 513, 602, 1000, 1030, 2050]))
        B = int(rng.choice([1, 7, 64, 300, 1000, 2500, 4500]))
        hops = int(rng.integers(1, 4))
        fan = [int(rng.choice([1, 2, 3, 5, 10, 15, 25, 33, 64])) for _ in range(hops)]
        if hops == 3:
            fan, B = [min(f, 15) for f in fan], min(B, 300)
        if hops == 2 and fan[0] * fan[1] > 400:
            B = min(B, 1000)
        if D > 600:
            B = min(B, 300)
        x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dt)
        seeds = rng.integers(0, n, B).astype(np.int32)
        seed = int(rng.integers(0, 2**63))
        what = "chunk %d case %d: n=%d %s D=%d B=%d fan=%s seed=%d" % (chunk, c, n, dt, D, B, fan, seed)
        print(what, flush=True)
        if hops == 3:
            three_hop_case(fsa, orc, indptr, indices, x, seeds, fan, seed, what)
        elif dt == torch.float16:
            x64 = x.to(torch.float64).numpy()                       # exact
            ref = orc.sample_mean_fwd(indptr, indices, x64, seeds, fan, seed)
            mag = orc.sample_mean_fwd(indptr, indices, np.abs(x64), seeds, fan, seed)[0]
            got = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), x.cuda(),
                                          torch.from_numpy(seeds).cuda(), fan, seed)
            torch.cuda.synchronize()
            assert np.array_equal(got[2].cpu().numpy(), ref[2]), what
            assert (np.abs(to_f64(got[0]) - ref[0]) <= 1e-3 * np.maximum(np.abs(ref[0]), mag)).all(), what
        else:
            run_case(fsa, orc, indptr, indices, x, seeds, fan, seed, check_bwd=(dt == torch.float32), what=what)
            if rng.integers(3) == 0:
                ew = rng.random(indices.size).astype(np.float32)
                weighted_case(fsa, orc, indptr, indices, ew, x, seeds, fan, seed & (2**62 - 1), what + " weighted",
                              check_bwd=(dt == torch.float32))
