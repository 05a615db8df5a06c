"""The library allocates nothing: device memory as the driver sees it (free bytes) and as the
caching allocator sees it is the same before and after every entry point, called through the C
ABI with caller-owned outputs."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_device_memory_is_unchanged_across_every_entry_point():
    from paper_2511_13645_amd import binding
    L = binding.lib()
    dev = "cuda:0"
    rng = np.random.default_rng(0)
    n, D, B, k1, k2, k3 = 5000, 64, 700, 6, 5, 4
    deg = rng.integers(0, 30, n)
    indptr = torch.from_numpy(np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)).to(dev)
    indices = torch.from_numpy(rng.integers(0, n, int(deg.sum())).astype(np.int32)).to(dev)
    ew = torch.rand(indices.shape[0], device=dev)
    x = torch.randn((n, D), device=dev)
    seeds = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(dev)
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device=dev)
    out, m1, h1, h2 = z(B, D), z(B, D), z(B, k1, D), z(B, k1, k2, D)
    ids1, ids2, ids3 = z(B, k1, dt=torch.int32), z(B, k1, k2, dt=torch.int32), z(B, k1, k2, k3, dt=torch.int32)
    cnt2, w1, w2 = z(B, k1, dt=torch.int32), z(B, k1), z(B, k1, k2)
    g, gh, gx, gx16, work = z(B, D) + 1, z(B, k1, D) + 1, z(n, D), z(n, D, dt=torch.bfloat16), z(B, k1, D)
    Dw = 2048                                              # wide rows: 700*6*5 entries x 8 KB take the owning route
    gw, gxw = z(B, Dw) + 1, z(n, Dw)
    need = L.fsa_mean_bwd_workspace_bytes(B, k1, k2, Dw)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    fan = (ctypes.c_int32 * 3)(k1, k2, k3)
    fp = ctypes.cast(fan, ctypes.c_void_p)
    st = torch.cuda.current_stream().cuda_stream
    P = lambda t: t.data_ptr()
    calls = {
        "fsa_sample_mean_fwd 1-hop": lambda: L.fsa_sample_mean_fwd(P(indptr), 0, P(indices), n, P(x), 0, D, P(seeds), B, fp, 1, 3,
                                                                   P(out), None, P(ids1), None, st),
        "fsa_sample_mean_fwd 2-hop": lambda: L.fsa_sample_mean_fwd(P(indptr), 0, P(indices), n, P(x), 0, D, P(seeds), B, fp, 2, 3,
                                                                   P(out), P(h1), P(ids1), P(ids2), st),
        "fsa_mean_replay_fwd": lambda: L.fsa_mean_replay_fwd(P(x), 0, D, n, P(ids1), P(ids2), B, k1, k2, P(out), P(h1), st),
        "fsa_mean_bwd": lambda: L.fsa_mean_bwd(P(g), P(gh), P(ids1), P(ids2), B, k1, k2, D, P(gx), n, st),
        "fsa_mean_bwd_ws (atomic route)": lambda: L.fsa_mean_bwd_ws(P(g), P(gh), P(ids1), P(ids2), B, k1, k2, D, P(gx), n,
                                                                    P(ws), ws.numel(), st),
        "fsa_mean_bwd_ws (owning route)": lambda: L.fsa_mean_bwd_ws(P(gw), None, P(ids1), P(ids2), B, k1, k2, Dw, P(gxw), n,
                                                                    P(ws), ws.numel(), st),
        "fsa_mean_bwd_lp": lambda: L.fsa_mean_bwd_lp(P(g), P(gh), 0, P(ids1), P(ids2), B, k1, k2, D, P(gx16), 1, n, st),
        "fsa_sample_wmean_fwd": lambda: L.fsa_sample_wmean_fwd(P(indptr), 0, P(indices), P(ew), n, P(x), 0, D, P(seeds), B, fp, 2, 3,
                                                               P(out), P(h1), P(ids1), P(ids2), P(w1), P(w2), st),
        "fsa_wmean_replay_fwd": lambda: L.fsa_wmean_replay_fwd(P(x), 0, D, n, P(ids1), P(ids2), P(w1), P(w2), B, k1, k2,
                                                               P(out), P(h1), st),
        "fsa_wmean_bwd": lambda: L.fsa_wmean_bwd(P(g), P(gh), P(ids1), P(ids2), P(w1), P(w2), B, k1, k2, D, P(gx), n, st),
        "fsa_sample_mean_layerwise_fwd": lambda: L.fsa_sample_mean_layerwise_fwd(P(indptr), 0, P(indices), n, P(x), 0, D, P(seeds), B,
                                                                                 fp, 3, P(out), P(h1), P(m1), P(ids1), P(ids2), st),
        "fsa_sample_mean3_fwd": lambda: L.fsa_sample_mean3_fwd(P(indptr), 0, P(indices), n, P(x), 0, D, P(seeds), B, fp, 3,
                                                               P(out), P(h1), P(h2), P(m1), P(ids1), P(ids2), P(ids3), P(cnt2), st),
        "fsa_mean3_replay_fwd": lambda: L.fsa_mean3_replay_fwd(P(x), 0, D, n, P(ids1), P(ids2), P(ids3), B, k1, k2, k3,
                                                               P(out), P(h1), P(h2), P(m1), P(cnt2), st),
        "fsa_mean3_bwd": lambda: L.fsa_mean3_bwd(P(g), P(gh), None, P(g), P(ids1), P(ids2), P(ids3), B, k1, k2, k3, D,
                                                 P(gx), n, P(work), st),
    }
    for name, call in calls.items():                     # first calls load the code objects
        assert call() == 0, name
    torch.cuda.synchronize()
    for name, call in calls.items():
        free0, _ = torch.cuda.mem_get_info()
        alloc0, reserved0 = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
        for _ in range(3):
            assert call() == 0, name
        torch.cuda.synchronize()
        free1, _ = torch.cuda.mem_get_info()
        assert free1 == free0, "%s: free device memory went from %d to %d" % (name, free0, free1)
        assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == (alloc0, reserved0), name
