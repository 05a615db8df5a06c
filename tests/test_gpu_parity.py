"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs -- element by element at sizes that span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from parity_util import TOL, assert_close, assert_ids_equal, forward_scales, host_x, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def ragged_graph(n, seed, max_deg=90, hub_deg=5000, wide=False):
    """Rows of every kind: empty, shorter than, equal to and far longer than any fanout used,
    one hub, parallel edges."""
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, max_deg + 1, size=n)
    deg[rng.random(n) < 0.15] = 0
    deg[:8] = [0, 1, 9, 10, 11, 64, 65, hub_deg]
    indptr = np.concatenate([[0], np.cumsum(deg)])
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    return indptr.astype(np.int64 if wide else np.int32), indices


def run_case(fsa, orc, indptr, indices, x, seeds, fan, seed, check_bwd=True, what=""):
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    d_x = x.to(dev)
    d_seeds = torch.from_numpy(seeds).to(dev)
    tol = TOL[x.dtype]
    hx, is_bf16 = host_x(x)
    r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(indptr, indices, hx, seeds, fan, seed, bf16=is_bf16)

    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, d_x, d_seeds, fan, seed)
    torch.cuda.synchronize()
    assert_ids_equal(ids1, r_ids1, what + " ids1")
    if len(fan) == 2:
        assert_ids_equal(ids2, r_ids2, what + " ids2")
    a_out, a_h1 = forward_scales(d_x, ids1, ids2)
    assert_close(to_f64(out), r_out, a_out, tol, what + " out")
    if len(fan) == 2:
        assert_close(to_f64(h1), r_h1, a_h1, tol, what + " out_h1")

    # without ID / per-slot emission the means are the same bits
    out_b, h1_b, i1_b, i2_b = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, d_x, d_seeds, fan, seed,
                                                      emit_ids=False, emit_h1=False)
    assert i1_b is None and i2_b is None and h1_b is None
    assert torch.equal(out_b.view(torch.uint8), out.view(torch.uint8)), what + " emit-off differs"

    # replay from the emitted IDs: bitwise equal to the sampling forward
    rp_out, rp_h1 = fsa.fsa_mean_replay_fwd(d_x, ids1, ids2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out.view(torch.uint8), out.view(torch.uint8)), what + " replay out differs"
    if len(fan) == 2:
        assert torch.equal(rp_h1.view(torch.uint8), h1.view(torch.uint8)), what + " replay h1 differs"

    if check_bwd:
        B, D, N = seeds.shape[0], x.shape[1], x.shape[0]
        g = torch.from_numpy(np.random.default_rng(3).standard_normal((B, D)).astype(np.float32)).to(dev)
        gh = None
        if len(fan) == 2:
            gh = torch.from_numpy(np.random.default_rng(4).standard_normal((B, fan[0], D)).astype(np.float32)).to(dev)
        gx = torch.zeros((N, D), dtype=torch.float32, device=dev)
        fsa.fsa_mean_bwd(g, ids1, ids2, gh, grad_x=gx)
        torch.cuda.synchronize()
        r_gx = orc.mean_bwd(to_f64(g), r_ids1, r_ids2, None if gh is None else to_f64(gh), num_nodes=N)
        scale = orc.mean_bwd(np.abs(to_f64(g)), r_ids1, r_ids2, None if gh is None else np.abs(to_f64(gh)), num_nodes=N)
        assert_close(to_f64(gx), r_gx, scale, 1e-5, what + " grad_x")
        # accumulation: a second call adds on top
        fsa.fsa_mean_bwd(g, ids1, ids2, gh, grad_x=gx)
        torch.cuda.synchronize()
        assert_close(to_f64(gx), 2 * r_gx, 2 * scale, 1e-5, what + " grad_x accumulated")
    return out, h1, ids1, ids2


def test_tiny_config_forward_ids_replay_backward(fsa, orc):
    """Config 'Tiny 1-hop': N=10,000, Zipf degrees, x[N,64] fp32, B=1024, k=10, seed 0."""
    from paper_2511_13645_amd import synth
    w = synth.make_workload("tiny")
    seeds = synth.seed_batches(w.graph.num_nodes, w.batch, 1, seed=2)[0].numpy()
    run_case(fsa, orc, w.graph.indptr.numpy(), w.graph.indices.numpy(), w.x, seeds, [10], 0, what="tiny")


F32_DIMS = [1, 3, 6, 64, 100, 128, 257, 602, 1000]
BF16_DIMS = [1, 3, 8, 100, 128, 130, 520]


@pytest.mark.parametrize("D", F32_DIMS)
@pytest.mark.parametrize("fan", [[10], [15, 10]])
def test_fp32_dims(fsa, orc, D, fan):
    n = 3000
    indptr, indices = ragged_graph(n, seed=D)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32))
    rng = np.random.default_rng(1)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, 250), [7, 7]]).astype(np.int32)   # ragged B, duplicates
    run_case(fsa, orc, indptr, indices, x, seeds, fan, 1234 + D, what="fp32 D=%d fan=%s" % (D, fan))


@pytest.mark.parametrize("D", BF16_DIMS)
@pytest.mark.parametrize("fan", [[15], [15, 10]])
def test_bf16_dims_and_wide_indptr(fsa, orc, D, fan):
    n = 2500
    indptr, indices = ragged_graph(n, seed=100 + D, wide=True)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32)).to(torch.bfloat16)
    seeds = np.concatenate([np.arange(8), np.random.default_rng(2).integers(0, n, 193)]).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, fan, 2**63 + D, check_bwd=False,
             what="bf16 D=%d fan=%s" % (D, fan))


@pytest.mark.parametrize("fan", [[1], [64], [25], [1, 1], [64, 64], [25, 10], [3, 33], [40, 7], [7, 64]])
def test_fanout_range(fsa, orc, fan):
    n = 2000
    indptr, indices = ragged_graph(n, seed=sum(fan), max_deg=150)
    x = torch.from_numpy(np.random.default_rng(0).standard_normal((n, 36)).astype(np.float32))
    seeds = np.concatenate([np.arange(8), np.random.default_rng(5).integers(0, n, 57)]).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, fan, 99, what="fan=%s" % fan)


def test_degenerate_graphs(fsa, orc):
    n, D = 64, 16
    x = torch.from_numpy(np.random.default_rng(0).standard_normal((n, D)).astype(np.float32))
    seeds = np.arange(n, dtype=np.int32)
    # no edges at all: every output is a zero row, every ID is -1
    indptr = np.zeros(n + 1, dtype=np.int32)
    indices = np.zeros(1, dtype=np.int32)
    for fan in ([5], [5, 4]):
        out, h1, ids1, ids2 = run_case(fsa, orc, indptr, indices, x, seeds, fan, 1, what="edgeless")
        assert (out == 0).all() and (ids1 == -1).all()
    # hop-1 nodes all empty: seeds point at sinks
    indptr = np.concatenate([np.arange(0, 33) * 3, np.full(32, 96)]).astype(np.int32)   # rows 0..31 have 3, rest 0
    indices = np.random.default_rng(1).integers(32, 64, 96).astype(np.int32)
    out, h1, ids1, ids2 = run_case(fsa, orc, indptr, indices, x, seeds, [4, 4], 2, what="sinks")
    assert (out == 0).all() and (h1 == 0).all() and (ids2 == -1).all() and (ids1[:32, :3] >= 32).all()
    # B = 1 and a single self-contained row
    run_case(fsa, orc, np.array([0, 5], np.int32), np.zeros(5, np.int32), x[:1].contiguous(),
             np.zeros(1, np.int32), [3, 2], 3, what="one node")


def test_empty_batch(fsa):
    dev = "cuda:0"
    indptr = torch.zeros(11, dtype=torch.int32, device=dev)
    indices = torch.zeros(1, dtype=torch.int32, device=dev)
    x = torch.zeros((10, 8), device=dev)
    seeds = torch.zeros(0, dtype=torch.int32, device=dev)
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(indptr, indices, x, seeds, [4, 3], 0)
    assert out.shape == (0, 8) and h1.shape == (0, 4, 8) and ids2.shape == (0, 4, 3)
    o, h = fsa.fsa_mean_replay_fwd(x, ids1, ids2)
    gx = torch.zeros_like(x)
    fsa.fsa_mean_bwd(out, ids1, ids2, grad_x=gx)
    torch.cuda.synchronize()
    assert (gx == 0).all()


def test_unaligned_table_falls_back_to_narrow_loads(fsa, orc):
    """A table whose base is only 4-byte (fp32) / 2-byte (bf16) aligned still works."""
    n, D = 1500, 128
    indptr, indices = ragged_graph(n, seed=9)
    seeds = np.random.default_rng(0).integers(0, n, 100).astype(np.int32)
    dev = "cuda:0"
    for dtype in (torch.float32, torch.bfloat16):
        flat = torch.from_numpy(np.random.default_rng(1).standard_normal(n * D + 1).astype(np.float32)).to(dtype).to(dev)
        x = flat[1:].view(n, D)
        assert x.data_ptr() % 16 != 0
        hx, is_bf16 = host_x(x)
        r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(indptr, indices, hx, seeds, [15, 10], 5, bf16=is_bf16)
        out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev),
                                                      x, torch.from_numpy(seeds).to(dev), [15, 10], 5)
        torch.cuda.synchronize()
        assert_ids_equal(ids2, r_ids2, "unaligned ids2")
        a_out, a_h1 = forward_scales(x, ids1, ids2)
        assert_close(to_f64(out), r_out, a_out, TOL[dtype], "unaligned out")
        assert_close(to_f64(h1), r_h1, a_h1, TOL[dtype], "unaligned h1")


def test_replay_with_holes_anywhere(fsa, orc):
    """Saved-ID arrays edited by the caller: negative entries in arbitrary places."""
    rng = np.random.default_rng(11)
    n, D, B, k1, k2 = 800, 48, 77, 9, 6
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    ids1 = rng.integers(0, n, (B, k1)).astype(np.int32)
    ids2 = rng.integers(0, n, (B, k1, k2)).astype(np.int32)
    ids1[rng.random(ids1.shape) < 0.3] = -1
    ids2[rng.random(ids2.shape) < 0.4] = -1
    ids2[3] = -1
    ids2[5, 2] = ids2[5, 2, 0]                      # a slot made of one repeated row
    dev = "cuda:0"
    d_x, d1, d2 = x.to(dev), torch.from_numpy(ids1).to(dev), torch.from_numpy(ids2).to(dev)
    for two in (False, True):
        r_out, r_h1 = orc.mean_replay_fwd(x.numpy(), ids1, ids2 if two else None)
        out, h1 = fsa.fsa_mean_replay_fwd(d_x, d1, d2 if two else None)
        torch.cuda.synchronize()
        masked2 = torch.where(d1[..., None] >= 0, d2, torch.full_like(d2, -1)) if two else None
        a_out, a_h1 = forward_scales(d_x, d1, masked2)
        assert_close(to_f64(out), r_out, a_out, 1e-5, "holes out")
        if two:
            assert_close(to_f64(h1), r_h1, a_h1, 1e-5, "holes h1")
        g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(dev)
        gh = torch.from_numpy(rng.standard_normal((B, k1, D)).astype(np.float32)).to(dev) if two else None
        gx = torch.zeros((n, D), device=dev)
        fsa.fsa_mean_bwd(g, d1, d2 if two else None, gh, grad_x=gx)
        torch.cuda.synchronize()
        r_gx = orc.mean_bwd(to_f64(g), ids1, ids2 if two else None, None if gh is None else to_f64(gh), num_nodes=n)
        scale = orc.mean_bwd(np.abs(to_f64(g)), ids1, ids2 if two else None,
                             None if gh is None else np.abs(to_f64(gh)), num_nodes=n)
        assert_close(to_f64(gx), r_gx, scale, 1e-5, "holes grad_x")


def test_ids_do_not_depend_on_batching_or_stream(fsa):
    """Draws are keyed by (seed, node, hop, step): any split of the seeds gives the same IDs
    and the same bits; a side stream gives the same result as the default one."""
    n, D = 5000, 128
    indptr, indices = ragged_graph(n, seed=21)
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    x = torch.randn((n, D), generator=torch.Generator().manual_seed(0)).to(dev)
    seeds = torch.from_numpy(np.random.default_rng(0).integers(0, n, 1000).astype(np.int32)).to(dev)
    full = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [15, 10], 7)
    parts = [fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds[a:b].contiguous(), [15, 10], 7)
             for a, b in ((0, 1), (1, 334), (334, 1000))]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        side = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [15, 10], 7)
    torch.cuda.synchronize()
    for i in range(4):
        assert torch.equal(torch.cat([p[i] for p in parts]), full[i])
        assert torch.equal(side[i], full[i])
    other = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [15, 10], 8)
    assert not torch.equal(other[3], full[3])


@pytest.mark.parametrize("n_targets,B", [(3, 700), (100, 4096), (1000, 20000)])
def test_backward_with_heavily_shared_rows(fsa, orc, n_targets, B):
    """Every row of the graph points into the same small set of nodes, so the seeds of a
    workgroup keep hitting the same rows: exercises the in-LDS aggregation of shared rows in
    the 1-hop backward (more shared rows than LDS rows when n_targets is large)."""
    rng = np.random.default_rng(n_targets)
    n, D, k = 30000, 96, 15
    deg = rng.integers(0, 40, size=n)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    hot = rng.permutation(n)[:n_targets]
    p = 1.0 / np.arange(1, n_targets + 1) ** 1.2
    indices = hot[rng.choice(n_targets, size=int(indptr[-1]), p=p / p.sum())].astype(np.int32)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    seeds = rng.integers(0, n, B).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [k], 3, what="shared rows %d" % n_targets)
    run_case(fsa, orc, indptr, indices, x, seeds[:777], [5, 4], 3, what="shared rows 2-hop %d" % n_targets)


def test_very_wide_rows_and_large_batch(fsa, orc):
    """Rows of 8192 floats (32 tiles per row) and a batch beyond 65,535 workgroups."""
    rng = np.random.default_rng(8)
    n = 600
    indptr, indices = ragged_graph(n, seed=8, max_deg=40, hub_deg=300)
    x = torch.from_numpy(rng.standard_normal((n, 8192)).astype(np.float32))
    seeds = rng.integers(0, n, 33).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [6, 5], 1, what="D=8192 2-hop")
    run_case(fsa, orc, indptr, indices, x, seeds, [9], 1, what="D=8192 1-hop")
    n = 5000
    indptr, indices = ragged_graph(n, seed=9, max_deg=30, hub_deg=500)
    x = torch.from_numpy(rng.standard_normal((n, 16)).astype(np.float32))
    seeds = rng.integers(0, n, 70_001).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [4, 3], 2, what="B=70001 2-hop")
    run_case(fsa, orc, indptr, indices, x, seeds, [5], 2, what="B=70001 1-hop")


@pytest.mark.parametrize("B,fan,D,bf16", [(4096, [15, 10], 64, False), (2048, [15, 10], 128, True),
                                          (8192, [9, 4], 40, False), (5000, [64, 3], 32, False), (4096, [8, 64], 602, False)])
def test_mid_size_batches_with_roots_of_every_weight(fsa, orc, B, fan, D, bf16):
    """Batches of 2048..8192 roots (one or two waves per root, every root resident at once): roots
    of every weight (no slots, a few, all of them) next to each other -- forward, emission off,
    replay (also with holes that change a root's weight) and backward."""
    n = 6000
    indptr, indices = ragged_graph(n, seed=B % 97, max_deg=30, hub_deg=3000)
    rng = np.random.default_rng(B)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    if bf16:
        x = x.to(torch.bfloat16)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    out, h1, ids1, ids2 = run_case(fsa, orc, indptr, indices, x, seeds, fan, 1234, check_bwd=not bf16,
                                   what="mid-size B=%d fan=%s" % (B, fan))
    # replay with holes: roots become lighter or empty
    h_ids1, h_ids2 = ids1.cpu().numpy().copy(), ids2.cpu().numpy().copy()
    h_ids1[rng.random(h_ids1.shape) < 0.5] = -1
    h_ids2[rng.random(h_ids2.shape) < 0.3] = -1
    hx, is_bf16 = host_x(x)
    r_out, r_h1 = orc.mean_replay_fwd(hx, h_ids1, h_ids2, bf16=is_bf16)
    d_x = x.to("cuda:0")
    d1, d2 = torch.from_numpy(h_ids1).to("cuda:0"), torch.from_numpy(h_ids2).to("cuda:0")
    g_out, g_h1 = fsa.fsa_mean_replay_fwd(d_x, d1, d2)
    torch.cuda.synchronize()
    a_out, a_h1 = forward_scales(d_x, d1, torch.where(d1[..., None] >= 0, d2, torch.full_like(d2, -1)))
    assert_close(to_f64(g_out), r_out, a_out, TOL[x.dtype], "mid-size replay holes out")
    assert_close(to_f64(g_h1), r_h1, a_h1, TOL[x.dtype], "mid-size replay holes h1")


@pytest.mark.parametrize("D,bf16", [(256, False), (260, False), (1024, False), (1028, False), (2048, False), (2052, False),
                                     (510, False), (1022, False),
                                     (512, True), (520, True), (2048, True), (2056, True), (4096, True), (4104, True)])
def test_row_widths_around_the_tile_boundaries(fsa, orc, D, bf16):
    """Rows of exactly 1, 2, 4, 5, 8 and 9 tiles of 64 lanes (16- and 8-byte chunks): the single-tile
    gather, both instantiations of the wide-row gather and the fall-back beyond eight tiles, for the
    1-hop, 2-hop and (through the 3-hop call) slot-mean kernels, with one and with several waves per root."""
    n = 700
    indptr, indices = ragged_graph(n, seed=D, max_deg=20, hub_deg=300)
    rng = np.random.default_rng(D)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    if bf16:
        x = x.to(torch.bfloat16)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, 40)]).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [7], 3, check_bwd=False, what="tiles 1-hop D=%d" % D)
    run_case(fsa, orc, indptr, indices, x, seeds, [6, 4], 3, check_bwd=False, what="tiles 2-hop D=%d" % D)
    big = np.concatenate([seeds] * 90)[:4200]                        # one wave per root
    run_case(fsa, orc, indptr, indices, x, big, [6, 4], 3, check_bwd=False, what="tiles 2-hop B=4200 D=%d" % D)
    hx, is_bf16 = host_x(x)
    ref = orc.sample_mean3_fwd(indptr, indices, hx, seeds, [3, 3, 2], 9, bf16=is_bf16, want_h2=False)
    r = fsa.fsa_sample_mean3_fwd(torch.from_numpy(indptr).to("cuda:0"), torch.from_numpy(indices).to("cuda:0"), x.to("cuda:0"),
                                 torch.from_numpy(seeds).to("cuda:0"), [3, 3, 2], 9)
    torch.cuda.synchronize()
    scale = orc.mean3_replay_fwd(np.abs(to_f64(x)), ref["ids1"], ref["ids2"], ref["ids3"], want_h2=False)
    assert_ids_equal(r["ids3"], ref["ids3"], "tiles 3-hop ids3")
    for k in ("out", "out_h1", "out_m1"):
        assert_close(to_f64(r[k]), ref[k], scale[k], TOL[x.dtype], "tiles 3-hop %s D=%d" % (k, D))


def test_maximum_fanouts_with_one_wave_per_root(fsa, orc):
    """Fanouts 64/64 at a batch size that gives every root a single wave: 4096 leaf slots per
    wave in LDS (more than 64 KB per workgroup).  The oracle checks the first 64 seeds (results do
    not depend on the rest of the batch); the backward runs over the whole batch."""
    n, D, B, fan = 3000, 32, 4100, [64, 64]
    indptr, indices = ragged_graph(n, seed=5, max_deg=200, hub_deg=4000)
    rng = np.random.default_rng(0)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    seeds = rng.integers(0, n, B).astype(np.int32)
    ref = orc.sample_mean_fwd(indptr, indices, x.numpy(), seeds[:64], fan, 3)
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), x.cuda(),
                                                  torch.from_numpy(seeds).cuda(), fan, 3)
    torch.cuda.synchronize()
    assert_ids_equal(ids1[:64], ref[2], "ids1")
    assert_ids_equal(ids2[:64], ref[3], "ids2")
    a_out, a_h1 = forward_scales(x.cuda(), ids1[:64], ids2[:64])
    assert_close(to_f64(out[:64]), ref[0], a_out, 1e-5, "out")
    assert_close(to_f64(h1[:64]), ref[1], a_h1, 1e-5, "out_h1")
    g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).cuda()
    gx = fsa.fsa_mean_bwd(g, ids1, ids2, grad_x=torch.zeros((n, D), device="cuda:0"))
    torch.cuda.synchronize()
    want = orc.mean_bwd(to_f64(g), ids1.cpu().numpy(), ids2.cpu().numpy(), num_nodes=n)
    mag = orc.mean_bwd(np.abs(to_f64(g)), ids1.cpu().numpy(), ids2.cpu().numpy(), num_nodes=n)
    assert_close(to_f64(gx), want, mag, 1e-5, "grad_x")
