"""GPU parity at the full sizes of the five workload shapes, in the launch configuration the
benchmark times.  Graphs and tables are generated on the GPU from the seeded recipes and the
very same bytes are copied to the host for the oracle."""
import time

import numpy as np
import pytest
import torch

from parity_util import TOL, assert_close, assert_ids_equal, forward_scales, host_x, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


def _build(name):
    from paper_2511_13645_amd import synth
    t0 = time.time()
    w = synth.make_workload(name, device="cuda:0")
    torch.cuda.synchronize()
    seeds = synth.seed_batches(w.graph.num_nodes, w.batch, 1, seed=2)[0]
    print("[%s] N=%d E=%d D=%d built in %.1fs" % (name, w.graph.num_nodes, w.graph.num_edges, w.x.shape[1],
                                                   time.time() - t0), flush=True)
    return w, seeds


_HOST = {}


def _host(w):
    """Host copies of a workload's graph and table for the oracle (made once per workload)."""
    if _HOST.get("graph") is not w.graph or _HOST.get("x") is not w.x:
        _HOST.clear()
        hx, is_bf16 = host_x(w.x)
        _HOST.update(graph=w.graph, x=w.x, data=(w.graph.indptr.cpu().numpy(), w.graph.indices.cpu().numpy(), hx, is_bf16))
    return _HOST["data"]


def _sampled_parity(fsa, orc, w, B, n_sample, what):
    """A batch too large for the oracle to redo whole (the benchmark's saturating batch): the GPU
    runs all B seeds, the oracle a sample of them as a batch of its own -- a seed's IDs and means
    do not depend on the batch it is in -- and the sampled rows are compared as everywhere else."""
    from paper_2511_13645_amd import synth
    fan = list(w.fanouts)
    g, x = w.graph, w.x
    seeds = synth.seed_batches(g.num_nodes, B, 1, seed=5)[0]
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(g.indptr, g.indices, x, seeds.cuda(), fan, w.sampler_seed)
    torch.cuda.synchronize()
    rng = np.random.default_rng(B)
    pick = np.unique(np.concatenate([rng.integers(0, B, n_sample), np.arange(B - 70, B), np.arange(0, 8)]))
    h_indptr, h_indices, hx, is_bf16 = _host(w)
    r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(h_indptr, h_indices, hx, seeds.numpy()[pick], fan, w.sampler_seed,
                                                      bf16=is_bf16)
    sel = torch.from_numpy(pick).cuda()
    assert_ids_equal(ids1[sel], r_ids1, what + " ids1 (sample)")
    two = len(fan) == 2
    if two:
        assert_ids_equal(ids2[sel], r_ids2, what + " ids2 (sample)")
    a_out, a_h1 = forward_scales(x, ids1[sel], ids2[sel] if two else None)
    tol = TOL[x.dtype]
    worst = assert_close(to_f64(out[sel]), r_out, a_out, tol, what + " out (sample)")
    if two:
        worst = max(worst, assert_close(to_f64(h1[sel]), r_h1, a_h1, tol, what + " out_h1 (sample)"))
    # properties that hold for every seed of the batch: padding, counts within the fanout, replay bitwise
    assert bool(((ids1 >= -1) & (ids1 < g.num_nodes)).all())
    if two:
        assert bool(((ids2 >= -1) & (ids2 < g.num_nodes)).all()) and bool((ids2[ids1 < 0] == -1).all())
    rp_out, rp_h1 = fsa.fsa_mean_replay_fwd(x, ids1, ids2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out.view(torch.uint8), out.view(torch.uint8)), what + " replay out differs"
    if two:
        assert torch.equal(rp_h1.view(torch.uint8), h1.view(torch.uint8)), what + " replay h1 differs"
    print("[%s] B=%d: %d sampled seeds ids bit-exact, worst relative error %.2e; replay of all %d bitwise"
          % (what, B, pick.size, worst, B), flush=True)


def _forward_parity(fsa, orc, w, seeds, what):
    fan = list(w.fanouts)
    g, x = w.graph, w.x
    d_seeds = seeds.cuda()
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(g.indptr, g.indices, x, d_seeds, fan, w.sampler_seed)
    torch.cuda.synchronize()
    t0 = time.time()
    h_indptr, h_indices, hx, is_bf16 = _host(w)
    t1 = time.time()
    r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(h_indptr, h_indices, hx, seeds.numpy(), fan, w.sampler_seed,
                                                      bf16=is_bf16)
    print("[%s] host copy %.1fs, oracle forward %.1fs" % (what, t1 - t0, time.time() - t1), flush=True)
    assert_ids_equal(ids1, r_ids1, what + " ids1")
    if len(fan) == 2:
        assert_ids_equal(ids2, r_ids2, what + " ids2")
    a_out, a_h1 = forward_scales(x, ids1, ids2)
    tol = TOL[x.dtype]
    worst = assert_close(to_f64(out), r_out, a_out, tol, what + " out")
    if len(fan) == 2:
        worst = max(worst, assert_close(to_f64(h1), r_h1, a_h1, tol, what + " out_h1"))
    print("[%s] ids bit-exact; worst relative error of the means %.2e (bound %.0e)" % (what, worst, tol), flush=True)
    rp_out, rp_h1 = fsa.fsa_mean_replay_fwd(x, ids1, ids2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out.view(torch.uint8), out.view(torch.uint8)), what + " replay out differs"
    if len(fan) == 2:
        assert torch.equal(rp_h1.view(torch.uint8), h1.view(torch.uint8)), what + " replay h1 differs"
    return ids1, ids2, r_ids1, r_ids2


def _backward_parity(fsa, orc, w, ids1, ids2, r_ids1, r_ids2, what, with_h1):
    from paper_2511_13645_amd import synth
    N, D = w.x.shape
    B, k1 = ids1.shape
    g = synth.upstream_grad((B, D), seed=3, device="cuda:0")
    gh = synth.upstream_grad((B, k1, D), seed=4, device="cuda:0") if with_h1 else None
    gx = torch.zeros((N, D), dtype=torch.float32, device="cuda:0")
    fsa.fsa_mean_bwd(g, ids1, ids2, gh, grad_x=gx)
    torch.cuda.synchronize()
    t0 = time.time()
    r_gx = orc.mean_bwd(to_f64(g), r_ids1, r_ids2, None if gh is None else to_f64(gh), num_nodes=N)
    scale = orc.mean_bwd(np.abs(to_f64(g)), r_ids1, r_ids2, None if gh is None else np.abs(to_f64(gh)), num_nodes=N)
    print("[%s] oracle backward %.1fs" % (what, time.time() - t0), flush=True)
    touched = np.unique(np.concatenate([r_ids2[r_ids2 >= 0]]) if r_ids2 is not None else r_ids1[r_ids1 >= 0])
    got = gx[torch.from_numpy(touched).cuda().long()].double().cpu().numpy()
    worst = assert_close(got, r_gx[touched], scale[touched], 1e-5, what + " grad_x (touched rows)")
    # rows nobody sampled stay exactly zero
    total = float(gx.double().abs().sum().item())
    assert abs(total - np.abs(got).sum()) <= 1e-6 * max(1.0, total), what + " gradient leaked outside the sampled rows"
    print("[%s] grad_x over %d touched rows: worst relative error %.2e" % (what, touched.size, worst), flush=True)


def test_products_shape_two_hop_forward(fsa, orc):
    """N=2,449,029, ~123.7M edges, x[N,100] fp32, B=1024, fanouts [15,10], forward only."""
    w, seeds = _build("products")
    assert w.graph.num_nodes == 2_449_029 and abs(w.graph.num_edges / 123.7e6 - 1) < 0.03
    _forward_parity(fsa, orc, w, seeds, "products")


def test_social_shape_two_hop_forward_backward(fsa, orc):
    """N=232,965, ~114.6M edges (mean ~492), x[N,602] fp32, B=1024, fanouts [25,10], fwd + bwd."""
    w, seeds = _build("social")
    assert w.graph.num_nodes == 232_965 and abs(w.graph.num_edges / 114.6e6 - 1) < 0.03
    ids = _forward_parity(fsa, orc, w, seeds, "social")
    _backward_parity(fsa, orc, w, *ids, "social", with_h1=True)


def test_kg_shape_one_hop_training(fsa, orc):
    """2.5M entities, 16.1M triples both directions, x[N,128] fp32 U(-0.1,0.1), B=4096, k=15."""
    w, seeds = _build("kg")
    assert w.graph.num_nodes == 2_500_000 and w.graph.num_edges == 32_200_000
    assert w.graph.degrees().max().item() > 1_000_000       # the Zipf(1.1) hub
    hub = int(torch.argmax(w.graph.degrees()).item())
    seeds = seeds.clone()
    seeds[0] = hub                                           # make sure the longest row is sampled
    ids1, ids2, r_ids1, r_ids2 = _forward_parity(fsa, orc, w, seeds, "kg")
    _backward_parity(fsa, orc, w, ids1, None, r_ids1, None, "kg", with_h1=False)
    _sampled_parity(fsa, orc, w, 65536 + 37, 800, "kg (several seeds per wave)")


def test_citation_shape_two_hop_forward_bf16_wide_indptr(fsa, orc):
    """N=111M, ~1.6B edges, int64 indptr, x[N,128] bf16 (~28 GB), B=4096, fanouts [15,10]."""
    w, seeds = _build("citation")
    assert w.graph.num_nodes == 111_000_000 and w.graph.indptr.dtype == torch.int64
    assert w.graph.num_edges > 2**31 - 1 or abs(w.graph.num_edges / 1.6e9 - 1) < 0.05
    assert w.x.dtype == torch.bfloat16
    _forward_parity(fsa, orc, w, seeds, "citation")
    _sampled_parity(fsa, orc, w, 65536, 600, "citation (the benchmark's saturating batch)")


def test_row_offsets_beyond_32_bits(fsa, orc):
    """A CSR whose `indices` array has more than 2^31 entries: row starts need the int64 indptr
    path end to end (the citation shape stays just below 2^31 entries)."""
    from paper_2511_13645_amd import synth
    dev = "cuda:0"
    n, deg, D = 300_000, 7_400, 32
    E = n * deg
    assert E > 2**31
    indptr = torch.arange(0, E + 1, deg, dtype=torch.int64, device=dev)
    indices = torch.empty(E, dtype=torch.int32, device=dev)
    step = 1 << 28
    for e0 in range(0, E, step):
        e1 = min(E, e0 + step)
        idx = torch.arange(e0, e1, dtype=torch.int64, device=dev)
        indices[e0:e1] = (synth.hash64(7, 0, idx) % n).abs().to(torch.int32)
        del idx
    x = synth.features(n, D, seed=1, device=dev)
    # seeds from the top of the ID range, whose rows start beyond 2^31 (and 2^32 / 4 bytes)
    seeds = torch.cat([torch.arange(n - 300, n, dtype=torch.int32), synth.seed_batches(n, 212, 1, seed=2)[0]])
    assert int(indptr[seeds[0].item()].item()) > 2**31
    w = synth.Workload("wide", synth.Graph(indptr, indices, n), x, seeds.shape[0], (15, 10))
    _forward_parity(fsa, orc, w, seeds, "wide offsets")
    w1 = synth.Workload("wide", w.graph, x, seeds.shape[0], (20,))
    _forward_parity(fsa, orc, w1, seeds, "wide offsets 1-hop")


def test_products_shape_three_hop(fsa, orc):
    """The product-graph shape with a third hop (fanouts [15,10,5], B=1024): IDs of all three
    levels, per-slot counts, every mean and the gradient of the touched rows against the oracle."""
    from paper_2511_13645_amd import synth
    w, seeds = _build("products")
    g, x = w.graph, w.x
    N, D = x.shape
    fan = [15, 10, 5]
    r = fsa.fsa_sample_mean3_fwd(g.indptr, g.indices, x, seeds.cuda(), fan, w.sampler_seed)
    torch.cuda.synchronize()
    h_indptr, h_indices, hx = g.indptr.cpu().numpy(), g.indices.cpu().numpy(), x.cpu().numpy()
    t0 = time.time()
    ref = orc.sample_mean3_fwd(h_indptr, h_indices, hx, seeds.numpy(), fan, w.sampler_seed, want_h2=False)
    print("[products 3-hop] oracle forward %.1fs, %d leaf rows" % (time.time() - t0, int((ref["ids3"] >= 0).sum())), flush=True)
    for k in ("ids1", "ids2", "ids3", "cnt2"):
        assert_ids_equal(r[k], ref[k], "products 3-hop " + k)
    scale = orc.mean3_replay_fwd(np.abs(hx), ref["ids1"], ref["ids2"], ref["ids3"], want_h2=False)
    worst = max(assert_close(to_f64(r[k]), ref[k], scale[k], 1e-5, "products 3-hop " + k) for k in ("out", "out_h1", "out_m1"))
    print("[products 3-hop] ids bit-exact; worst relative error of the means %.2e" % worst, flush=True)
    B, k1 = ref["ids1"].shape
    gout = synth.upstream_grad((B, D), seed=3, device="cuda:0")
    gh1 = synth.upstream_grad((B, k1, D), seed=4, device="cuda:0")
    gx = torch.zeros((N, D), dtype=torch.float32, device="cuda:0")
    fsa.fsa_mean3_bwd(gout, r["ids1"], r["ids2"], r["ids3"], grad_h1=gh1, grad_x=gx)
    torch.cuda.synchronize()
    want = orc.mean3_bwd(to_f64(gout), ref["ids1"], ref["ids2"], ref["ids3"], grad_h1=to_f64(gh1), num_nodes=N)
    mag = orc.mean3_bwd(np.abs(to_f64(gout)), ref["ids1"], ref["ids2"], ref["ids3"], grad_h1=np.abs(to_f64(gh1)), num_nodes=N)
    touched = np.unique(ref["ids3"][ref["ids3"] >= 0])
    got = gx[torch.from_numpy(touched).cuda().long()].double().cpu().numpy()
    worst = assert_close(got, want[touched], mag[touched], 1e-5, "products 3-hop grad_x (touched rows)")
    total = float(gx.double().abs().sum().item())
    assert abs(total - np.abs(got).sum()) <= 1e-6 * max(1.0, total)
    print("[products 3-hop] grad_x over %d touched rows: worst relative error %.2e" % (touched.size, worst), flush=True)


def test_social_shape_backward_into_bf16_table(fsa, orc):
    """The dense social shape at full size with bf16 upstream gradients into a bf16 grad_x by
    packed atomics: within (n+1) * (2^-8 * sum|contribution| + 2^-133) of the oracle, n = number
    of additions into the row."""
    from paper_2511_13645_amd import synth
    w, seeds = _build("social")
    g, x = w.graph, w.x
    N, D = x.shape
    fan = list(w.fanouts)
    _, _, ids1, ids2 = fsa.fsa_sample_mean_fwd(g.indptr, g.indices, x, seeds.cuda(), fan, w.sampler_seed, emit_h1=False)
    B, k1 = ids1.shape
    gout = synth.upstream_grad((B, D), seed=3, device="cuda:0").to(torch.bfloat16)
    gh1 = synth.upstream_grad((B, k1, D), seed=4, device="cuda:0").to(torch.bfloat16)
    gx = torch.zeros((N, D), dtype=torch.bfloat16, device="cuda:0")
    fsa.fsa_mean_bwd_lp(gout, ids1, ids2, gh1, grad_x=gx)
    torch.cuda.synchronize()
    h1, h2 = ids1.cpu().numpy(), ids2.cpu().numpy()
    want = orc.mean_bwd(to_f64(gout), h1, h2, to_f64(gh1), num_nodes=N)
    mag = orc.mean_bwd(np.abs(to_f64(gout)), h1, h2, np.abs(to_f64(gh1)), num_nodes=N)
    n_add = np.bincount(h2[h2 >= 0], minlength=N).astype(np.float64)[:, None]
    err = np.abs(to_f64(gx) - want)
    bound = (n_add + 1.0) * (2.0 ** -8 * mag + 2.0 ** -133)
    assert (err <= bound).all(), "worst excess %g" % float((err - bound).max())
    assert (to_f64(gx)[n_add[:, 0] == 0] == 0).all()
    print("[social bf16 backward] worst error / bound %.3f over %d touched rows" %
          (float((err / np.maximum(bound, 1e-300)).max()), int((n_add > 0).sum())), flush=True)
