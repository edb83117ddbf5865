"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Sizes span several tiles, several splits and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import freeze_oracle as fo
from paper_2002_02645_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu

TIGHT = 1e-5   # tighter than the contract's 1e-4: the fp32 re-scoring is good to ~1e-6


def _host_entries(t: torch.Tensor) -> np.ndarray:
    return synth.bf16_bits(t) if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def run_lookup(entries, labels, queries, num_classes, k, thr, r=0):
    fc = binding.FreezeCache(1)
    try:
        fc.build_layer(0, entries.cuda().contiguous(), labels.cuda().contiguous(), num_classes)
        out = fc.lookup(0, queries.cuda().contiguous(), k, thr, r)
        torch.cuda.synchronize()
        return {key: v.cpu().numpy() for key, v in out.items()}
    finally:
        fc.close()


def check_case(entries, labels, queries, num_classes, k, thr, r=0, rel=TIGHT):
    got = run_lookup(entries, labels, queries, num_classes, k, thr, r)
    e_h, l_h, q_h = _host_entries(entries), labels.cpu().numpy(), queries.cpu().numpy()
    ref = parity.oracle_reference(q_h, e_h, l_h, num_classes, k, thr)
    near = parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, num_classes, k, thr, rel=rel, dist_rel=TIGHT)
    # the contract's own tolerance must hold as well
    parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, num_classes, k, thr)
    return got, ref, near


def test_config1_tiny_full_batch():
    wl = synth.WORKLOADS["c1_tiny"]
    data = synth.make_workload(wl)
    L = data.layers[0]
    got, ref, near = check_case(L.entries, L.labels, data.queries[0], 10, wl.k, wl.vote_thresholds[0])
    assert got["hit"].all() and (got["votes"] == 5).all()
    assert near < 64


def test_hand_example_on_gpu():
    ent = torch.tensor([[0, 0], [1, 0], [0, 2], [3, 0], [1, 0], [4, 4]], dtype=torch.float32)
    lab = torch.tensor([0, 0, 1, 1, 1, 0], dtype=torch.int32)
    q = torch.tensor([[1, 1], [1, 0]], dtype=torch.float32)
    for dt in (torch.float32, torch.bfloat16):
        got = run_lookup(ent.to(dt), lab, q, 2, 3, 2)
        assert got["idx"][0].tolist() == [1, 4, 0] and got["dist"][0].tolist() == [1.0, 1.0, 2.0]
        assert (got["label"][0], got["votes"][0], got["hit"][0]) == (0, 2, 1)
        got = run_lookup(ent.to(dt), lab, q, 2, 5, 4)
        assert got["idx"][0].tolist() == [1, 4, 0, 2, 3] and (got["label"][0], got["votes"][0], got["hit"][0]) == (1, 3, 0)
        got = run_lookup(ent.to(dt), lab, q, 2, 2, 1)
        assert got["idx"][1].tolist() == [1, 4] and got["dist"][1].tolist() == [0.0, 0.0]
        assert (got["label"][1], got["votes"][1]) == (0, 1)
        got = run_lookup(ent.to(dt), lab, q, 2, 6, 3)   # k = N
        assert got["idx"][0].tolist() == [1, 4, 0, 2, 3, 5] and (got["label"][0], got["votes"][0]) == (0, 3)


@pytest.mark.parametrize("n,d,b,k,r,dtype", [
    (777, 100, 37, 7, 0, torch.float32),      # nothing a multiple of a tile; d not a multiple of 8
    (777, 100, 37, 7, 0, torch.bfloat16),
    (5000, 1024, 600, 10, 0, torch.bfloat16),  # 3 query tiles (ragged), 20 cache tiles, several splits
    (3000, 256, 300, 10, 32, torch.bfloat16),  # R = 32 kernel variant
    (3000, 320, 130, 20, 64, torch.float32),   # R = 64 kernel variant (128-query tiles), k = 20
    (40, 64, 5, 40, 0, torch.bfloat16),        # k = N
    (300, 64, 1, 1, 0, torch.float32),         # batch 1, k = 1
    (1500, 192, 9, 33, 0, torch.bfloat16),     # k > 24 -> default R = 64
    (20000, 512, 8, 20, 0, torch.bfloat16),    # small-batch kernel, many tiles per workgroup
    (5000, 1024, 16, 10, 0, torch.bfloat16),   # small-batch kernel, longest supported activation
    (3000, 960, 3, 5, 0, torch.float32),       # small-batch kernel, fp32 cache, d not a multiple of 64
    (5000, 512, 4, 40, 0, torch.bfloat16),     # small-batch kernel, R = 64 and k > 32: the selection's fallbacks
    (3000, 100, 2, 5, 0, torch.float32),       # small-batch kernel, d not a multiple of 8
    (2000, 128, 5, 10, 0, torch.bfloat16),     # small-batch kernel, fewer workgroups than blocks to take
    (70000, 256, 16, 10, 0, torch.bfloat16),   # small-batch kernel, one tile per workgroup
    (3000, 1100, 3, 5, 0, torch.bfloat16),     # d too long for the small-batch kernel -> tiled kernel
    (3000, 2048, 100, 10, 0, torch.bfloat16),  # one query tile, long activation -> keys-out kernel + selection
    (2500, 4160, 200, 10, 64, torch.float32),  # keys-out, R = 64, fp32 cache, ragged everything
    (1000, 640, 20, 5, 0, torch.bfloat16),     # keys-out with few cache tiles
    (50000, 2048, 64, 10, 0, torch.bfloat16),  # keys-out, 196 cache tiles on 256 CUs: stream-K over (tile, k-step)
    (36000, 2080, 100, 10, 64, torch.float32), # stream-K, ragged d, workgroup ranges that span three tiles' parts
    (600, 16384, 40, 10, 0, torch.bfloat16),   # long activation, few queries: 1024-thread finishing blocks
    (600, 16392, 300, 10, 0, torch.float32),   # fused kernel, fp32 cache, long activation, d not a multiple of 64
    (5000, 128, 50, 48, 0, torch.bfloat16),    # a large k on the tiled kernel (R = 64)
    (5000, 128, 4, 48, 0, torch.float32),      # ... and on the small-batch kernel
    (5000, 128, 50, 64, 0, torch.bfloat16),    # k = R = 64: no spare candidate, the bf16 ranking alone gets the 64th wrong for some queries
    (5000, 128, 4, 64, 0, torch.float32),      # ... and on the small-batch kernel
    (1585, 6, 2140, 34, 63, torch.bfloat16),   # low-dimensional dense data: many entries within the bf16 rounding of the 34th neighbour
    (4000, 64, 300, 10, 0, torch.bfloat16),    # (see test_clusters_far_from_the_origin for this shape on offset data)
    (64, 128, 20, 64, 0, torch.bfloat16),      # k = n = the re-scoring width: every entry is a candidate
    (50000, 64, 10000, 10, 0, torch.bfloat16), # 40 x 196 tiles on 256 CUs: balanced decomposition, workgroups that serve two query tiles
    (33000, 96, 7000, 5, 0, torch.float32),    # balanced decomposition, ragged last query tile
    (4000, 512, 300, 5, 12, torch.bfloat16),   # R = 12: lists shorter than the kernel variant's 16 slots
    (4000, 512, 300, 9, 24, torch.float32),    # R = 24 on the 32-slot variant
    (1, 1, 3, 1, 0, torch.float32),            # a cache of one scalar entry
    (5, 3, 2, 2, 0, torch.bfloat16),           # a handful of short entries, small-batch kernel
    (7, 5, 40, 3, 0, torch.float32),           # ... and the tiled kernel (more queries than entries)
    (257, 33, 257, 4, 0, torch.bfloat16),      # one entry and one query past a tile
    (20000, 2048, 1800, 10, 0, torch.bfloat16),  # 8 x 79 tiles in 32 splits of 2 or 3 tiles, long rows
    (9000, 2112, 4000, 20, 0, torch.float32),    # 16 query tiles on the R = 32 variant, ragged d, fp32 cache
    (9000, 2048, 2000, 10, 64, torch.bfloat16),  # 16 query tiles on the R = 64 variant (128-query tiles)
    (2000000, 64, 300, 48, 0, torch.bfloat16),   # two million entries, the largest k
    (3000, 64, 100000, 10, 0, torch.bfloat16),   # a hundred thousand queries (391 query tiles)
    (1500000, 96, 16, 20, 0, torch.bfloat16),    # small-batch kernel at its largest batch, 1.5 million entries
    (120, 70000, 40, 10, 0, torch.bfloat16),     # activations longer than any benchmark layer
])
def test_shapes_against_oracle(n, d, b, k, r, dtype):
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b)
    spec = wl.layers[0]
    spec = type(spec)(n, d, 10, spec.sigma, relu=True, store_bf16=(dtype == torch.bfloat16))
    data = synth.make_workload(type(wl)(wl.name, (spec,), b, k, (max(1, k - 2),), r, 77 + n + d))
    L = data.layers[0]
    check_case(L.entries, L.labels, data.queries[0], 10, k, max(1, k - 2), r)


def _verdicts(fc):
    c = torch.zeros(3, dtype=torch.int64, device="cuda")
    binding.freeze_lookup_stats_attach(fc.ctx, c)
    return c


@pytest.mark.parametrize("b,store_bf16,n,d,k", [
    (300, True, 4000, 64, 10),      # fused kernel; most queries need the wider re-scoring or the exact scan
    (300, False, 4000, 64, 10),     # ... with the cache stored in fp32
    (6, True, 4000, 64, 10),        # small-batch kernel: few flagged queries, each scanned by many workgroups
    (3000, True, 20000, 64, 10),    # more flagged queries than the exact scan has workgroups: several per workgroup
    (40, True, 3000, 2048, 10),     # keys-out kernel, long rows: the scan's whole-block re-scoring
    (25, False, 2500, 4104, 5),     # ... fp32 cache, ragged depth
    (200, True, 5000, 96, 64),      # k = 64: the scan's lists at their longest
])
def test_clusters_far_from_the_origin(b, store_bf16, n, d, k):
    """Every coordinate offset by +100: the bf16 keys (|c|^2 - 2 q.c, both of order 10^6) cannot tell
    neighbours whose distances differ by a few units apart, so the coarse candidates miss true
    neighbours for many queries.  The certificate must notice every such query and the wider
    re-scoring or the exact scan must repair it: the results equal the oracle's."""
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=n, batch=b)
    spec = type(wl.layers[0])(n, d, 10, 1.0, store_bf16=store_bf16)
    thr = max(1, k - 2)
    data = synth.make_workload(type(wl)(wl.name, (spec,), b, k, (thr,), 0, 991))
    L = data.layers[0]
    ent = (L.entries.float() + 100.0).to(L.entries.dtype)
    q = data.queries[0] + 100.0
    e_h, l_h, q_h = _host_entries(ent), L.labels.numpy(), q.numpy()
    ref = parity.oracle_reference(q_h, e_h, l_h, 10, k, thr)
    fc = binding.FreezeCache(1)
    try:
        counters = _verdicts(fc)
        # 1. without centring: the plain bf16 copy cannot rank these entries, the slower paths must
        binding.freeze_set_centring(fc.ctx, 0)
        fc.build_layer(0, ent.cuda(), L.labels.cuda(), 10)
        out = fc.lookup(0, q.cuda(), k, thr)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        c = counters.cpu().numpy()
        parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, 10, k, thr, rel=TIGHT, dist_rel=TIGHT)
        assert c.sum() == b
        assert c[1] + c[2] > 0, "this input is meant to defeat the coarse ranking"
        # 2. the default: the library sees at build time that the mean dominates the spread and ranks
        #    relative to it; the same exact result, now without the slower paths (k = R leaves no spare)
        counters.zero_()
        binding.freeze_set_centring(fc.ctx, 1)
        fc.build_layer(0, ent.cuda(), L.labels.cuda(), 10)
        out = fc.lookup(0, q.cuda(), k, thr)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        c2 = counters.cpu().numpy()
        parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, 10, k, thr, rel=TIGHT, dist_rel=TIGHT)
        assert c2.sum() == b
        if k < 64:
            assert c2[0] >= 0.98 * b - 1 and c2[2] <= c[2], (c, c2)
    finally:
        fc.close()


def test_cascade_on_clusters_far_from_the_origin():
    """The cascade's later layers run on the device-side miss list: the flagged queries' positions go
    through that list on their way to the wider re-scoring and the exact scan."""
    wl = synth.scaled(synth.WORKLOADS["c4_cascade_noisy"], n=2500, d_div=512, batch=400)
    data = synth.make_workload(wl)
    nl = len(wl.layers)
    ents = [(L.entries.float() + 100.0).to(L.entries.dtype) for L in data.layers]
    qs = [q + 100.0 for q in data.queries]
    fc = binding.FreezeCache(nl)
    try:
        counters = _verdicts(fc)
        binding.freeze_set_centring(fc.ctx, 0)      # keep the plain copy: this test is about the slower paths
        for l, L in enumerate(data.layers):
            fc.build_layer(l, ents[l].cuda(), L.labels.cuda(), L.spec.num_classes)
        out = fc.lookup_cascade(list(range(nl)), [q.cuda() for q in qs], wl.k, list(wl.vote_thresholds), wl.rescore_r)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        c = counters.cpu().numpy()
    finally:
        fc.close()
    exp_l, exp_x, exp_h, _ = fo.cascade([q.numpy() for q in qs], [_host_entries(e) for e in ents],
                                        [L.labels.numpy() for L in data.layers],
                                        [L.spec.num_classes for L in data.layers], wl.k, wl.vote_thresholds)
    assert np.array_equal(got["exit_layer"], exp_x) and np.array_equal(got["label"], exp_l)
    assert got["hits_per_layer"].tolist() == exp_h.tolist()
    assert len(set(exp_x.tolist())) >= 3 and c[1] + c[2] > 0


@pytest.mark.parametrize("n,d,b,k,dtype", [
    (3000, 256, 300, 10, torch.bfloat16),    # fused kernel
    (20000, 512, 8, 20, torch.bfloat16),     # small-batch kernel (the queries are converted inside the streaming kernel)
    (2500, 4160, 100, 10, torch.float32),    # keys-out kernel, fp32 cache, ragged depth
])
def test_forced_centring_keeps_results_exact(n, d, b, k, dtype):
    # centring changes which copy the matrix cores rank with, never the answer
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b)
    spec = type(wl.layers[0])(n, d, 10, 0.8, relu=True, store_bf16=(dtype == torch.bfloat16))
    thr = max(1, k - 2)
    data = synth.make_workload(type(wl)(wl.name, (spec,), b, k, (thr,), 0, 5150 + n))
    L = data.layers[0]
    e_h, l_h, q_h = _host_entries(L.entries), L.labels.numpy(), data.queries[0].numpy()
    ref = parity.oracle_reference(q_h, e_h, l_h, 10, k, thr)
    fc = binding.FreezeCache(1)
    try:
        binding.freeze_set_centring(fc.ctx, 2)
        fc.build_layer(0, L.entries.cuda(), L.labels.cuda(), 10)
        out = fc.lookup(0, data.queries[0].cuda(), k, thr)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
    finally:
        fc.close()
    parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, 10, k, thr, rel=TIGHT, dist_rel=TIGHT)


@pytest.mark.parametrize("n,d,b,k,offset,dtype", [
    (3000, 4096, 300, 10, 0.0, torch.bfloat16),   # width 16: twelve candidates first, four more when unconfirmed
    (3000, 4096, 300, 10, 3.0, torch.float32),    # ... fp32 cache, a mean the automatic rule leaves alone
    (2500, 4104, 280, 20, 1.0, torch.bfloat16),   # width 32: 24 first, then 8; ragged depth
    (3000, 4096, 60, 10, 2.0, torch.bfloat16),    # one query tile: the keys-out selection in front of the same finish
])
def test_two_step_rescoring_on_dense_data(n, d, b, k, offset, dtype):
    """Long activations are re-scored in two steps (three quarters of the width, the rest only when
    the certificate over those does not confirm).  One dense Gaussian cloud: the distances of the
    k-th and the following neighbours are within the bf16 keys' noise of each other for some queries,
    so both outcomes occur: most queries are confirmed after the first step, and a few (2 to 33 of
    them in these cases, measured with the width set to the first step's alone) need the second."""
    g = torch.Generator().manual_seed(4242 + n + d + b)
    ent = (torch.randn(n, d, generator=g) + offset).to(dtype)
    lab = torch.randint(0, 10, (n,), generator=g, dtype=torch.int32)
    q = torch.randn(b, d, generator=g) * 0.7 + offset
    thr = max(1, k - 3)
    e_h, l_h, q_h = _host_entries(ent), lab.numpy(), q.numpy()
    ref = parity.oracle_reference(q_h, e_h, l_h, 10, k, thr)
    fc = binding.FreezeCache(1)
    try:
        counters = _verdicts(fc)
        fc.build_layer(0, ent.cuda(), lab.cuda(), 10)
        out = fc.lookup(0, q.cuda(), k, thr)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        c = counters.cpu().numpy()
    finally:
        fc.close()
    parity.assert_lookup_matches(got, ref, q_h, e_h, l_h, 10, k, thr, rel=TIGHT, dist_rel=TIGHT)
    assert c.sum() == b, c


@pytest.mark.parametrize("frac,scale,dtype", [
    (0.01, 100.0, torch.bfloat16),    # five channels in 512 a hundred times larger than the rest
    (0.004, 300.0, torch.float32),    # two channels three hundred times larger: they carry nearly all of every distance
])
def test_outlier_channels(frac, scale, dtype):
    """Activations with a few channels far larger than the others (common in trained networks): the
    distances are dominated by those channels, the bf16 keys resolve the rest poorly, and more
    queries need the wider re-scoring; the results stay the oracle's."""
    n, d, b, k = 4000, 512, 300, 10
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b)
    spec = type(wl.layers[0])(n, d, 10, 0.8, relu=True, store_bf16=(dtype == torch.bfloat16))
    data = synth.make_workload(type(wl)(wl.name, (spec,), b, k, (8,), 0, 31337))
    L = data.layers[0]
    g = torch.Generator().manual_seed(5)
    cols = torch.randperm(d, generator=g)[: max(1, int(d * frac))]
    ent = L.entries.float().clone()
    q = data.queries[0].clone()
    ent[:, cols] *= scale
    q[:, cols] *= scale
    check_case(ent.to(L.entries.dtype), L.labels, q, 10, k, 8)


@pytest.mark.parametrize("kind,dtype", [
    ("student_t2", torch.bfloat16),       # heavy tails: a few huge coordinates per row
    ("sparse", torch.bfloat16),           # 95 % zeros
    ("scale_1e6", torch.float32),         # large magnitudes (squares of 1e12 per coordinate)
    ("scale_1e-6", torch.bfloat16),       # small magnitudes
    ("binary", torch.float32),            # 0 / 1 entries: integer distances, many exact ties at the k-th place
    ("bytes", torch.bfloat16),            # integers 0 .. 255 (exact in bf16)
])
def test_value_distributions(kind, dtype):
    """Inputs unlike the benchmark's Gaussian clusters; every one must still give the oracle's answer
    (ties at the k-th place go by the entry index, which the certificate leaves to the wider re-scoring)."""
    g = torch.Generator().manual_seed(7)
    n, d, b, k = 6000, 768, 400, 10
    lab = torch.randint(0, 10, (n,), generator=g, dtype=torch.int32)
    cent = torch.randn(10, d, generator=g)
    ce, cq = cent[lab.long()], cent[torch.randint(0, 10, (b,), generator=g)]
    if kind == "student_t2":
        t = torch.distributions.StudentT(2.0)
        torch.manual_seed(11)
        e, q = ce + t.sample((n, d)), cq + t.sample((b, d))
    elif kind == "sparse":
        e, q = torch.relu(ce + torch.randn(n, d, generator=g) - 1.8), torch.relu(cq + torch.randn(b, d, generator=g) - 1.8)
    elif kind in ("scale_1e6", "scale_1e-6"):
        f = 1e6 if kind == "scale_1e6" else 1e-6
        e, q = (ce + 0.8 * torch.randn(n, d, generator=g)) * f, (cq + 0.8 * torch.randn(b, d, generator=g)) * f
    elif kind == "binary":
        e, q = (torch.rand(n, d, generator=g) < 0.3).float(), (torch.rand(b, d, generator=g) < 0.3).float()
    else:
        e, q = torch.randint(0, 256, (n, d), generator=g).float(), torch.randint(0, 256, (b, d), generator=g).float()
    check_case(e.to(dtype), lab, q, 10, k, 8)


def test_certificate_verdicts_on_clustered_data():
    # the paper's kind of input: nearly every query is confirmed after the first re-scoring
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=20000, d_div=4, batch=2000)
    data = synth.make_workload(wl)
    L = data.layers[0]
    fc = binding.FreezeCache(1)
    try:
        counters = _verdicts(fc)
        fc.build_layer(0, L.entries.cuda(), L.labels.cuda(), 10)
        fc.lookup(0, data.queries[0].cuda(), wl.k, wl.vote_thresholds[0])
        torch.cuda.synchronize()
        c = counters.cpu().numpy()
        binding.freeze_lookup_stats_attach(fc.ctx, None)
        fc.lookup(0, data.queries[0].cuda(), wl.k, wl.vote_thresholds[0])
        torch.cuda.synchronize()
        assert np.array_equal(counters.cpu().numpy(), c)     # detached: no longer counted
    finally:
        fc.close()
    assert c.sum() == 2000 and c[0] >= 1900 and c[2] <= 5, c


def test_random_labels_and_duplicates():
    # labels independent of geometry: votes span 1..k and label ties occur; duplicate rows: exact ties
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=900, batch=120)
    data = synth.make_workload(wl)
    L = data.layers[0]
    ent = L.entries.clone()
    ent[500:520] = ent[100:120]            # exact duplicates: lower index must come first
    lab = synth.random_labels(900, 4, 5)
    q = data.queries[0].clone()
    q[:20] = ent[100:120]                  # queries identical to cached rows: distance exactly 0
    got, ref, _ = check_case(ent, lab, q, 4, 7, 4)
    assert (got["dist"][:20, 0] == 0.0).all() and (got["dist"][:20, 1] == 0.0).all()
    assert got["idx"][:20, 0].tolist() == list(range(100, 120))
    assert got["idx"][:20, 1].tolist() == list(range(500, 520))
    assert len(set(got["votes"].tolist())) >= 3
    assert (got["dist"] >= 0).all()


def test_threshold_monotone_and_extremes():
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=600, batch=64)
    data = synth.make_workload(wl)
    L = data.layers[0]
    lab = synth.random_labels(600, 3, 9)
    prev = None
    for thr in range(1, 6):
        got = run_lookup(L.entries, lab, data.queries[0], 3, 5, thr)
        if prev is not None:
            assert (got["hit"] <= prev).all()
        prev = got["hit"]
        assert np.array_equal(got["hit"], (got["votes"] >= thr).astype(np.uint8))
        if thr == 1:
            assert got["hit"].all()


def test_results_are_deterministic():
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=4000, d_div=16, batch=300)
    data = synth.make_workload(wl)
    L = data.layers[0]
    a = run_lookup(L.entries, L.labels, data.queries[0], 10, 10, 8)
    b = run_lookup(L.entries, L.labels, data.queries[0], 10, 10, 8)
    for key in a:
        assert np.array_equal(a[key], b[key]), key


def test_compact_misses_against_oracle():
    rng = np.random.default_rng(3)
    for count in (0, 1, 63, 64, 1023, 1024, 1025, 10000):
        hit = (rng.random(count) < 0.37).astype(np.uint8)
        sel = rng.permutation(max(count, 1) * 3)[:count].astype(np.int32)
        for use_sel in (True, False):
            hit_d = torch.from_numpy(hit).cuda()
            sel_d = torch.from_numpy(sel).cuda() if use_sel else None
            out = torch.full((max(count, 1),), -7, dtype=torch.int32, device="cuda")
            cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
            binding.freeze_compact_misses(hit_d, sel_d, out, cnt)
            torch.cuda.synchronize()
            exp = fo.compact(hit, sel if use_sel else np.arange(count, dtype=np.int32))
            assert int(cnt.item()) == exp.size
            assert np.array_equal(out.cpu().numpy()[:exp.size], exp)


def _cascade_case(wl_name, n, d_div, batch, thresholds=None):
    wl = synth.scaled(synth.WORKLOADS[wl_name], n=n, d_div=d_div, batch=batch)
    if thresholds is not None:
        wl = type(wl)(wl.name, wl.layers, wl.batch, wl.k, tuple(thresholds), wl.rescore_r, wl.seed)
    data = synth.make_workload(wl)
    nl = len(wl.layers)
    fc = binding.FreezeCache(nl)
    try:
        for l, L in enumerate(data.layers):
            fc.build_layer(l, L.entries.cuda(), L.labels.cuda(), L.spec.num_classes)
        qs = [q.cuda() for q in data.queries]
        out = fc.lookup_cascade(list(range(nl)), qs, wl.k, list(wl.vote_thresholds), wl.rescore_r)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
    finally:
        fc.close()
    exp_l, exp_x, exp_h, _ = fo.cascade([q.numpy() for q in data.queries],
                                        [_host_entries(L.entries) for L in data.layers],
                                        [L.labels.numpy() for L in data.layers],
                                        [L.spec.num_classes for L in data.layers], wl.k, wl.vote_thresholds)
    return got, exp_l, exp_x, exp_h


def test_cascade_against_oracle_noisy():
    got, exp_l, exp_x, exp_h = _cascade_case("c4_cascade_noisy", 2000, 64, 700)
    assert np.array_equal(got["exit_layer"], exp_x)
    assert np.array_equal(got["label"], exp_l)
    assert got["hits_per_layer"].tolist() == exp_h.tolist()
    assert len(set(exp_x.tolist())) >= 3                      # requests freeze at several layers
    assert got["hits_per_layer"].sum() + (got["exit_layer"] == -1).sum() == 700


def test_cascade_with_fall_through():
    # unanimity demanded at every layer: many requests hit nowhere and fall through (-1, -1)
    got, exp_l, exp_x, exp_h = _cascade_case("c4_cascade_noisy", 1800, 64, 333, thresholds=(10, 10, 10, 10))
    assert np.array_equal(got["exit_layer"], exp_x) and np.array_equal(got["label"], exp_l)
    assert got["hits_per_layer"].tolist() == exp_h.tolist()
    assert (exp_x == -1).any() and (exp_x >= 0).any()
    assert (got["label"][exp_x == -1] == -1).all()


def test_cascade_against_oracle_clean():
    got, exp_l, exp_x, exp_h = _cascade_case("c4_cascade", 1500, 64, 300)
    assert np.array_equal(got["exit_layer"], exp_x) and np.array_equal(got["label"], exp_l)
    assert got["hits_per_layer"].tolist() == exp_h.tolist()


def test_argument_errors_launch_nothing():
    fc = binding.FreezeCache(2)
    try:
        ent = torch.randn(100, 32, device="cuda")
        lab = torch.zeros(100, dtype=torch.int32, device="cuda")
        fc.build_layer(0, ent, lab, 3)
        q = torch.randn(4, 32, device="cuda")
        out = fc.alloc_outputs(4, 5)
        for key in out:
            out[key].fill_(42)
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")

        def call(layer=0, k=5, thr=3, r=0, wsz=None):
            return binding.lib().freeze_lookup(fc.ctx, layer, q.data_ptr(), 4, k, thr, r, out["label"].data_ptr(),
                                               out["hit"].data_ptr(), out["votes"].data_ptr(), out["idx"].data_ptr(),
                                               out["dist"].data_ptr(), ws.data_ptr(),
                                               ws.numel() if wsz is None else wsz, None)
        assert call(layer=5) == binding.FREEZE_ELAYER
        assert call(layer=1) == binding.FREEZE_ENOTBUILT
        assert call(k=0) == binding.FREEZE_EINVAL
        assert call(k=101) == binding.FREEZE_EINVAL
        assert call(k=65, thr=3) == binding.FREEZE_EINVAL      # above the largest k (the cache has 100 entries)
        assert call(thr=0) == binding.FREEZE_EINVAL
        assert call(thr=6) == binding.FREEZE_EINVAL
        assert call(r=3) == binding.FREEZE_EINVAL
        assert call(r=65) == binding.FREEZE_EINVAL
        assert call(wsz=16) == binding.FREEZE_EWORKSPACE
        torch.cuda.synchronize()
        for key in out:
            assert (out[key] == 42).all()    # nothing was written
        assert call() == binding.FREEZE_OK
        torch.cuda.synchronize()
    finally:
        fc.close()


def test_empty_batch_and_stage_timing():
    fc = binding.FreezeCache(2)
    try:
        ent = torch.randn(300, 64, device="cuda")
        lab = torch.zeros(300, dtype=torch.int32, device="cuda")
        fc.build_layer(0, ent, lab, 2)
        fc.build_layer(1, ent.to(torch.bfloat16), lab, 2)
        # b == 0: a no-op that still succeeds
        q0 = torch.empty((0, 64), dtype=torch.float32, device="cuda")
        out = fc.lookup(0, q0, 3, 2)
        assert out["idx"].shape == (0, 3)
        oc = fc.lookup_cascade([0, 1], [q0, q0], 3, [2, 2])
        torch.cuda.synchronize()
        assert oc["hits_per_layer"].tolist() == [0, 0]
        # stage timing covers exactly the recorded look-ups and clears itself
        q = torch.randn(40, 64, device="cuda")
        binding.freeze_profile_enable(fc.ctx, True)
        fc.lookup(0, q, 3, 2)
        fc.lookup_cascade([0, 1], [q, q], 3, [3, 3])
        calls = binding.freeze_profile_read_calls(fc.ctx)
        assert len(calls) == 3 and all(len(c) == 3 and min(c) >= 0.0 for c in calls)
        ms, n = binding.freeze_profile_read(fc.ctx)
        assert n == 0 and ms == [0.0, 0.0, 0.0]
        binding.freeze_profile_enable(fc.ctx, False)
        fc.lookup(0, q, 3, 2)
        assert binding.freeze_profile_read(fc.ctx)[1] == 0
        # the sampled mode brackets the distance pass of every eighth look-up, the first included
        binding.freeze_profile_enable(fc.ctx, 3)
        for _ in range(17):
            fc.lookup(0, q, 3, 2)
        calls = binding.freeze_profile_read_calls(fc.ctx)
        assert len(calls) == 3 and all(c[0] == 0.0 and c[1] > 0.0 and c[2] == 0.0 for c in calls)
        binding.freeze_profile_enable(fc.ctx, False)
    finally:
        fc.close()


def test_cascade_single_tile_and_rebuild():
    # a cascade over few requests (one query tile), and rebuilding a layer replaces its cache
    got, exp_l, exp_x, exp_h = _cascade_case("c4_cascade_noisy", 700, 128, 9)
    assert np.array_equal(got["exit_layer"], exp_x) and np.array_equal(got["label"], exp_l)
    fc = binding.FreezeCache(1)
    try:
        a = torch.randn(200, 32, device="cuda")
        b2 = torch.randn(260, 32, device="cuda") + 5.0
        lab_a = torch.zeros(200, dtype=torch.int32, device="cuda")
        lab_b = torch.ones(260, dtype=torch.int32, device="cuda")
        q = torch.randn(10, 32, device="cuda") + 5.0
        fc.build_layer(0, a, lab_a, 2)
        o1 = fc.lookup(0, q, 3, 2)
        torch.cuda.synchronize()
        assert (o1["label"] == 0).all()
        fc.build_layer(0, b2, lab_b, 2)
        o2 = fc.lookup(0, q, 3, 2)
        torch.cuda.synchronize()
        assert (o2["label"] == 1).all() and (o2["idx"] < 260).all()
    finally:
        fc.close()


def test_calibration_microbenchmarks():
    scratch = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
    tf, mhz = binding.freeze_calibrate_mfma(scratch)
    assert 300.0 < tf < 2600.0 and 500.0 < mhz < 3000.0      # below the published 2.5 PFLOP/s, above a tenth of it
    buf = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
    gbs = binding.freeze_calibrate_hbm_read(buf)
    assert 1000.0 < gbs < 8100.0                               # below the published 8 TB/s
    assert (buf[:64] == 0).all()
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    assert binding.lib().freeze_calibrate_mfma(tiny.data_ptr(), 16, None, None) == binding.FREEZE_EINVAL
