"""Pins for the CPU oracle: each checks it against something other than itself
(a hand-worked example, closed forms, exact integer brute force, a library
routine on a special case, invariants), so that a dropped term, a wrong sign or
index, a transposed operand or a wrong tie-break fails at least one of them."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import freeze_oracle as fo
from paper_2002_02645_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _hand_example():
    entries, cases, hits, confs = [], [], [], []
    with open(os.path.join(GOLDEN, "hand_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            kind, rest = line.split(" ", 1)
            if kind == "entry":
                i, x, y, lab = (int(v) for v in rest.split())
                assert i == len(entries)
                entries.append((x, y, lab))
            elif kind == "case":
                parts = [p.split() for p in rest.split("|")]
                qx, qy, k = (int(v) for v in parts[0])
                cases.append((qx, qy, k, [int(v) for v in parts[1]], [float(v) for v in parts[2]],
                              int(parts[3][0]), int(parts[3][1])))
            elif kind == "hit":
                hits.append(tuple(int(v) for v in rest.split()))
            elif kind == "conf":
                parts = [p.split() for p in rest.split("|")]
                qx, qy, k = (int(v) for v in parts[0])
                confs.append((qx, qy, k, {int(p[0]): float(p[1]) for p in parts[1:]}))
    ent = np.array([[e[0], e[1]] for e in entries], dtype=np.float32)
    lab = np.array([e[2] for e in entries], dtype=np.int32)
    return ent, lab, cases, hits, confs


def test_hand_example_neighbours_votes_hits():
    ent, lab, cases, hits, _ = _hand_example()
    for qx, qy, k, idx, d2, label, votes in cases:
        q = np.array([[qx, qy]], dtype=np.float32)
        r = fo.lookup(q, ent, lab, 2, k, 1)
        assert r["idx"][0].tolist() == idx
        assert r["sqdist"][0].tolist() == d2
        assert (int(r["label"][0]), int(r["votes"][0])) == (label, votes)
    for qx, qy, k, thr, hit in hits:
        q = np.array([[qx, qy]], dtype=np.float32)
        r = fo.lookup(q, ent, lab, 2, k, thr)
        assert int(r["hit"][0]) == hit


def test_hand_example_bf16_storage_gives_same_result():
    ent, lab, cases, _, _ = _hand_example()
    bits = synth.bf16_bits(torch.from_numpy(ent).to(torch.bfloat16))   # small integers: exact in bf16
    for qx, qy, k, idx, d2, label, votes in cases:
        q = np.array([[qx, qy]], dtype=np.float32)
        r = fo.lookup(q, bits, lab, 2, k, 1)
        assert r["idx"][0].tolist() == idx and r["sqdist"][0].tolist() == d2


def test_hand_example_confidence():
    ent, lab, _, _, confs = _hand_example()
    for qx, qy, k, per_label in confs:
        q = np.array([[qx, qy]], dtype=np.float32)
        idx, d2, _ = fo.knn(q, ent, k)
        label, conf = fo.confidence(lab, idx, d2, 2)
        best = max(per_label, key=lambda c: per_label[c])
        assert int(label[0]) == best
        assert conf[0] == pytest.approx(per_label[best], rel=1e-6)
    # a neighbour at distance zero makes the confidence infinite (identical output => same label)
    q = np.array([[1, 0]], dtype=np.float32)
    idx, d2, _ = fo.knn(q, ent, 2)
    label, conf = fo.confidence(lab, idx, d2, 2)
    assert math.isinf(conf[0])


def _confidence_by_hand(labels, idx, d2, k):
    """The heuristic of Sec. 3 written out with dictionaries: an independent restatement used
    only on tiny inputs."""
    share, inv = {}, {}
    for i, dd in zip(idx, d2):
        c = int(labels[i])
        share[c] = share.get(c, 0) + 1
        inv[c] = inv.get(c, 0.0) + (math.inf if dd == 0 else 1.0 / math.sqrt(dd))
    conf = {c: (share[c] / k) * inv[c] for c in share}
    best = min(conf, key=lambda c: (-conf[c], c))
    return best, conf[best]


def test_confidence_closed_forms():
    # k = 1: the confidence is the reciprocal distance of the nearest entry
    ent = np.array([[3, 4], [6, 8], [0, 10]], dtype=np.float32)
    lab = np.array([2, 1, 0], dtype=np.int32)
    r = fo.lookup_confidence(np.zeros((1, 2), np.float32), ent, lab, 3, 1, 0.1)
    assert int(r["label"][0]) == 2 and r["conf"][0] == np.float32(0.2) and int(r["hit"][0]) == 1
    # strict comparison: a confidence equal to the threshold is a miss
    r = fo.lookup_confidence(np.zeros((1, 2), np.float32), ent, lab, 3, 1, float(np.float32(0.2)))
    assert int(r["hit"][0]) == 0
    # k neighbours of one label, all at distance rho: C = (k/k) * k / rho
    rho, k = 4.0, 6
    ring = np.array([[rho, 0, 0], [-rho, 0, 0], [0, rho, 0], [0, -rho, 0], [0, 0, rho], [0, 0, -rho], [50, 50, 50]],
                    dtype=np.float32)
    r = fo.lookup_confidence(np.zeros((1, 3), np.float32), ring, np.array([1] * 6 + [0], np.int32), 2, k, 0.0)
    assert int(r["label"][0]) == 1 and r["conf"][0] == np.float32(k / rho)
    # closeness beats plurality: two neighbours of label 0 at distance 1, three of label 1 at 10
    ent = np.array([[1, 0], [-1, 0], [10, 0], [-10, 0], [0, 10]], dtype=np.float32)
    lab = np.array([0, 0, 1, 1, 1], dtype=np.int32)
    r = fo.lookup_confidence(np.zeros((1, 2), np.float32), ent, lab, 2, 5, 0.5)
    assert int(r["label"][0]) == 0 and r["conf"][0] == pytest.approx(0.8, rel=1e-6)
    assert fo.lookup(np.zeros((1, 2), np.float32), ent, lab, 2, 5, 3)["label"][0] == 1
    # equal confidences: the smaller label id
    ent = np.array([[2, 0], [-2, 0]], dtype=np.float32)
    r = fo.lookup_confidence(np.zeros((1, 2), np.float32), ent, np.array([5, 3], np.int32), 6, 2, 0.0)
    assert int(r["label"][0]) == 3 and r["conf"][0] == np.float32(0.25)


def test_confidence_scales_inversely_with_distance_and_matches_restatement():
    rng = np.random.default_rng(11)
    ent = rng.integers(-9, 10, size=(60, 5)).astype(np.float32)
    lab = rng.integers(0, 4, size=60).astype(np.int32)
    q = rng.integers(-9, 10, size=(12, 5)).astype(np.float32) + 0.5   # no zero distances
    k = 7
    r1 = fo.lookup_confidence(q, ent, lab, 4, k, 0.0)
    r2 = fo.lookup_confidence(2 * q, 2 * ent, lab, 4, k, 0.0)            # distances double exactly
    assert np.array_equal(r1["idx"], r2["idx"]) and np.array_equal(r1["label"], r2["label"])
    idx, d2, _ = fo.knn(q, ent, k)
    _, c1 = fo.confidence(lab, idx, d2, 4)
    _, c2 = fo.confidence(lab, idx, 4 * d2, 4)
    assert np.array_equal(c1, 2 * c2)
    for i in range(q.shape[0]):
        best, conf = _confidence_by_hand(lab, idx[i], d2[i], k)
        assert int(r1["label"][i]) == best
        assert r1["conf"][i] == pytest.approx(conf, rel=1e-6)


def _threshold_problem(seed):
    rng = np.random.default_rng(seed)
    spec = [(40, 6), (40, 4), (40, 3)]
    ents = [rng.normal(size=(n, d)).astype(np.float32) for n, d in spec]
    labs = [rng.integers(0, 3, size=n).astype(np.int32) for n, _ in spec]
    val = [rng.normal(size=(25, d)).astype(np.float32) for _, d in spec]
    y = rng.integers(0, 3, size=25).astype(np.int32)
    return ents, labs, val, y


def test_compute_thresholds_is_max_confidence_of_wrong_lookups_and_gives_zero_validation_error():
    ents, labs, val, y = _threshold_problem(5)
    k = 5
    thr = fo.compute_thresholds(val, ents, labs, [3, 3, 3], k, y)
    assert thr.dtype == np.float32 and thr.shape == (3,)
    for l in range(3):
        idx, d2, _ = fo.knn(val[l], ents[l], k)
        wrong = []
        for i in range(25):
            best, conf = _confidence_by_hand(labs[l], idx[i], d2[i], k)
            if best != y[i]:
                wrong.append(conf)
        assert wrong, "the random labels must produce wrong look-ups"
        assert thr[l] == pytest.approx(max(wrong), rel=1e-6)
    # Sec. 3.1: with these thresholds no validation item is frozen with a label other than the model's
    out_l, out_x, hits = fo.cascade_confidence(val, ents, labs, [3, 3, 3], k, thr)
    frozen = out_x >= 0
    assert np.array_equal(out_l[frozen], y[frozen])
    assert hits.sum() == frozen.sum()
    # no wrong look-up anywhere -> thresholds stay at 0
    own = [labs[l][fo.knn(val[l], ents[l], 1)[0][:, 0]] for l in range(3)]
    assert fo.compute_thresholds(val[:1], ents[:1], labs[:1], [3], 1, own[0])[0] == 0.0


def test_cascade_confidence_exit_is_first_layer_above_threshold():
    ents, labs, val, _ = _threshold_problem(9)
    k = 4
    per = [fo.lookup_confidence(val[l], ents[l], labs[l], 3, k, 0.0) for l in range(3)]
    thr = [float(np.median(per[l]["conf"])) for l in range(3)]
    out_l, out_x, hits = fo.cascade_confidence(val, ents, labs, [3, 3, 3], k, thr)
    seen = set()
    for i in range(25):
        above = [l for l in range(3) if per[l]["conf"][i] > np.float32(thr[l])]
        exp = above[0] if above else -1
        seen.add(exp)
        assert out_x[i] == exp
        assert out_l[i] == (per[exp]["label"][i] if exp >= 0 else -1)
    assert len(seen) >= 3
    assert [int(h) for h in hits] == [int((out_x == l).sum()) for l in range(3)]


def test_lattice_closed_form():
    # entries c_n = (n, n, ..., n) in d dims, query (x, ..., x): D = d * (x - n)^2 exactly.
    n, d, k = 41, 7, 6
    ent = np.repeat(np.arange(n, dtype=np.float32)[:, None], d, axis=1)
    for x in (0.0, 3.25, 17.5, 40.0, 55.0, -2.0):
        q = np.full((1, d), x, dtype=np.float32)
        idx, d2, _ = fo.knn(q, ent, k)
        order = sorted(range(n), key=lambda i: ((x - i) ** 2, i))[:k]
        assert idx[0].tolist() == order
        assert d2[0].tolist() == [d * (x - i) ** 2 for i in order]


def test_exact_integer_bruteforce():
    # small integer coordinates: exact integer arithmetic in pure Python is the ground truth
    rng = np.random.default_rng(5)
    n, d, b, k = 37, 5, 9, 8
    ent = rng.integers(-3, 4, size=(n, d))
    qs = rng.integers(-3, 4, size=(b, d))
    idx, d2, _ = fo.knn(qs.astype(np.float32), ent.astype(np.float32), k)
    for i in range(b):
        D = [sum((int(qs[i, t]) - int(ent[r, t])) ** 2 for t in range(d)) for r in range(n)]
        order = sorted(range(n), key=lambda r: (D[r], r))[:k]
        assert idx[i].tolist() == order          # many exact ties: the lower index must come first
        assert d2[i].tolist() == [float(D[r]) for r in order]


def test_against_cdist_and_stable_argsort():
    # special case that reduces to library routines: pairwise distances + stable sort, fp64
    g = torch.Generator().manual_seed(11)
    ent = torch.randn(300, 33, generator=g)
    qs = torch.randn(17, 33, generator=g)
    k = 12
    idx, d2, _ = fo.knn(qs.numpy(), ent.numpy(), k)
    ref = torch.cdist(qs.double(), ent.double(), compute_mode="donot_use_mm_for_euclid_dist") ** 2
    order = torch.argsort(ref, dim=1, stable=True)[:, :k]
    assert np.array_equal(idx, order.numpy().astype(np.int32))
    np.testing.assert_allclose(d2, torch.gather(ref, 1, order).numpy(), rtol=1e-12)


def test_query_equal_to_entry_is_rank_one_at_zero_and_lowest_duplicate():
    g = torch.Generator().manual_seed(3)
    ent = torch.randn(50, 16, generator=g)
    ent[31] = ent[7]                      # duplicate rows: the lower index must be reported first
    idx, d2, _ = fo.knn(ent.numpy(), ent.numpy(), 2)
    for r in range(50):
        first = 7 if r == 31 else r
        assert idx[r, 0] == first and d2[r, 0] == 0.0
    assert idx[7, 1] == 31 and d2[7, 1] == 0.0
    assert (d2 >= 0).all()


def test_distance_symmetric_bitwise():
    g = torch.Generator().manual_seed(4)
    a = torch.randn(20, 40, generator=g).numpy()
    _, dab, _ = fo.knn(a, a, 20)
    idx, _, _ = fo.knn(a, a, 20)
    full = np.zeros((20, 20))
    for i in range(20):
        full[i, idx[i]] = dab[i]
    assert np.array_equal(full, full.T)


def test_permutation_invariance():
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=400, batch=23)
    data = synth.make_workload(wl)
    ent = data.layers[0].entries.numpy()
    lab = data.layers[0].labels.numpy()
    q = data.queries[0].numpy()
    perm = np.random.default_rng(8).permutation(ent.shape[0])
    r0 = fo.lookup(q, ent, lab, 10, 5, 4)
    r1 = fo.lookup(q, ent[perm], lab[perm], 10, 5, 4)
    assert np.array_equal(perm[r1["idx"]], r0["idx"])
    assert np.array_equal(r0["sqdist"], r1["sqdist"])
    for key in ("label", "votes", "hit"):
        assert np.array_equal(r0[key], r1[key])


def test_vote_counts_ties_and_threshold_monotone():
    n, k, ncls, b = 500, 7, 4, 200
    labels = synth.random_labels(n, ncls, 21).numpy()
    rng = np.random.default_rng(2)
    nbr = np.stack([rng.choice(n, size=k, replace=False) for _ in range(b)]).astype(np.int32)
    prev_hit = None
    saw_tie = False
    for thr in range(1, k + 2):
        lab, votes, hit = fo.vote(labels, nbr, ncls, thr)
        for i in range(b):
            counts = np.bincount(labels[nbr[i]], minlength=ncls)
            assert counts.sum() == k
            assert votes[i] == counts.max()
            winners = np.flatnonzero(counts == counts.max())
            saw_tie |= len(winners) > 1
            assert lab[i] == winners[0]            # equal counts: the smaller label id
            assert hit[i] == (counts.max() >= thr)
        if prev_hit is not None:
            assert (hit <= prev_hit).all()         # raising the threshold never creates a hit
        prev_hit = hit
    assert saw_tie
    lab, votes, hit = fo.vote(labels, nbr, ncls, 1)
    assert hit.all()
    lab, votes, hit = fo.vote(labels, nbr, ncls, k + 1)
    assert not hit.any()


def test_k_equals_n_returns_every_index_once_sorted():
    g = torch.Generator().manual_seed(6)
    ent = torch.randn(64, 9, generator=g).numpy()
    q = torch.randn(3, 9, generator=g).numpy()
    idx, d2, _ = fo.knn(q, ent, 64)
    for i in range(3):
        assert sorted(idx[i].tolist()) == list(range(64))
        assert (np.diff(d2[i]) >= 0).all()


def test_bf16_bits_widen_exactly():
    g = torch.Generator().manual_seed(9)
    ent = torch.randn(200, 24, generator=g).to(torch.bfloat16)
    q = torch.randn(10, 24, generator=g).numpy()
    i0, d0, _ = fo.knn(q, ent.float().numpy(), 6)
    i1, d1, _ = fo.knn(q, synth.bf16_bits(ent), 6)
    assert np.array_equal(i0, i1) and np.array_equal(d0, d1)


def test_thread_count_does_not_change_results():
    g = torch.Generator().manual_seed(10)
    ent = torch.randn(300, 20, generator=g).numpy()
    q = torch.randn(33, 20, generator=g).numpy()
    i1, d1, u1 = fo.knn(q, ent, 5, nthreads=1)
    i4, d4, u4 = fo.knn(q, ent, 5, nthreads=4)
    assert u1 == 1 and u4 == 4
    assert np.array_equal(i1, i4) and np.array_equal(d1, d4)


def test_same_class_distance_closed_form():
    # E[d^2] between two draws of one class = 2 sigma^2 d; across classes add |mu_a - mu_b|^2 ~ 2 d
    wl = synth.WORKLOADS["c1_tiny"]
    data = synth.make_workload(wl)
    L = data.layers[0]
    r = fo.lookup(data.queries[0].numpy(), L.entries.numpy(), L.labels.numpy(), 10, 5, 4)
    sigma, d = L.spec.sigma, L.spec.d
    assert abs(r["sqdist"].mean() / (2 * sigma * sigma * d) - 1.0) < 0.15
    # all five neighbours share the query's class: unanimous votes, every lookup hits
    assert (r["label"] == data.query_classes.numpy()).all()
    assert (r["votes"] == 5).all() and r["hit"].all()


def test_compact_matches_boolean_mask():
    rng = np.random.default_rng(12)
    hit = (rng.random(1000) < 0.4).astype(np.uint8)
    sel = rng.permutation(5000)[:1000].astype(np.int32)
    out = fo.compact(hit, sel)
    assert np.array_equal(out, sel[hit == 0])
    assert fo.compact(np.ones(5, np.uint8), np.arange(5, dtype=np.int32)).size == 0
    assert fo.compact(np.zeros(0, np.uint8), np.zeros(0, np.int32)).size == 0


def test_cascade_exit_is_first_hitting_layer():
    wl = synth.scaled(synth.WORKLOADS["c4_cascade_noisy"], n=600, d_div=128, batch=60)
    data = synth.make_workload(wl)
    qs = [q.numpy() for q in data.queries]
    es = [synth.bf16_bits(L.entries) for L in data.layers]
    labs = [L.labels.numpy() for L in data.layers]
    ncls = [L.spec.num_classes for L in data.layers]
    label, exit_layer, hits, _ = fo.cascade(qs, es, labs, ncls, wl.k, wl.vote_thresholds)
    per = [fo.lookup(qs[l], es[l], labs[l], ncls[l], wl.k, wl.vote_thresholds[l]) for l in range(len(qs))]
    for i in range(wl.batch):
        hitting = [l for l in range(len(qs)) if per[l]["hit"][i]]
        if hitting:
            assert exit_layer[i] == hitting[0] and label[i] == per[hitting[0]]["label"][i]
        else:
            assert exit_layer[i] == -1 and label[i] == -1
    assert hits.tolist() == [int((exit_layer == l).sum()) for l in range(len(qs))]
    assert 0 < (exit_layer == -1).sum() + (exit_layer > 0).sum()   # the noisy variant does forward misses
    # the miss list after layer 0 is the ascending ids not frozen there
    miss0 = fo.compact(per[0]["hit"], np.arange(wl.batch, dtype=np.int32))
    assert miss0.tolist() == [i for i in range(wl.batch) if not per[0]["hit"][i]]


def test_invalid_arguments_are_rejected():
    ent = np.zeros((4, 3), np.float32)
    q = np.zeros((1, 3), np.float32)
    with pytest.raises(ValueError):
        fo.knn(q, ent, 5)      # k > n
    with pytest.raises(ValueError):
        fo.knn(q, ent, 0)


def test_table1_arithmetic_gives_the_layer_sizes():
    vals = {}
    with open(os.path.join(GOLDEN, "table1_memory.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    # fp32, 40,000 points per layer, two blocks each of 64x32x32, 128x16x16, 256x8x8, 512x4x4
    floats_per_point = 2 * (64 * 32 * 32 + 128 * 16 * 16 + 256 * 8 * 8 + 512 * 4 * 4)
    mib = vals["cached_points_per_layer"] * 4 * floats_per_point / 2 ** 20
    assert mib == vals["knn_without_dimensionality_reduction_MB"]
    dims = {l.d for l in synth.WORKLOADS["c4_cascade"].layers} | {synth.WORKLOADS["c2_batched"].layers[0].d}
    assert {65536, 32768, 16384, 8192} <= dims


# ---------------------------------------------------------------------------------------------
# k-means cache (Sec. 4): the oracle's Lloyd iterations, majority labels / fractions and look-up
# ---------------------------------------------------------------------------------------------
def test_kmeans_hand_example():
    # 1-D points 0, 1, 10, 11, 12 with labels a a b b a; initial centres 0 and 10
    pts = np.array([[0.0], [1.0], [10.0], [11.0], [12.0]], dtype=np.float32)
    lab = np.array([0, 0, 1, 1, 0], dtype=np.int32)
    res = fo.kmeans_build(pts, lab, 2, np.array([[0.0], [10.0]], np.float32), iters=1)
    assert res["centers"][:, 0].tolist() == [0.5, 11.0]
    assert res["assign"].tolist() == [0, 0, 1, 1, 1]
    assert res["majority"].tolist() == [0, 1] and res["sizes"].tolist() == [2, 3]
    assert res["fraction"].tolist() == [1.0, np.float32(2.0 / 3.0)]
    # look-up: query 2.5 is 2 away from centre 0.5 -> confidence 1 / 2; query 9 is 2 from 11 -> (2/3) / 2
    out = fo.kmeans_lookup(np.array([[2.5], [9.0], [11.0]], np.float32), res["centers"], res["majority"],
                           res["fraction"], 0.4)
    assert out["idx"].tolist() == [0, 1, 1] and out["label"].tolist() == [0, 1, 1]
    assert out["conf"][0] == np.float32(0.5) and out["conf"][1] == np.float32((2.0 / 3.0) / 2.0)
    assert np.isposinf(out["conf"][2])            # a query on a centre: always a hit
    assert out["hit"].tolist() == [1, 0, 1]
    # equidistant centres: the lower index; equal label counts: the smaller label
    res = fo.kmeans_build(np.array([[5.0], [5.0]], np.float32), np.array([3, 1], np.int32), 4,
                          np.array([[0.0], [10.0]], np.float32), iters=0)
    assert res["assign"].tolist() == [0, 0] and res["majority"].tolist() == [1, 0]
    assert res["fraction"].tolist() == [0.5, 0.0] and res["sizes"].tolist() == [2, 0]   # an empty cluster never hits


def test_kmeans_against_library_lloyd_and_invariants():
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(3)
    K, d = 6, 5
    true = rng.normal(scale=6.0, size=(K, d))
    pts = (true[rng.integers(0, K, size=400)] + rng.normal(size=(400, d))).astype(np.float32)
    lab = rng.integers(0, 3, size=400).astype(np.int32)
    init = pts[:K].copy()
    prev_inertia = None
    for iters in (1, 2, 5):
        res = fo.kmeans_build(pts, lab, 3, init, iters)
        km = KMeans(n_clusters=K, init=init.astype(np.float64), n_init=1, max_iter=iters, tol=0.0,
                    algorithm="lloyd").fit(pts.astype(np.float64))
        assert (res["sizes"] > 0).all()
        assert np.allclose(res["centers"], km.cluster_centers_, rtol=1e-5, atol=1e-6), iters
        # every point sits with its nearest centre, and the inertia never grows from round to round
        d2 = ((pts[:, None, :].astype(np.float64) - res["centers"][None].astype(np.float64)) ** 2).sum(-1)
        assert np.array_equal(res["assign"], d2.argmin(axis=1))
        inertia = d2.min(axis=1).sum()
        assert prev_inertia is None or inertia <= prev_inertia * (1 + 1e-12)
        prev_inertia = inertia
        # majority label and fraction by an independent count
        for c in range(K):
            cnt = np.bincount(lab[res["assign"] == c], minlength=3)
            assert res["majority"][c] == cnt.argmax() and res["fraction"][c] == np.float32(cnt.max() / cnt.sum())
    # relabelling the points by a permutation gives the same clustering
    perm = rng.permutation(400)
    res_p = fo.kmeans_build(pts[perm], lab[perm], 3, init, 2)
    res_0 = fo.kmeans_build(pts, lab, 3, init, 2)
    assert np.allclose(res_p["centers"], res_0["centers"], rtol=1e-6)
    assert np.array_equal(res_p["assign"], res_0["assign"][perm])


# ---------------------------------------------------------------------------------------------
# projection in front of the look-up (Sec. 3: one-layer dimensionality reduction)
# ---------------------------------------------------------------------------------------------
def test_bf16_rounding_matches_library_conversion_and_ties_go_to_even():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.normal(size=5000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, size=5000),
                        np.array([0.0, -0.0, 1.0, -1.0, 3.3895314e38, 1e-40], np.float32)]).astype(np.float32)
    assert np.array_equal(fo.round_to_bf16(x), torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())
    # halfway cases: 1 + 2^-8 lies between the bf16 neighbours 1 and 1 + 2^-7 -> even mantissa (1);
    # 1 + 3 * 2^-8 lies between 1 + 2^-7 and 1 + 2^-6 -> even mantissa (1 + 2^-6)
    assert fo.round_to_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8], np.float32)).tolist() == [1.0, 1 + 2.0 ** -6]


def test_projection_closed_forms_and_library_matmul():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(7, 48)).astype(np.float32)
    bias = rng.normal(size=48).astype(np.float32)
    # identity weights: y = bf16(x) + b; with ReLU the negative part is cut
    y = fo.project(x, np.eye(48, dtype=np.float32), bias, relu=False)
    assert np.array_equal(y, (fo.round_to_bf16(x).astype(np.float64) + bias.astype(np.float64)).astype(np.float32))
    yr = fo.project(x, np.eye(48, dtype=np.float32), bias, relu=True)
    assert np.array_equal(yr, np.maximum(y, 0)) and (y < 0).any()
    # general weights against a float64 library matmul on operands rounded by the library
    w = rng.normal(size=(20, 48)).astype(np.float32)
    xb = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64)
    wb = torch.from_numpy(w).to(torch.bfloat16).to(torch.float64)
    ref = (xb @ wb.T + torch.from_numpy(bias[:20]).to(torch.float64)).to(torch.float32).numpy()
    got = fo.project(x, w, bias[:20], relu=False)
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    # weights handed over in bf16 are taken as they are, and a transposed operand would not pass
    wbits = synth.bf16_bits(torch.from_numpy(w).to(torch.bfloat16))
    assert np.array_equal(fo.project(x, wbits, bias[:20], relu=False), got)
    assert got.shape == (7, 20)
