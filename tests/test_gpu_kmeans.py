"""GPU parity for the k-means cache (Sec. 4): Lloyd iterations whose assignment step is the
batched look-up, majority labels and shares, and the look-up with confidence = share / distance,
through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import freeze_oracle as fo
from paper_2002_02645_amd import binding, synth

pytestmark = pytest.mark.gpu

TIGHT = 1e-5


def _points(n, d, classes, seed, sigma=1.0):
    g = torch.Generator().manual_seed(seed)
    cent = torch.randn(classes, d, generator=g) * 2.0
    cls = torch.randint(0, classes, (n,), generator=g)
    pts = cent[cls] + sigma * torch.randn(n, d, generator=g)
    # labels mostly follow the geometry, some do not: majority shares below 1
    flip = torch.rand(n, generator=g) < 0.2
    lab = torch.where(flip, torch.randint(0, classes, (n,), generator=g), cls).to(torch.int32)
    return pts.contiguous(), lab.contiguous()


REL = 1e-4   # the look-up's near-tie tolerance: two distances closer than this may rank either way


def _subset_means(pts, fixed, free):
    """Means (float32) of the rows `fixed` plus every subset of the rows `free`, summed in point order in fp64."""
    out = []
    for mask in range(1 << len(free)):
        members = sorted(list(fixed) + [free[j] for j in range(len(free)) if mask >> j & 1])
        if not members:
            out.append(None)
            continue
        acc = np.zeros(pts.shape[1], dtype=np.float64)
        for i in members:
            acc += pts[i].astype(np.float64)
        out.append((members, (acc / float(len(members))).astype(np.float32)))
    return out


def _check_round(pts, lab, classes, cen_prev, cen_next=None, majority=None, fraction=None):
    """One round of Lloyd's iteration from the centres `cen_prev`, by the oracle's distances, under a
    defined rule for near-ties: a point whose two nearest centres are within REL (relative) of each
    other may be assigned to either of the two; every other point goes to its nearest centre (lower
    index on exactly equal distances cannot occur outside the tolerance).  A cluster no such point
    can reach must come out exactly as the oracle computes it; a cluster some can reach must equal
    the oracle's result for ONE choice of which of them it receives (every subset is tried).
    Checks the next centres (cen_next) and / or the majority labels and shares.  Returns the number
    of points that were free to go either way."""
    K = cen_prev.shape[0]
    idx2, d2, _ = fo.knn(pts, np.ascontiguousarray(cen_prev, dtype=np.float32), min(2, K))
    free = np.zeros(pts.shape[0], bool) if K == 1 else (d2[:, 1] - d2[:, 0]) <= REL * d2[:, 1]
    nearest = idx2[:, 0]
    for c in range(K):
        fixed = np.nonzero(~free & (nearest == c))[0].tolist()
        reach = np.nonzero(free & ((idx2[:, 0] == c) | (idx2[:, min(1, K - 1)] == c)))[0].tolist()
        assert len(reach) <= 10, "too many near-tie points around one centre for an exhaustive check"
        options = _subset_means(pts, fixed, reach)
        if cen_next is not None:
            ok = False
            for opt in options:
                want = cen_prev[c] if opt is None else opt[1]      # an empty cluster keeps its centre
                ok = ok or np.allclose(cen_next[c], want, rtol=1e-6, atol=1e-7)
            assert ok, f"centre {c}: no assignment of its {len(reach)} near-tie points gives the reported mean"
        if majority is not None:
            ok = False
            for opt in options:
                if opt is None:
                    ok = ok or (majority[c] == 0 and fraction[c] == 0.0)
                    continue
                counts = np.bincount(lab[opt[0]], minlength=classes)
                best = int(np.argmax(counts))                       # first maximum: the smaller label
                ok = ok or (majority[c] == best and fraction[c] == np.float32(float(counts[best]) / float(len(opt[0]))))
            assert ok, f"centre {c}: majority label / share match no assignment of its near-tie points"
    return int(free.sum())


@pytest.mark.parametrize("n,d,kc,classes,iters,plant", [
    (3002, 96, 20, 5, 3, False),      # several cache tiles of points, one tile of centres
    (5000, 520, 300, 7, 2, False),    # more than one tile of centres, d not a multiple of 64
    (700, 40, 700, 3, 1, False),      # as many centres as points: every cluster is its own point
    (2000, 64, 8, 4, 0, False),       # no iteration: labels and shares for the given centres
    (1500, 48, 12, 4, 2, True),       # points planted (nearly) halfway between two centres: near-tie assignments
])
def test_kmeans_build_and_lookup_against_oracle(n, d, kc, classes, iters, plant):
    pts, lab = _points(n, d, classes, 900 + n + kc)
    init = pts[:kc].clone()
    if plant:
        for j in range(4):     # within 1e-6 of the midpoint of two initial centres: either assignment is right
            pts[kc + j] = (init[2 * j] + init[2 * j + 1]) * 0.5 + 1e-6 * (j - 1.5) * (init[2 * j + 1] - init[2 * j])
    pts_h, lab_h = pts.numpy(), lab.numpy().astype(np.int64)
    fc = binding.FreezeCache(1)
    try:
        # round by round: the library's centres after t rounds are the start of the oracle's round t + 1
        runs = [fc.build_kmeans_layer(0, pts.cuda(), lab.cuda(), classes, init.cuda(), t) for t in range(iters + 1)]
        torch.cuda.synchronize()
        cens = [r["centers"].cpu().numpy() for r in runs]
        assert np.array_equal(cens[0], init.numpy())
        free_total = 0
        for t in range(iters):
            free_total += _check_round(pts_h, lab_h, classes, cens[t], cen_next=cens[t + 1])
        got = runs[iters]
        free_total += _check_round(pts_h, lab_h, classes, cens[iters], majority=got["majority"].cpu().numpy(),
                                   fraction=got["fraction"].cpu().numpy())
        assert free_total > 0 or not plant       # the planted case exercises the near-tie rule
        cen_g = cens[iters]
        ref = dict(majority=got["majority"].cpu().numpy(), fraction=got["fraction"].cpu().numpy())
        if free_total == 0:
            # no near-tie anywhere: the whole build equals the oracle's own run from the same start
            full = fo.kmeans_build(pts_h, lab_h, classes, init.numpy(), iters)
            assert np.allclose(cen_g, full["centers"], rtol=1e-6, atol=1e-7)
            assert np.array_equal(ref["majority"], full["majority"]) and np.array_equal(ref["fraction"], full["fraction"])
        # look-ups: fresh points, and some exactly on a centre
        q, _ = _points(300, d, classes, 77 + n)
        q[:5] = got["centers"][:5].cpu()
        exp = fo.kmeans_lookup(q.numpy(), cen_g, ref["majority"], ref["fraction"], 0.0)
        finite = np.isfinite(exp["conf"])
        thr = float(np.float32(np.median(exp["conf"][finite])))
        exp = fo.kmeans_lookup(q.numpy(), cen_g, ref["majority"], ref["fraction"], thr)
        for batch in (q, q[:7].contiguous()):      # the tiled path and the small-batch path
            e = {key: v[:batch.shape[0]] for key, v in exp.items()}
            out = fc.lookup_confidence(0, batch.cuda(), 1, thr)
            torch.cuda.synchronize()
            o = {key: v.cpu().numpy() for key, v in out.items()}
            part = np.partition(((batch.numpy()[:, None, :].astype(np.float64) - cen_g[None].astype(np.float64)) ** 2)
                                .sum(-1), 1, axis=1) if kc > 1 else None
            clear = np.ones(batch.shape[0], bool) if part is None else (part[:, 1] - part[:, 0]) > 1e-4 * part[:, 1]
            assert clear.sum() > batch.shape[0] * 0.9
            assert np.array_equal(o["idx"][clear, 0], e["idx"][clear])
            assert np.array_equal(o["label"][clear], e["label"][clear])
            assert np.allclose(o["dist"][clear, 0], e["sqdist"][clear], rtol=TIGHT, atol=0)
            assert (o["dist"][:5, 0] == 0).all() and np.isposinf(o["conf"][:5]).all() and o["hit"][:5].all()
            fin = clear & np.isfinite(e["conf"])
            assert np.allclose(o["conf"][fin], e["conf"][fin], rtol=TIGHT)
            decided = fin & (np.abs(e["conf"].astype(np.float64) - thr) > 1e-4 * thr)
            assert np.array_equal(o["hit"][decided], e["hit"][decided])
            if batch.shape[0] > 100:
                assert 0 < o["hit"][decided].sum() < decided.sum()      # both outcomes occur
            # the plain look-up on a k-means layer: nearest centre, its majority label
            plain = fc.lookup(0, batch.cuda(), 1, 1)
            torch.cuda.synchronize()
            assert np.array_equal(plain["idx"].cpu().numpy()[clear, 0], e["idx"][clear])
            assert np.array_equal(plain["label"].cpu().numpy()[clear], e["label"][clear])
        # the k-means confidence is defined for one neighbour only
        with pytest.raises(binding.FreezeError):
            fc.lookup_confidence(0, q.cuda(), 2, thr)
    finally:
        fc.close()


def test_kmeans_thresholds_and_cascade_with_a_knn_layer():
    # a cascade of a k-means layer and a k-NN layer under the confidence rule, thresholds from a validation set
    n, d, kc, classes = 4000, 128, 40, 6
    pts, lab = _points(n, d, classes, 4321)
    val, y = _points(600, d, classes, 99)
    init = pts[:kc].clone()
    fc = binding.FreezeCache(2)
    try:
        km = fc.build_kmeans_layer(0, pts.cuda(), lab.cuda(), classes, init.cuda(), 2)
        fc.build_layer(1, pts.cuda(), lab.cuda(), classes)
        torch.cuda.synchronize()
        # k = 1 throughout: the k-means confidence needs it
        thr = fc.compute_thresholds([0, 1], [val.cuda(), val.cuda()], 1, y.cuda())
        torch.cuda.synchronize()
        thr_h = thr.cpu().numpy()
        cen = km["centers"].cpu().numpy()
        exp0 = fo.kmeans_lookup(val.numpy(), cen, km["majority"].cpu().numpy(), km["fraction"].cpu().numpy(), 0.0)
        wrong0 = exp0["conf"][exp0["label"] != y.numpy()]
        assert wrong0.size and np.isclose(thr_h[0], wrong0.max(), rtol=TIGHT)
        exp1 = fo.compute_thresholds([val.numpy()], [pts.numpy()], [lab.numpy()], [classes], 1, y.numpy())
        assert np.isclose(thr_h[1], exp1[0], rtol=TIGHT)
        out = fc.lookup_cascade_confidence([0, 1], [val.cuda(), val.cuda()], 1, thr_h.tolist())
        torch.cuda.synchronize()
        x, l = out["exit_layer"].cpu().numpy(), out["label"].cpu().numpy()
        assert (l[x >= 0] == y.numpy()[x >= 0]).all()      # zero error on the validation set (Sec. 3.1)
        assert out["hits_per_layer"].cpu().numpy().sum() == (x >= 0).sum()
    finally:
        fc.close()
