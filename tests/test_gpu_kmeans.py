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


def _no_assignment_near_tie(pts, centers, rel=3e-6):
    d2 = ((pts[:, None, :].astype(np.float64) - centers[None].astype(np.float64)) ** 2).sum(-1)
    part = np.partition(d2, 1, axis=1)
    return bool(((part[:, 1] - part[:, 0]) > rel * part[:, 1]).all())


@pytest.mark.parametrize("n,d,kc,classes,iters", [
    (3002, 96, 20, 5, 3),       # several cache tiles of points, one tile of centres
    (5000, 520, 300, 7, 2),     # more than one tile of centres, d not a multiple of 64
    (700, 40, 700, 3, 1),       # as many centres as points: every cluster is its own point
    (2000, 64, 8, 4, 0),        # no iteration: labels and shares for the given centres
])
def test_kmeans_build_and_lookup_against_oracle(n, d, kc, classes, iters):
    pts, lab = _points(n, d, classes, 900 + n + kc)   # (sizes chosen so that the seeded run has no near-tie)
    init = pts[:kc].clone()
    ref = fo.kmeans_build(pts.numpy(), lab.numpy(), classes, init.numpy(), iters)
    # the comparison below needs the same assignments on both sides: no point may sit (nearly)
    # halfway between two centres in any round of the oracle's run
    cen = init.numpy().copy()
    for _ in range(iters + 1):
        assert _no_assignment_near_tie(pts.numpy(), cen), "choose another seed: an assignment is a near-tie"
        a, _ = fo.kmeans_assign(pts.numpy(), cen)
        new = cen.copy()
        for c in range(kc):
            m = np.nonzero(a == c)[0]
            if m.size:
                new[c] = (pts.numpy()[m].astype(np.float64).sum(axis=0) / m.size).astype(np.float32)
        cen = new
    fc = binding.FreezeCache(1)
    try:
        got = fc.build_kmeans_layer(0, pts.cuda(), lab.cuda(), classes, init.cuda(), iters)
        torch.cuda.synchronize()
        cen_g = got["centers"].cpu().numpy()
        # same assignments, sums in the same order in fp64, one rounding: the centres agree to the last bit or two
        assert np.allclose(cen_g, ref["centers"], rtol=1e-6, atol=1e-7)
        assert np.array_equal(got["majority"].cpu().numpy(), ref["majority"])
        assert np.array_equal(got["fraction"].cpu().numpy(), ref["fraction"])
        # look-ups: fresh points, and some exactly on a centre
        q, _ = _points(300, d, classes, 77 + n)
        q[:5] = got["centers"][:5].cpu()
        exp = fo.kmeans_lookup(q.numpy(), ref["centers"], ref["majority"], ref["fraction"], 0.0)
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
