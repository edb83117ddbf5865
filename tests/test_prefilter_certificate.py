"""CPU model of the bf16 pre-filter and of its exactness certificate (no GPU, no HIP library).

The look-up ranks cache entries by a coarse key |c_bf|^2 - 2 q_bf.c_bf formed from bf16-rounded
operands in fp32 and re-scores the R best exactly.  These tests emulate that key in numpy on the
inputs that defeat it (low-dimensional dense data, clusters far from the origin, k = R) and pin

  * that the hole is real: for such inputs the coarse top-R does not always hold the exact
    top-k, and the share of queries affected falls as R grows;
  * that the certificate as the kernels compute it (sample mean / standard deviation of
    coarse key minus exact distance over the re-scored candidates, margin of 8 standard
    deviations widened by 1 + 4/m for m samples, at least 8 distinct samples, bound = smallest
    coarse key left out) never
    confirms a query whose coarse candidates miss a true neighbour, while it confirms nearly
    every query of the class-clustered high-dimensional data the paper's caches hold.

The exact distances come from the oracle (brute force in fp64); the emulation of the key and
the restated certificate are this test's own."""
import numpy as np
import pytest
import torch

from oracle import freeze_oracle as fo

Z, MIN_SAMPLES = 8.0, 8


def _bf16(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _coarse_keys(q, c, stored_bf16):
    qb = _bf16(q)
    cb = c if stored_bf16 else _bf16(c)
    norm = (cb * cb).sum(axis=1, dtype=np.float32)
    return (norm[None, :] - np.float32(2.0) * (qb @ cb.T)).astype(np.float32)


def _clustered(rng, n, d, b, sigma, relu, offset, stored_bf16):
    cent = rng.standard_normal((10, d)).astype(np.float32)
    c = cent[rng.integers(0, 10, n)] + sigma * rng.standard_normal((n, d)).astype(np.float32) + offset
    q = cent[rng.integers(0, 10, b)] + sigma * rng.standard_normal((b, d)).astype(np.float32) + offset
    if relu:
        c, q = np.maximum(c, 0), np.maximum(q, 0)
    c = _bf16(c) if stored_bf16 else c.astype(np.float32)
    return q.astype(np.float32), c


def _exact_order(q, c, k):
    idx, dist, _ = fo.knn(q, c, k)          # oracle: brute force, (distance, index) order
    return idx, dist


def _certify(kappa, dist, k, kappa_excl):
    """The kernels' rule, restated: candidates with coarse keys kappa and exact distances dist."""
    m = len(kappa)
    dk = np.sort(dist)[k - 1]
    if not np.isfinite(kappa_excl):
        return True
    if m < MIN_SAMPLES or len(np.unique(dist)) < MIN_SAMPLES:
        return False
    e = kappa.astype(np.float64) - dist.astype(np.float64)
    mean, sd = e.mean(), e.std(ddof=1)
    margin = max(Z * (1.0 + 4.0 / m) * sd * np.sqrt(1.0 + 1.0 / m), 4 * 2.0 ** -24 * (abs(kappa_excl) + abs(mean) + dk))
    return bool(kappa_excl - mean - margin > dk)


def _run(q, c, stored_bf16, k, r):
    """Returns (queries whose coarse top-r misses a true neighbour, confirmed queries, confirmed AND missed)."""
    n = c.shape[0]
    kap = _coarse_keys(q, c, stored_bf16)
    true_idx, _ = _exact_order(q, c, k)
    missed = confirmed = wrong = 0
    ar = np.arange(n)
    for i in range(q.shape[0]):
        order = np.lexsort((ar, kap[i]))
        cand = order[:r]
        d_c = ((q[i].astype(np.float64)[None, :] - c[cand].astype(np.float64)) ** 2).sum(axis=1)
        miss = not set(true_idx[i].tolist()) <= set(cand.tolist())
        ok = _certify(kap[i][cand], d_c, k, kap[i][order[r]] if r < n else np.inf)
        missed += miss
        confirmed += ok
        wrong += ok and miss
    return missed, confirmed, wrong


def test_coarse_ranking_misses_neighbours_on_offset_clusters_and_recall_grows_with_r():
    rng = np.random.default_rng(11)
    q, c = _clustered(rng, 4000, 64, 150, 1.0, False, 100.0, True)
    miss = {r: _run(q, c, True, 10, r)[0] for r in (10, 16, 32, 64)}
    assert miss[10] > 50, miss                 # no spare candidate: most queries lose a neighbour
    assert miss[16] > 0, miss                  # the default width for k = 10 is not enough here
    assert miss[10] >= miss[16] >= miss[32] >= miss[64], miss
    assert miss[64] == 0, miss


@pytest.mark.parametrize("name,args,stored,k,r", [
    ("offset clusters, bf16 cache", (4000, 64, 150, 1.0, False, 100.0, True), True, 10, 16),
    ("offset clusters, fp32 cache", (4000, 64, 150, 1.0, False, 100.0, False), False, 10, 16),
    ("low-dimensional dense", (1585, 6, 400, 0.8, True, 0.0, True), True, 34, 40),
    ("k = R = 64", (5000, 128, 100, 0.8, True, 0.0, True), True, 64, 64),
    ("narrow width", (5000, 128, 150, 0.8, True, 0.0, True), True, 10, 11),
])
def test_certificate_never_confirms_a_missed_neighbour(name, args, stored, k, r):
    rng = np.random.default_rng(5)
    q, c = _clustered(rng, *args)
    missed, confirmed, wrong = _run(q, c, stored, k, r)
    assert wrong == 0, f"{name}: {wrong} queries confirmed although the candidates miss a true neighbour"
    if name in ("offset clusters, bf16 cache", "offset clusters, fp32 cache", "k = R = 64"):
        assert missed > 0, f"{name}: this input is meant to defeat the coarse ranking"


def test_certificate_confirms_the_papers_kind_of_data_at_the_default_width():
    rng = np.random.default_rng(3)
    q, c = _clustered(rng, 8000, 1024, 120, 0.8, True, 0.0, True)     # class-clustered post-ReLU activations
    missed, confirmed, wrong = _run(q, c, True, 10, 16)
    assert missed == 0 and wrong == 0
    assert confirmed >= 114, confirmed       # >= 95 %: the slower paths stay rare


def _misses_with_centring(q, c, k, r, centre):
    """Queries whose coarse top-r misses a true neighbour when both sides are shifted by the cache's
    mean vector before the bf16 rounding (distances do not change under a common shift; the stored
    values are still the cache, so the shifted bf16 copy is a second, rounded copy of it)."""
    n = c.shape[0]
    mu = c.astype(np.float64).mean(axis=0).astype(np.float32) if centre else np.float32(0.0)
    kap = _coarse_keys(q - mu, _bf16(c - mu), True)
    true_idx, _ = _exact_order(q, c, k)
    ar = np.arange(n)
    missed = 0
    for i in range(q.shape[0]):
        cand = np.lexsort((ar, kap[i]))[:r]
        missed += not set(true_idx[i].tolist()) <= set(cand.tolist())
    return missed


def test_centring_trial_helps_offset_data_only():
    """The trial behind the library's rule to centre a cache only when its mean dominates its spread:
    subtracting the cache's mean before rounding removes the misses on clusters far from the origin,
    and gains nothing on post-ReLU class-clustered activations stored in bf16 (there the shifted
    copy has a rounding error the stored one does not)."""
    rng = np.random.default_rng(21)
    q, c = _clustered(rng, 4000, 64, 150, 1.0, False, 100.0, True)
    assert _misses_with_centring(q, c, 10, 16, False) > 0
    assert _misses_with_centring(q, c, 10, 16, True) == 0
    q, c = _clustered(rng, 8000, 1024, 100, 0.8, True, 0.0, True)
    plain, centred = _misses_with_centring(q, c, 10, 11, False), _misses_with_centring(q, c, 10, 11, True)
    assert centred >= plain - 2, (plain, centred)       # no gain worth a second copy of the cache
