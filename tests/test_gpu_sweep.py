"""GPU parity on seeded random shapes: every path (tiled kernels with 4 and 8 waves, balanced
decomposition, keys-out with stream-K, small-batch kernel) against the CPU oracle, with the default
re-scoring width or any width from k to 64 (a narrow one makes the certificate send queries to the
wider re-scoring or to the exact scan).  The shapes are drawn once from a fixed seed."""
import random

import pytest
import torch

from paper_2002_02645_amd import synth
from tests.test_gpu_parity import check_case

pytestmark = pytest.mark.gpu


def _draw(rng, kind):
    if kind == "small":
        n, d, b = rng.randint(1, 40000), rng.randint(1, 1024), rng.randint(1, 16)
    elif kind == "keys":
        d = rng.randint(500, 5000)
        b, n = rng.randint(17, max(17, min(256, d // 20))), rng.randint(200, 6000)
    elif kind == "wide":
        n, d, b = rng.randint(100, 3000), rng.randint(1, 300), rng.randint(257, 3000)
    elif kind == "balanced":
        b, n = rng.randint(1500, 4200), rng.randint(30000, 70000)
        d = rng.randint(8, max(8, int(2.4e9 / (b * n))))
    else:
        n, d, b = rng.randint(1, 9000), rng.randint(1, 1600), rng.randint(17, 900)
    while n * d * b > 2.5e9:
        n = max(1, n // 2)
    k = rng.randint(1, min(n, 64))
    r = rng.choice([0, 0, rng.randint(k, 64)])   # any width down to k itself: the width never changes the result
    if r > n:
        r = 0
    return n, d, b, k, r


def _cases():
    rng = random.Random(20020264)
    kinds = ["tiled"] * 8 + ["small"] * 4 + ["keys"] * 4 + ["wide"] * 4 + ["balanced"] * 4
    out = []
    for i, kind in enumerate(kinds):
        n, d, b, k, r = _draw(rng, kind)
        out.append((kind, n, d, b, k, r, rng.random() < 0.5, rng.random() < 0.5, 3000 + i))
    return out


@pytest.mark.parametrize("kind,n,d,b,k,r,bf16,relu,seed", _cases())
def test_random_shape(kind, n, d, b, k, r, bf16, relu, seed):
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b)
    spec = wl.layers[0]
    spec = type(spec)(n, d, 10, spec.sigma, relu=relu, store_bf16=bf16)
    data = synth.make_workload(type(wl)(wl.name, (spec,), b, k, (max(1, k - 2),), r, seed))
    L = data.layers[0]
    check_case(L.entries, L.labels, data.queries[0], 10, k, max(1, k - 2), r)
