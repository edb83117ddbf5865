"""Seeded synthetic inputs for the Freeze Inference cache-lookup path.

The paper evaluates on CIFAR-10/100 activations of trained ResNets (Sec. 4);
neither the datasets nor the weights exist here, so class-clustered Gaussian
activations of the same shapes stand in: a per-class centroid drawn from
N(0,1)^d, each cached entry / query = centroid of its class + N(0, sigma^2)
noise, optionally passed through ReLU (post-activation block outputs), with
balanced classes in a seeded random order.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no distances, no neighbour selection, no votes) and is the one module that
both the HIP path's tests/bench and the CPU oracle's tests may import.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import torch


@dataclass(frozen=True)
class LayerSpec:
    """One per-layer cache (Pseudocode 1, ConstructCache: a list of <output, label>)."""
    n: int                    # cached entries
    d: int                    # flattened activation size
    num_classes: int
    sigma: float              # within-class noise std
    relu: bool = False        # entries/queries pass through ReLU after the noise
    store_bf16: bool = True   # cache handed over as bf16 (else fp32)
    label_flip_p: float = 0.0  # each cache label replaced by a different random class w.p. p


@dataclass(frozen=True)
class Workload:
    name: str
    layers: Tuple[LayerSpec, ...]
    batch: int
    k: int
    vote_thresholds: Tuple[int, ...]
    rescore_r: int            # 0 = library default
    seed: int


BASE_SEED = 20020264


def _wl(name, idx, layers, batch, k, thr, r=0):
    layers = tuple(layers)
    if isinstance(thr, int):
        thr = (thr,) * len(layers)
    return Workload(name, layers, batch, k, tuple(thr), r, BASE_SEED + idx)


# The five benchmark configurations (the d values are CIFAR ResNet-18 block
# output sizes implied by Table 1: 64x32x32, 128x16x16, 256x8x8, 512x4x4).
WORKLOADS = {
    "c1_tiny": _wl("c1_tiny", 0, [LayerSpec(2000, 512, 10, 0.5, store_bf16=False)], 256, 5, 4),
    "c2_batched": _wl("c2_batched", 1, [LayerSpec(50000, 8192, 10, 0.8, relu=True)], 10000, 10, 8),
    "c3_wide": _wl("c3_wide", 2, [LayerSpec(50000, 65536, 10, 1.5)], 256, 10, 9, r=64),
    "c4_cascade": _wl("c4_cascade", 3, [
        LayerSpec(50000, 65536, 10, 1.5), LayerSpec(50000, 32768, 10, 1.0),
        LayerSpec(50000, 16384, 10, 0.6), LayerSpec(50000, 512, 10, 0.3)], 4096, 10, 8),
    "c4_cascade_noisy": _wl("c4_cascade_noisy", 3, [
        LayerSpec(50000, 65536, 10, 1.5, label_flip_p=0.35),
        LayerSpec(50000, 32768, 10, 1.0, label_flip_p=0.25),
        LayerSpec(50000, 16384, 10, 0.6, label_flip_p=0.15),
        LayerSpec(50000, 512, 10, 0.3, label_flip_p=0.05)], 4096, 10, 8),
    "c5_latency_b1": _wl("c5_latency_b1", 4, [LayerSpec(1000000, 512, 100, 0.7)], 1, 20, 15),
    "c5_latency_b8": _wl("c5_latency_b8", 4, [LayerSpec(1000000, 512, 100, 0.7)], 8, 20, 15),
}


def scaled(wl: Workload, *, n: Optional[int] = None, d_div: int = 1, batch: Optional[int] = None,
           name: Optional[str] = None) -> Workload:
    """A smaller workload of the same recipe (for parity tests the oracle finishes in seconds)."""
    layers = tuple(replace(l, n=(n if n is not None else l.n), d=max(1, l.d // d_div)) for l in wl.layers)
    return replace(wl, layers=layers, batch=(batch if batch is not None else wl.batch),
                   name=name or (wl.name + "_scaled"))


@dataclass
class LayerData:
    spec: LayerSpec
    entries: torch.Tensor      # [n, d] bf16 or fp32, on `device`
    labels: torch.Tensor       # [n] int32 (after optional label flips)
    centroids: torch.Tensor    # [num_classes, d] fp32
    clean_labels: torch.Tensor  # [n] int32 geometry-aligned class of each entry


@dataclass
class WorkloadData:
    workload: Workload
    layers: List[LayerData]
    queries: List[torch.Tensor]   # per layer [batch, d] fp32 (row b = request b)
    query_classes: torch.Tensor   # [batch] int32
    device: torch.device = field(default_factory=lambda: torch.device("cpu"))


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def balanced_labels(n: int, num_classes: int, seed: int) -> torch.Tensor:
    """n labels with (almost) equal class counts in a seeded random order (drawn on the CPU)."""
    g = _gen("cpu", seed)
    base = torch.arange(n, dtype=torch.int64) % num_classes
    return base[torch.randperm(n, generator=g)].to(torch.int32)


def _draw_rows(centroids: torch.Tensor, classes: torch.Tensor, sigma: float, relu: bool,
               out_dtype: torch.dtype, gen: torch.Generator, chunk_elems: int = 1 << 27) -> torch.Tensor:
    n = classes.numel()
    d = centroids.shape[1]
    dev = centroids.device
    out = torch.empty((n, d), dtype=out_dtype, device=dev)
    rows = max(1, chunk_elems // d)
    cls = classes.to(device=dev, dtype=torch.int64)
    for lo in range(0, n, rows):
        hi = min(n, lo + rows)
        x = torch.randn((hi - lo, d), generator=gen, device=dev, dtype=torch.float32)
        x.mul_(sigma).add_(centroids.index_select(0, cls[lo:hi]))
        if relu:
            x.clamp_(min=0.0)
        out[lo:hi] = x.to(out_dtype)   # bf16: round-to-nearest-even, once, here
        del x
    return out


def make_layer(spec: LayerSpec, seed: int, device="cpu") -> LayerData:
    device = torch.device(device)
    cent = torch.randn((spec.num_classes, spec.d), generator=_gen(device, seed), device=device,
                       dtype=torch.float32)
    clean = balanced_labels(spec.n, spec.num_classes, seed + 1)
    dt = torch.bfloat16 if spec.store_bf16 else torch.float32
    entries = _draw_rows(cent, clean, spec.sigma, spec.relu, dt, _gen(device, seed + 2))
    labels = make_layer_labels(spec, seed)
    return LayerData(spec, entries, labels.to(device), cent, clean.to(device))


def make_layer_labels(spec: LayerSpec, seed: int) -> torch.Tensor:
    """The labels make_layer(spec, seed) gives the entries, without drawing the entries (CPU tensor)."""
    clean = balanced_labels(spec.n, spec.num_classes, seed + 1)
    if spec.label_flip_p <= 0.0:
        return clean
    g = _gen("cpu", seed + 3)
    flip = torch.rand(spec.n, generator=g) < spec.label_flip_p
    shift = torch.randint(1, spec.num_classes, (spec.n,), generator=g, dtype=torch.int64)
    flipped = ((clean.to(torch.int64) + shift) % spec.num_classes).to(torch.int32)
    return torch.where(flip, flipped, clean)


def make_workload_labels(wl: Workload) -> List[torch.Tensor]:
    """Per layer, the cache labels make_workload(wl) would produce."""
    return [make_layer_labels(spec, wl.seed + 100 * li + 10) for li, spec in enumerate(wl.layers)]


def make_queries(layer: LayerData, classes: torch.Tensor, seed: int) -> torch.Tensor:
    """fp32 queries drawn like the entries of `layer` for the given per-request classes."""
    dev = layer.centroids.device
    return _draw_rows(layer.centroids, classes, layer.spec.sigma, layer.spec.relu, torch.float32,
                      _gen(dev, seed))


def make_workload(wl: Workload, device="cpu") -> WorkloadData:
    device = torch.device(device)
    g = _gen("cpu", wl.seed + 7)
    ncls = wl.layers[0].num_classes
    qcls = torch.randint(0, ncls, (wl.batch,), generator=g, dtype=torch.int64).to(torch.int32)
    layers, queries = [], []
    for li, spec in enumerate(wl.layers):
        ld = make_layer(spec, wl.seed + 100 * li + 10, device)
        layers.append(ld)
        queries.append(make_queries(ld, qcls, wl.seed + 100 * li + 50))
    return WorkloadData(wl, layers, queries, qcls.to(device), device)


def random_labels(n: int, num_classes: int, seed: int) -> torch.Tensor:
    """i.i.d. uniform labels, independent of geometry (adversarial input for the vote)."""
    return torch.randint(0, num_classes, (n,), generator=_gen("cpu", seed), dtype=torch.int64).to(torch.int32)


def bf16_bits(t: torch.Tensor):
    """bf16 tensor -> numpy uint16 array of its bit patterns (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")
