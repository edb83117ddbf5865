"""ctypes front end of the CPU oracle (freeze_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the library's product path.  It takes
and returns numpy arrays; the k-NN look-up arithmetic is in the C file, and the
heuristics built on it (confidence thresholds, the k-means cache) are plain
numpy / Python loops below.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "freeze_oracle.c")
_LIB = os.path.join(_HERE, "libfreeze_oracle.so")

F32, BF16 = 0, 1


_LIB_SAN = os.path.join(_HERE, "libfreeze_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math, no BLAS).

    With FREEZE_ORACLE_SANITIZE=1 in the environment the same source is built with the address and
    undefined-behaviour sanitizers instead (the process must then have the sanitizer runtime
    preloaded: tests/test_oracle_sanitized.py runs the pins that way)."""
    san = os.environ.get("FREEZE_ORACLE_SANITIZE") == "1"
    target = _LIB_SAN if san else _LIB
    stale = (not os.path.exists(target)) or os.path.getmtime(target) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = target + ".tmp%d" % os.getpid()
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined"] if san else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-std=c11", "-fPIC", "-shared", "-pthread", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, target)
    return target


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c_p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.fz_oracle_host_threads.restype = i32
        L.fz_oracle_knn.restype = i32
        L.fz_oracle_knn.argtypes = [c_p, i64, c_p, i32, i64, i64, i32, c_p, c_p, i32]
        L.fz_oracle_vote.restype = i32
        L.fz_oracle_vote.argtypes = [c_p, c_p, i64, i32, i32, i32, c_p, c_p, c_p]
        L.fz_oracle_confidence.restype = i32
        L.fz_oracle_confidence.argtypes = [c_p, c_p, c_p, i64, i32, i32, c_p, c_p]
        L.fz_oracle_compact.restype = i64
        L.fz_oracle_compact.argtypes = [c_p, c_p, i64, c_p]
        L.fz_oracle_cascade.restype = i32
        L.fz_oracle_cascade.argtypes = [i32, c_p, i64, c_p, c_p, c_p, c_p, c_p, c_p, i32, c_p, c_p, c_p,
                                        c_p, i32]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _entries(entries: np.ndarray) -> Tuple[np.ndarray, int]:
    if entries.dtype == np.float32:
        return np.ascontiguousarray(entries), F32
    if entries.dtype == np.uint16:
        return np.ascontiguousarray(entries), BF16
    raise TypeError("entries must be float32 or uint16 (bf16 bit patterns)")


def host_threads() -> int:
    return int(lib().fz_oracle_host_threads())


def knn(queries: np.ndarray, entries: np.ndarray, k: int, nthreads: int = 0):
    """Exact k-NN.  Returns (idx [b,k] int32, sqdist [b,k] float64, threads used)."""
    q = np.ascontiguousarray(queries, dtype=np.float32)
    e, kind = _entries(entries)
    b, d = q.shape
    n, d2 = e.shape
    assert d == d2
    idx = np.empty((b, k), dtype=np.int32)
    dist = np.empty((b, k), dtype=np.float64)
    used = lib().fz_oracle_knn(_ptr(q), b, _ptr(e), kind, n, d, k, _ptr(idx), _ptr(dist), nthreads)
    if used < 0:
        raise ValueError("fz_oracle_knn: invalid arguments")
    return idx, dist, used


def vote(labels: np.ndarray, nbr_idx: np.ndarray, num_classes: int, vote_threshold: int):
    """Returns (label [b] int32, votes [b] int32, hit [b] uint8)."""
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    nbr = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    b, k = nbr.shape
    out_l = np.empty(b, dtype=np.int32)
    out_v = np.empty(b, dtype=np.int32)
    out_h = np.empty(b, dtype=np.uint8)
    rc = lib().fz_oracle_vote(_ptr(lab), _ptr(nbr), b, k, num_classes, vote_threshold, _ptr(out_l),
                              _ptr(out_v), _ptr(out_h))
    if rc != 0:
        raise ValueError("fz_oracle_vote: invalid arguments")
    return out_l, out_v, out_h


def confidence(labels: np.ndarray, nbr_idx: np.ndarray, nbr_sqdist: np.ndarray, num_classes: int):
    """Paper's distance-weighted confidence.  Returns (label [b] int32, confidence [b] float64)."""
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    nbr = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    dist = np.ascontiguousarray(nbr_sqdist, dtype=np.float64)
    b, k = nbr.shape
    out_l = np.empty(b, dtype=np.int32)
    out_c = np.empty(b, dtype=np.float64)
    rc = lib().fz_oracle_confidence(_ptr(lab), _ptr(nbr), _ptr(dist), b, k, num_classes, _ptr(out_l),
                                    _ptr(out_c))
    if rc != 0:
        raise ValueError("fz_oracle_confidence: invalid arguments")
    return out_l, out_c


def lookup(queries, entries, labels, num_classes, k, vote_threshold, nthreads: int = 0):
    """k-NN + vote.  Returns dict(idx, sqdist, label, votes, hit, threads)."""
    idx, dist, used = knn(queries, entries, k, nthreads)
    lab, votes, hit = vote(labels, idx, num_classes, vote_threshold)
    return dict(idx=idx, sqdist=dist, label=lab, votes=votes, hit=hit, threads=used)


def compact(hit: np.ndarray, sel_in: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(hit, dtype=np.uint8)
    s = np.ascontiguousarray(sel_in, dtype=np.int32)
    out = np.empty_like(s)
    m = lib().fz_oracle_compact(_ptr(h), _ptr(s), s.shape[0], _ptr(out))
    return out[:m].copy()


def cascade(queries: Sequence[np.ndarray], entries: Sequence[np.ndarray], labels: Sequence[np.ndarray],
            num_classes: Sequence[int], k: int, thresholds: Sequence[int], nthreads: int = 0):
    """Cascaded lookup.  Returns (label [b], exit_layer [b], hits_per_layer [L], threads used)."""
    L = len(queries)
    qs = [np.ascontiguousarray(q, dtype=np.float32) for q in queries]
    es: List[np.ndarray] = []
    kinds = np.empty(L, dtype=np.int32)
    for l, e in enumerate(entries):
        ee, kind = _entries(e)
        es.append(ee)
        kinds[l] = kind
    labs = [np.ascontiguousarray(x, dtype=np.int32) for x in labels]
    b = qs[0].shape[0]
    ns = np.array([e.shape[0] for e in es], dtype=np.int64)
    ds = np.array([e.shape[1] for e in es], dtype=np.int64)
    for l in range(L):
        assert qs[l].shape == (b, ds[l])
    ncls = np.array(list(num_classes), dtype=np.int32)
    thr = np.array(list(thresholds), dtype=np.int32)
    vp = ctypes.c_void_p * L
    qp = vp(*[q.ctypes.data for q in qs])
    ep = vp(*[e.ctypes.data for e in es])
    lp = vp(*[x.ctypes.data for x in labs])
    out_l = np.empty(b, dtype=np.int32)
    out_x = np.empty(b, dtype=np.int32)
    hits = np.zeros(L, dtype=np.int64)
    used = lib().fz_oracle_cascade(L, qp, b, ep, _ptr(kinds), _ptr(ns), _ptr(ds), lp, _ptr(ncls), k,
                                   _ptr(thr), _ptr(out_l), _ptr(out_x), _ptr(hits), nthreads)
    if used < 0:
        raise ValueError("fz_oracle_cascade: invalid arguments")
    return out_l, out_x, hits, used


def lookup_confidence(queries, entries, labels, num_classes, k, conf_threshold, nthreads: int = 0):
    """Look-up under the paper's distance-weighted confidence (Sec. 3) and the strict float
    threshold of Pseudocode 1 (FreezeInference: hit iff confidence > threshold).  The confidence
    is formed in double from the double distances, rounded once to fp32, and compared in fp32.
    Returns dict(idx, sqdist, label, conf (float32), hit)."""
    idx, dist, used = knn(queries, entries, k, nthreads)
    lab, conf = confidence(labels, idx, dist, num_classes)
    with np.errstate(over="ignore"):
        conf32 = conf.astype(np.float32)
    hit = (conf32 > np.float32(conf_threshold)).astype(np.uint8)
    return dict(idx=idx, sqdist=dist, label=lab, conf=conf32, hit=hit, threads=used)


def cascade_confidence(queries: Sequence[np.ndarray], entries: Sequence[np.ndarray], labels: Sequence[np.ndarray],
                       num_classes: Sequence[int], k: int, thresholds: Sequence[float], nthreads: int = 0):
    """Pseudocode 1, FreezeInference, under the confidence rule: layers in order, the first layer
    whose confidence exceeds its threshold ends the request; none -> (-1, -1).
    Returns (label [b], exit_layer [b], hits_per_layer [L])."""
    L = len(queries)
    b = queries[0].shape[0]
    out_l = np.full(b, -1, dtype=np.int32)
    out_x = np.full(b, -1, dtype=np.int32)
    hits = np.zeros(L, dtype=np.int64)
    per_layer = [lookup_confidence(queries[l], entries[l], labels[l], num_classes[l], k, thresholds[l], nthreads)
                 for l in range(L)]
    for i in range(b):
        for l in range(L):
            if per_layer[l]["hit"][i]:
                out_l[i] = per_layer[l]["label"][i]
                out_x[i] = l
                hits[l] += 1
                break
    return out_l, out_x, hits


def compute_thresholds(val_queries: Sequence[np.ndarray], entries: Sequence[np.ndarray],
                       labels: Sequence[np.ndarray], num_classes: Sequence[int], k: int,
                       model_labels: np.ndarray, nthreads: int = 0) -> np.ndarray:
    """Pseudocode 1, ComputeThresholds (Sec. 3.1): per layer, the largest confidence among the
    validation items whose look-up label differs from the model's label; the running maximum
    starts at 0 (the paper gives no initial value; confidences are positive).  float32 [L]."""
    L = len(val_queries)
    y = np.asarray(model_labels)
    thr = np.zeros(L, dtype=np.float32)
    for l in range(L):
        res = lookup_confidence(val_queries[l], entries[l], labels[l], num_classes[l], k, 0.0, nthreads)
        for i in range(y.shape[0]):
            if res["label"][i] != y[i]:
                thr[l] = max(thr[l], res["conf"][i])
    return thr


# ---------------------------------------------------------------------------------------------
# k-means cache (Sec. 4, "k-means": intermediate points of a layer are clustered and each
# cluster is represented by its centre; a cache item is the centre, the majority label of the
# cluster and the fraction of the cluster that carries it; a look-up returns the majority label
# of the closest centre, with confidence = that fraction / the distance to the centre; thresholds
# work as for k-NN).  Readings where the paper is silent: Lloyd's iterations from given initial
# centres for a fixed number of rounds; a point goes to the nearest centre by Euclidean distance
# (equal distances -> the lower centre index); a centre becomes the mean of its points, summed in
# index order in double and rounded once to fp32; a cluster that loses all its points keeps its
# centre (majority label 0, fraction 0, so it never hits); equal label counts -> the smaller
# label; the distance in the confidence is the square root of the squared distance, a zero
# distance gives +inf; the confidence is rounded once to fp32 and compared with `>` in fp32.
# ---------------------------------------------------------------------------------------------
def kmeans_assign(points: np.ndarray, centers: np.ndarray, nthreads: int = 0):
    """Index of the nearest centre of every point and the squared distance to it (double)."""
    idx, dist, _ = knn(points, np.ascontiguousarray(centers, dtype=np.float32), 1, nthreads)
    return idx[:, 0].copy(), dist[:, 0].copy()


def kmeans_build(points: np.ndarray, labels: np.ndarray, num_classes: int, init_centers: np.ndarray,
                 iters: int, nthreads: int = 0):
    """Returns dict(centers float32 [K,d], majority int32 [K], fraction float32 [K], sizes int64 [K],
    assign int32 [n]) after `iters` rounds of (assign, update); labels and fractions come from a
    final assignment to the final centres."""
    pts = np.ascontiguousarray(points, dtype=np.float32)
    lab = np.asarray(labels)
    centers = np.array(init_centers, dtype=np.float32, copy=True)
    K = centers.shape[0]

    def update(assign):
        new = centers.copy()
        for c in range(K):
            members = np.nonzero(assign == c)[0]          # ascending point index
            if members.size:
                acc = np.zeros(pts.shape[1], dtype=np.float64)
                for i in members:
                    acc += pts[i].astype(np.float64)
                new[c] = (acc / float(members.size)).astype(np.float32)
        return new

    for _ in range(iters):
        assign, _ = kmeans_assign(pts, centers, nthreads)
        centers = update(assign)
    assign, _ = kmeans_assign(pts, centers, nthreads)
    majority = np.zeros(K, dtype=np.int32)
    fraction = np.zeros(K, dtype=np.float32)
    sizes = np.zeros(K, dtype=np.int64)
    for c in range(K):
        members = np.nonzero(assign == c)[0]
        sizes[c] = members.size
        if members.size:
            counts = np.zeros(num_classes, dtype=np.int64)
            for i in members:
                counts[int(lab[i])] += 1
            best = 0
            for l in range(num_classes):
                if counts[l] > counts[best]:
                    best = l
            majority[c] = best
            fraction[c] = np.float32(float(counts[best]) / float(members.size))
    return dict(centers=centers, majority=majority, fraction=fraction, sizes=sizes, assign=assign.astype(np.int32))


def kmeans_lookup(queries: np.ndarray, centers: np.ndarray, majority: np.ndarray, fraction: np.ndarray,
                  conf_threshold: float, nthreads: int = 0):
    """Returns dict(idx [b] nearest centre, sqdist [b] double, label, conf float32, hit)."""
    idx, dist = kmeans_assign(queries, centers, nthreads)
    frac = np.asarray(fraction, dtype=np.float64)[idx]
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        conf = np.where(dist > 0, frac / np.sqrt(dist), np.where(frac > 0, np.inf, 0.0)).astype(np.float32)
    hit = (conf > np.float32(conf_threshold)).astype(np.uint8)
    return dict(idx=idx.astype(np.int32), sqdist=dist, label=np.asarray(majority, dtype=np.int32)[idx], conf=conf,
                hit=hit)


# ---------------------------------------------------------------------------------------------
# Dimensionality reduction in front of the look-up (Sec. 3: a one-layer network whose hidden
# layer has 1,024 nodes projects the layer output before it is cached and looked up).  The paper
# gives no activation and no precision.  Reading: y = W x + b, optionally through ReLU; the
# operation is defined on bf16 operands (x and W rounded to nearest even; a W given in bf16 is
# taken as it is), exact products, wide accumulation: here fp64, rounded once to fp32.
# ---------------------------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> the nearest bf16 value (ties to even), returned widened to fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return (r.astype(np.uint32) << 16).view(np.float32).reshape(np.shape(x))


def project(x: np.ndarray, weights: np.ndarray, bias: np.ndarray, relu: bool) -> np.ndarray:
    """x [b, d] fp32, weights [m, d] fp32 or bf16 bit patterns (uint16), bias [m] -> [b, m] float32."""
    xr = round_to_bf16(x).astype(np.float64)
    if weights.dtype == np.uint16:
        wr = (weights.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        wr = round_to_bf16(weights).astype(np.float64)
    b, m = xr.shape[0], wr.shape[0]
    out = np.empty((b, m), dtype=np.float64)
    for i in range(b):
        for j in range(m):
            out[i, j] = float(np.dot(xr[i], wr[j])) + float(bias[j])
    if relu:
        out = np.maximum(out, 0.0)
    return out.astype(np.float32)
