"""Comparator between a lookup result and the oracle's, with the near-tie rule.

Rule (one place, used by every parity test): with the oracle's sorted squared
distances D(1) <= ... <= D(k+1) (the first excluded neighbour included), a
query is *near-tie* if any adjacent pair among those ranks differs by less than
REL relative.  Not near-tie: neighbour indices, label, votes and hit must equal
the oracle's exactly.  Near-tie: the reported indices must be distinct, valid,
each with an oracle distance <= D(k) * (1 + REL), non-decreasing within REL,
and label/votes/hit must equal the oracle's vote applied to the reported
indices.  In every case each reported distance must be within REL relative of
the oracle's distance of the reported index, and exactly 0 where that is 0.
"""
from __future__ import annotations

import numpy as np

from oracle import freeze_oracle as fo

REL = 1e-4


def _rel(a, b):
    m = np.maximum(np.maximum(np.abs(a), np.abs(b)), 1e-30)
    return np.abs(a - b) / m


def oracle_reference(queries, entries, labels, num_classes, k, vote_threshold, nthreads=0):
    """Oracle lookup with one extra neighbour (for the near-tie test)."""
    n = entries.shape[0]
    kk = min(k + 1, n)
    idx, dist, used = fo.knn(queries, entries, kk, nthreads)
    lab, votes, hit = fo.vote(labels, idx[:, :k], num_classes, vote_threshold)
    return dict(idx=idx[:, :k], sqdist=dist[:, :k], idx_ext=idx, sqdist_ext=dist, label=lab,
                votes=votes, hit=hit, threads=used)


def exact_sqdist(query, entries, rows):
    """Squared distances of one fp32 query to selected cache rows in float64 (numpy; comparator only)."""
    if entries.dtype == np.uint16:
        sel = (entries[rows].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        sel = entries[rows].astype(np.float64)
    diff = query.astype(np.float64)[None, :] - sel
    return (diff * diff).sum(axis=1)


def compare_lookup(got, ref, queries, entries, labels, num_classes, k, vote_threshold, rel=REL, dist_rel=REL):
    """got: dict(idx [b,k], dist [b,k] fp32, label, votes, hit) as numpy arrays.
    rel: the near-tie tolerance (the contract's 1e-4, or a tighter one); dist_rel: the tolerance on
    reported distances.
    Returns (number of near-tie queries, list of failure strings)."""
    REL = rel
    b = ref["idx"].shape[0]
    n = entries.shape[0]
    fails = []
    near = 0
    for i in range(b):
        D = ref["sqdist_ext"][i]
        is_near = bool((_rel(D[1:], D[:-1]) < REL).any()) if D.shape[0] > 1 else False
        gi = got["idx"][i]
        gd = got["dist"][i].astype(np.float64)
        if not is_near:
            if not np.array_equal(gi, ref["idx"][i]):
                fails.append(f"q{i}: idx {gi.tolist()} != oracle {ref['idx'][i].tolist()}")
                continue
            true_d = ref["sqdist"][i]
            exp = (ref["label"][i], ref["votes"][i], ref["hit"][i])
        else:
            near += 1
            if len(set(gi.tolist())) != k or gi.min() < 0 or gi.max() >= n:
                fails.append(f"q{i}: near-tie but indices invalid {gi.tolist()}")
                continue
            true_d = exact_sqdist(queries[i], entries, gi)
            if (true_d > ref["sqdist"][i, k - 1] * (1 + REL)).any():
                fails.append(f"q{i}: near-tie, reported neighbour farther than D(k)(1+rel)")
                continue
            if ((true_d[1:] < true_d[:-1]) & (_rel(true_d[1:], true_d[:-1]) >= REL)).any():
                fails.append(f"q{i}: near-tie, reported order decreasing beyond rel")
                continue
            l, v, h = fo.vote(labels, gi[None, :], num_classes, vote_threshold)
            exp = (l[0], v[0], h[0])
        bad = (_rel(gd, true_d) > dist_rel) | ((true_d == 0.0) & (gd != 0.0))
        if bad.any():
            fails.append(f"q{i}: dist {gd.tolist()} vs oracle {true_d.tolist()}")
        gotv = (got["label"][i], got["votes"][i], got["hit"][i])
        if tuple(int(x) for x in gotv) != tuple(int(x) for x in exp):
            fails.append(f"q{i}: (label,votes,hit) {gotv} != {exp}")
    return near, fails


def assert_lookup_matches(got, ref, queries, entries, labels, num_classes, k, vote_threshold, rel=REL,
                          dist_rel=REL):
    near, fails = compare_lookup(got, ref, queries, entries, labels, num_classes, k, vote_threshold, rel,
                                 dist_rel)
    assert not fails, f"{len(fails)} mismatching queries, first: {fails[:5]}"
    return near


# ---------------------------------------------------------------------------------------------
# Confidence rule (Sec. 3 heuristic, strict float threshold).  The neighbour lists obey the same
# near-tie rule as above.  The expected (label, confidence) is the oracle's confidence function
# applied to the reported indices with the ORACLE's distances of those indices (for a query that
# is not near-tie these are simply the oracle's own result).  A decision is *ambiguous*, and then
# either outcome is accepted, when the floating-point margin that decides it is below the
# tolerance: the two best labels' confidences within `rel` of each other (label), or the
# confidence within `rel` of the threshold (hit).  The reported confidence must be within `rel`.
# ---------------------------------------------------------------------------------------------
def _per_label_confidence(labels, idx, d2, k):
    """Comparator-only: all labels' C_i, to find the runner-up (the expected values come from the oracle)."""
    out = {}
    for c in set(int(labels[j]) for j in idx):
        m = [dd for j, dd in zip(idx, d2) if int(labels[j]) == c]
        with np.errstate(divide="ignore"):
            out[c] = (len(m) / k) * float(np.sum(1.0 / np.sqrt(np.asarray(m, dtype=np.float64))))
    return out


def compare_confidence(got, ref, queries, entries, labels, num_classes, k, conf_threshold, rel=REL):
    """got: dict(idx, dist, label, conf, hit).  ref: oracle_reference(...) (its vote fields are unused).
    Returns (near-tie queries, ambiguous decisions, failures)."""
    b = ref["idx"].shape[0]
    n = entries.shape[0]
    thr = np.float32(conf_threshold)
    fails, near, ambiguous = [], 0, 0
    for i in range(b):
        D = ref["sqdist_ext"][i]
        is_near = bool((_rel(D[1:], D[:-1]) < rel).any()) if D.shape[0] > 1 else False
        gi = got["idx"][i]
        gd = got["dist"][i].astype(np.float64)
        if not is_near:
            if not np.array_equal(gi, ref["idx"][i]):
                fails.append(f"q{i}: idx {gi.tolist()} != oracle {ref['idx'][i].tolist()}")
                continue
            true_d = ref["sqdist"][i]
        else:
            near += 1
            if len(set(gi.tolist())) != k or gi.min() < 0 or gi.max() >= n:
                fails.append(f"q{i}: near-tie but indices invalid {gi.tolist()}")
                continue
            true_d = exact_sqdist(queries[i], entries, gi)
            if (true_d > ref["sqdist"][i, k - 1] * (1 + rel)).any():
                fails.append(f"q{i}: near-tie, reported neighbour farther than D(k)(1+rel)")
                continue
        bad = (_rel(gd, true_d) > rel) | ((true_d == 0.0) & (gd != 0.0))
        if bad.any():
            fails.append(f"q{i}: dist {gd.tolist()} vs oracle {true_d.tolist()}")
            continue
        exp_l, exp_c = fo.confidence(labels, gi[None, :], true_d[None, :], num_classes)
        exp_l, exp_c = int(exp_l[0]), float(exp_c[0])
        per = sorted(_per_label_confidence(labels, gi, true_d, k).values(), reverse=True)
        label_amb = len(per) > 1 and not np.isinf(per[0]) and \
            (per[0] == per[1] or _rel(np.float64(per[0]), np.float64(per[1])) < rel)
        gc = float(got["conf"][i])
        if np.isinf(exp_c):
            if not (np.isinf(gc) and gc > 0 and int(got["hit"][i]) == 1):
                fails.append(f"q{i}: zero distance must give +inf confidence and a hit, got {gc}")
            if int(got["label"][i]) != exp_l:
                fails.append(f"q{i}: label {got['label'][i]} != {exp_l}")
            continue
        if label_amb:
            ambiguous += 1
            if _rel(np.float64(gc), np.float64(per[0])) > rel and _rel(np.float64(gc), np.float64(per[1])) > rel:
                fails.append(f"q{i}: confidence {gc} matches neither of the tied labels {per[:2]}")
            continue
        if int(got["label"][i]) != exp_l:
            fails.append(f"q{i}: label {got['label'][i]} != {exp_l} (C {per[:2]})")
        if _rel(np.float64(gc), np.float64(exp_c)) > rel:
            fails.append(f"q{i}: confidence {gc} vs oracle {exp_c}")
        exp_hit = int(np.float32(exp_c) > thr)
        if _rel(np.float64(exp_c), np.float64(thr)) < rel:
            ambiguous += 1                      # the threshold sits inside the rounding margin
            exp_hit = int(np.float32(gc) > thr)   # then the decision must at least follow the reported value
        if int(got["hit"][i]) != exp_hit:
            fails.append(f"q{i}: hit {got['hit'][i]} != {exp_hit} (conf {gc}, oracle {exp_c}, thr {thr})")
    return near, ambiguous, fails
