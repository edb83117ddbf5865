"""The comparator itself: accepts the oracle's own answer, rejects planted mistakes,
and applies the near-tie clause only where two candidate distances are within 1e-4."""
import numpy as np
import torch

from oracle import freeze_oracle as fo
from paper_2002_02645_amd import synth
from tests import parity


def _case():
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=300, batch=40)
    data = synth.make_workload(wl)
    L = data.layers[0]
    q, e, lab = data.queries[0].numpy(), L.entries.numpy(), L.labels.numpy()
    ref = parity.oracle_reference(q, e, lab, 10, wl.k, 4)
    got = dict(idx=ref["idx"].copy(), dist=ref["sqdist"].astype(np.float32), label=ref["label"].copy(),
               votes=ref["votes"].copy(), hit=ref["hit"].copy())
    return q, e, lab, wl.k, ref, got


def test_accepts_oracle_answer():
    q, e, lab, k, ref, got = _case()
    near = parity.assert_lookup_matches(got, ref, q, e, lab, 10, k, 4)
    near_tight = parity.assert_lookup_matches(got, ref, q, e, lab, 10, k, 4, rel=1e-6)
    assert near_tight <= near < 40


def test_rejects_planted_mistakes():
    q, e, lab, k, ref, got = _case()
    for mutate in ("swap", "dist", "label", "hit", "votes", "wrong_idx"):
        g = {key: v.copy() for key, v in got.items()}
        if mutate == "swap":
            g["idx"][3, [0, 1]] = g["idx"][3, [1, 0]]
        elif mutate == "dist":
            g["dist"][5, 2] *= 1.001
        elif mutate == "label":
            g["label"][7] = (g["label"][7] + 1) % 10
        elif mutate == "hit":
            g["hit"][9] ^= 1
        elif mutate == "votes":
            g["votes"][11] -= 1
        else:
            g["idx"][13, k - 1] = (ref["idx_ext"][13, k] if k < e.shape[0] else 0)
        _, fails = parity.compare_lookup(g, ref, q, e, lab, 10, k, 4, rel=1e-6)
        assert fails, mutate


def test_near_tie_clause():
    # two cache rows equidistant from the query up to 2e-5 relative: either order is accepted,
    # but a farther row is not, and the vote must follow the reported indices.
    d = 8
    e = np.zeros((5, d), np.float32)
    e[0, 0] = 1.0
    e[1, 1] = 1.00001
    e[2, 2] = 1.5
    e[3, 3] = 3.0
    e[4, 4] = 4.0
    lab = np.array([0, 1, 1, 0, 0], np.int32)
    q = np.zeros((1, d), np.float32)
    k = 1
    ref = parity.oracle_reference(q, e, lab, 2, k, 1)
    assert ref["idx"][0, 0] == 0
    for first, ok in ((0, True), (1, True), (2, False)):
        d2 = float(parity.exact_sqdist(q[0], e, np.array([first]))[0])
        l, v, h = fo.vote(lab, np.array([[first]], np.int32), 2, 1)
        g = dict(idx=np.array([[first]], np.int32), dist=np.array([[d2]], np.float32), label=l, votes=v, hit=h)
        near, fails = parity.compare_lookup(g, ref, q, e, lab, 2, k, 1)
        assert near == 1 and (not fails) == ok
    # label must be the vote of the reported index, not the oracle's
    g = dict(idx=np.array([[1]], np.int32), dist=np.array([[1.00001 ** 2]], np.float32),
             label=np.array([0], np.int32), votes=np.array([1], np.int32), hit=np.array([1], np.uint8))
    _, fails = parity.compare_lookup(g, ref, q, e, lab, 2, k, 1)
    assert fails


def _confidence_case():
    wl = synth.scaled(synth.WORKLOADS["c1_tiny"], n=300, batch=40)
    data = synth.make_workload(wl)
    L = data.layers[0]
    q, e = data.queries[0].numpy(), L.entries.numpy()
    lab = synth.random_labels(300, 3, 8).numpy()
    ref = parity.oracle_reference(q, e, lab, 3, wl.k, 1)
    res = fo.lookup_confidence(q, e, lab, 3, wl.k, 0.0)
    thr = float(np.median(res["conf"]))
    res = fo.lookup_confidence(q, e, lab, 3, wl.k, thr)
    got = dict(idx=res["idx"].copy(), dist=res["sqdist"].astype(np.float32), label=res["label"].copy(),
               conf=res["conf"].copy(), hit=res["hit"].copy())
    return q, e, lab, wl.k, thr, ref, got


def test_confidence_comparator_accepts_oracle_and_rejects_planted_mistakes():
    q, e, lab, k, thr, ref, got = _confidence_case()
    _, amb, fails = parity.compare_confidence(got, ref, q, e, lab, 3, k, thr, rel=1e-6)
    assert not fails and amb <= 2
    assert 0 < got["hit"].sum() < 40
    for mutate in ("swap", "dist", "label", "hit", "conf"):
        g = {key: v.copy() for key, v in got.items()}
        if mutate == "swap":
            g["idx"][3, [0, 1]] = g["idx"][3, [1, 0]]
        elif mutate == "dist":
            g["dist"][5, 2] *= 1.001
        elif mutate == "label":
            g["label"][7] = (g["label"][7] + 1) % 3
        elif mutate == "hit":
            g["hit"][9] ^= 1
        else:
            g["conf"][11] *= np.float32(1.001)
        _, _, fails = parity.compare_confidence(g, ref, q, e, lab, 3, k, thr, rel=1e-6)
        assert fails, mutate
