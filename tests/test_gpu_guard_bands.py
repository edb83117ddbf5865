"""Out-of-bounds writes: every output and the workspace sit between two 4 KiB guard bands filled
with a poison byte, the workspace is exactly as large as the library says it needs, and after
the call the bands must be untouched (and the outputs must still match a run with ordinary
buffers).  Shapes are ragged on purpose and cover the fused kernel, the keys-out kernel with and
without stream-K, the small-batch kernel, the cascade, the compaction and the row gather."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2002_02645_amd import binding, synth

pytestmark = pytest.mark.gpu

GUARD, POISON = 4096, 0xA5


class Guarded:
    """A device buffer of `nbytes` usable bytes between two poisoned guard bands (256-byte aligned payload)."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        pad = (256 - self.nbytes % 256) % 256
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), POISON, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        self.payload = self.raw[GUARD:GUARD + self.nbytes]

    def view(self, dtype, shape):
        return self.payload.view(dtype).view(shape)

    def intact(self) -> bool:
        # everything outside the payload, including the padding up to the next 256 bytes
        return bool((self.raw[:GUARD] == POISON).all()) and bool((self.raw[GUARD + self.nbytes:] == POISON).all())


def _guarded_outputs(b, k):
    bufs = dict(label=Guarded(b * 4), hit=Guarded(b), votes=Guarded(b * 4), idx=Guarded(b * k * 4), dist=Guarded(b * k * 4))
    out = dict(label=bufs["label"].view(torch.int32, (b,)), hit=bufs["hit"].view(torch.uint8, (b,)),
               votes=bufs["votes"].view(torch.int32, (b,)), idx=bufs["idx"].view(torch.int32, (b, k)),
               dist=bufs["dist"].view(torch.float32, (b, k)))
    return bufs, out


def _make(n, d, b, k, r, dtype, seed):
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b)
    spec = type(wl.layers[0])(n, d, 10, 0.8, relu=True, store_bf16=(dtype == torch.bfloat16))
    return synth.make_workload(type(wl)(wl.name, (spec,), b, k, (max(1, k - 2),), r, seed))


@pytest.mark.parametrize("n,d,b,k,r,dtype", [
    (2999, 250, 301, 7, 0, torch.bfloat16),      # fused kernel, two query tiles, nothing a multiple of a tile
    (3001, 333, 301, 20, 0, torch.float32),      # ... the 32-slot variant, fp32 cache
    (2500, 4160, 37, 10, 64, torch.float32),     # keys-out kernel, R = 64
    (50000, 2048, 64, 10, 0, torch.bfloat16),    # keys-out kernel under stream-K
    (20001, 500, 7, 20, 0, torch.bfloat16),      # small-batch kernel
    (4000, 64, 50, 10, 10, torch.bfloat16),      # no spare candidates: the wider re-scoring and the exact scan run
    (300, 40, 1, 1, 0, torch.float32),           # one query, one neighbour
])
def test_lookup_stays_inside_its_buffers(n, d, b, k, r, dtype):
    data = _make(n, d, b, k, r, dtype, 600 + n)
    L = data.layers[0]
    thr = max(1, k - 2)
    fc = binding.FreezeCache(1)
    try:
        dt = binding.FREEZE_BF16 if dtype == torch.bfloat16 else binding.FREEZE_F32
        storage = Guarded(binding.freeze_cache_storage_bytes(n, d, dt))
        binding.freeze_cache_build(fc.ctx, 0, L.entries.cuda(), L.labels.cuda(), 10, storage.payload)
        q = data.queries[0].cuda()
        ref = fc.lookup(0, q, k, thr, r)                      # ordinary buffers (the holder's own workspace)
        ws = Guarded(binding.freeze_lookup_workspace_bytes(fc.ctx, 0, b, k, r))
        bufs, out = _guarded_outputs(b, k)
        binding.freeze_lookup(fc.ctx, 0, q, k, thr, r, out["label"], out["hit"], out["votes"], out["idx"], out["dist"],
                              ws.payload)
        torch.cuda.synchronize()
        assert storage.intact(), "cache build wrote outside its storage"
        assert ws.intact(), "look-up wrote outside its workspace"
        for key, g in bufs.items():
            assert g.intact(), f"look-up wrote outside out_{key}"
            assert torch.equal(out[key], ref[key]), key
    finally:
        fc.close()


def test_cascade_compaction_and_gather_stay_inside_their_buffers():
    wl = synth.scaled(synth.WORKLOADS["c4_cascade_noisy"], n=1801, d_div=128, batch=333)
    data = synth.make_workload(wl)
    nl = len(wl.layers)
    fc = binding.FreezeCache(nl)
    try:
        for l, L in enumerate(data.layers):
            fc.build_layer(l, L.entries.cuda(), L.labels.cuda(), L.spec.num_classes)
        qs = [q.cuda() for q in data.queries]
        b = wl.batch
        ref = fc.lookup_cascade(list(range(nl)), qs, wl.k, list(wl.vote_thresholds), wl.rescore_r)
        ws = Guarded(binding.freeze_cascade_workspace_bytes(fc.ctx, list(range(nl)), b, wl.k, wl.rescore_r))
        g_lab, g_exit, g_hits = Guarded(b * 4), Guarded(b * 4), Guarded(nl * 8)
        binding.freeze_lookup_cascade(fc.ctx, list(range(nl)), qs, wl.k, list(wl.vote_thresholds), wl.rescore_r,
                                      g_lab.view(torch.int32, (b,)), g_exit.view(torch.int32, (b,)),
                                      g_hits.view(torch.int64, (nl,)), ws.payload)
        torch.cuda.synchronize()
        assert ws.intact() and g_lab.intact() and g_exit.intact() and g_hits.intact()
        assert torch.equal(g_lab.view(torch.int32, (b,)), ref["label"])
        assert torch.equal(g_exit.view(torch.int32, (b,)), ref["exit_layer"])
        assert torch.equal(g_hits.view(torch.int64, (nl,)), ref["hits_per_layer"])

        # compaction of the misses of the first layer, then the gather of their rows
        hit = (ref["exit_layer"] == 0).to(torch.uint8)
        misses = int((hit == 0).sum())
        g_sel, g_cnt = Guarded(b * 4), Guarded(4)
        binding.freeze_compact_misses(hit, None, g_sel.view(torch.int32, (b,)), g_cnt.view(torch.int32, (1,)))
        d1 = qs[1].shape[1]
        g_rows = Guarded(b * d1 * 4)
        binding.freeze_gather_rows(qs[1], g_sel.view(torch.int32, (b,)), g_cnt.view(torch.int32, (1,)),
                                   g_rows.view(torch.float32, (b, d1)))
        torch.cuda.synchronize()
        assert g_sel.intact() and g_cnt.intact() and g_rows.intact()
        assert int(g_cnt.view(torch.int32, (1,)).item()) == misses
        sel = g_sel.view(torch.int32, (b,))[:misses].long()
        assert torch.equal(sel, torch.nonzero(hit == 0).flatten())
        assert torch.equal(g_rows.view(torch.float32, (b, d1))[:misses], qs[1][sel])
        # rows past the count are never written
        assert bool((g_rows.payload.view(torch.uint8)[misses * d1 * 4:] == POISON).all())
    finally:
        fc.close()
