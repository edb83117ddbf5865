"""The entry point that allocates nothing (freeze_lookup_static: the workspace is a buffer inside
the library's device code) against freeze_lookup on the same inputs, through the C ABI: two calls
in a row, the second with a smaller input, each compared output by output (same kernels, same
layout of the scratch: the results are bit-identical), and the first also against the oracle."""
import numpy as np
import pytest
import torch

from paper_2002_02645_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu


def _outputs(b, k):
    dev = "cuda"
    return dict(label=torch.full((b,), -9, dtype=torch.int32, device=dev),
                hit=torch.full((b,), 9, dtype=torch.uint8, device=dev),
                votes=torch.full((b,), -9, dtype=torch.int32, device=dev),
                idx=torch.full((b, k), -9, dtype=torch.int32, device=dev),
                dist=torch.full((b, k), -9.0, dtype=torch.float32, device=dev))


def _both(fc, q, k, thr, r):
    b = q.shape[0]
    ref = fc.lookup(0, q, k, thr, r, out=_outputs(b, k))
    got = _outputs(b, k)
    rc = binding.lib().freeze_lookup_static(fc.ctx, 0, q.data_ptr(), b, k, thr, r, got["label"].data_ptr(),
                                            got["hit"].data_ptr(), got["votes"].data_ptr(), got["idx"].data_ptr(),
                                            got["dist"].data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == binding.FREEZE_OK, binding.freeze_strerror(rc)
    torch.cuda.synchronize()
    for key in ref:
        assert torch.equal(got[key], ref[key]), key
    return {key: v.cpu().numpy() for key, v in got.items()}


@pytest.mark.parametrize("n,d,b1,b2,k,r,dtype", [
    (3000, 256, 300, 41, 10, 0, torch.bfloat16),     # fused kernel, two query tiles, then one ragged tile (keys-out)
    (20000, 512, 8, 3, 20, 0, torch.bfloat16),       # small-batch kernel twice
    (2000, 512, 256, 100, 5, 0, torch.float32),      # keys-out kernel, fp32 cache
])
def test_static_scratch_matches_workspace_variant(n, d, b1, b2, k, r, dtype):
    wl = synth.scaled(synth.WORKLOADS["c2_batched"], n=n, batch=b1)
    spec = wl.layers[0]
    spec = type(spec)(n, d, 10, spec.sigma, relu=True, store_bf16=(dtype == torch.bfloat16))
    thr = max(1, k - 2)
    data = synth.make_workload(type(wl)(wl.name, (spec,), b1, k, (thr,), r, 4321 + n))
    L = data.layers[0]
    fc = binding.FreezeCache(1)
    try:
        fc.build_layer(0, L.entries.cuda(), L.labels.cuda(), 10)
        q1 = data.queries[0].cuda().contiguous()
        got1 = _both(fc, q1, k, thr, r)
        q2 = q1[b1 - b2:].contiguous()            # the second call: fewer queries, other rows first
        got2 = _both(fc, q2, k, thr, r)
        for key in got1:
            assert np.array_equal(got2[key], got1[key][b1 - b2:]), key
    finally:
        fc.close()
    e_h = synth.bf16_bits(L.entries) if L.entries.dtype == torch.bfloat16 else L.entries.numpy()
    l_h, q_h = L.labels.numpy(), data.queries[0].numpy()
    ref = parity.oracle_reference(q_h, e_h, l_h, 10, k, thr)
    parity.assert_lookup_matches(got1, ref, q_h, e_h, l_h, 10, k, thr, rel=1e-5, dist_rel=1e-5)


def test_static_scratch_limit_and_arguments():
    fc = binding.FreezeCache(1)
    try:
        ent = torch.randn(5000, 512, device="cuda")
        lab = torch.zeros(5000, dtype=torch.int32, device="cuda")
        fc.build_layer(0, ent, lab, 2)
        b = 40000                                   # workspace of this look-up: well above the static buffer
        assert binding.freeze_lookup_workspace_bytes(fc.ctx, 0, b, 5, 0) > binding.FREEZE_STATIC_SCRATCH_BYTES
        q = torch.randn(b, 512, device="cuda")
        out = _outputs(b, 5)
        L = binding.lib()
        s = torch.cuda.current_stream().cuda_stream

        def call(nq=b, k=5, thr=3):
            return L.freeze_lookup_static(fc.ctx, 0, q.data_ptr(), nq, k, thr, 0, out["label"].data_ptr(),
                                          out["hit"].data_ptr(), out["votes"].data_ptr(), out["idx"].data_ptr(),
                                          out["dist"].data_ptr(), s)
        assert call() == binding.FREEZE_ESCRATCH
        assert b"scratch" in L.freeze_strerror(binding.FREEZE_ESCRATCH)
        assert call(k=0) == binding.FREEZE_EINVAL
        assert call(thr=6) == binding.FREEZE_EINVAL
        torch.cuda.synchronize()
        assert (out["label"] == -9).all() and (out["idx"] == -9).all()    # a refused call writes nothing
        assert call(nq=0) == binding.FREEZE_OK
        assert call(nq=100) == binding.FREEZE_OK
        torch.cuda.synchronize()
        assert (out["label"][:100] >= 0).all() and (out["label"][100:] == -9).all()
    finally:
        fc.close()
