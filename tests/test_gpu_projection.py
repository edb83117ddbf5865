"""GPU parity for the projection in front of the look-up (Sec. 3: one-layer dimensionality
reduction): y = W x + bias on bf16-rounded operands, through the C ABI, against the CPU oracle.

The paper fixes no precision for this layer.  The reading taken here DEFINES the projection on
operands rounded to bf16 (x always; W unless it is handed over in bf16), with exact products
and wide accumulation, and the oracle computes exactly that.  So the rounding of the operands is
part of the definition on both sides and this test cannot see it: what it bounds is the error of
the fp32 accumulation on the matrix cores (a few 1e-6 of sum |x_i w_i|).  Against a projection
defined on the unrounded fp32 operands the result would differ by about 2^-9 relative per term."""
import numpy as np
import pytest
import torch

from oracle import freeze_oracle as fo
from paper_2002_02645_amd import binding, synth

pytestmark = pytest.mark.gpu


def _abs_scale(x, w):
    """sum_i |x_i w_i| on the rounded operands: the magnitude the fp32 accumulation error is relative to."""
    xr = np.abs(fo.round_to_bf16(x)).astype(np.float64)
    wr = np.abs(fo.round_to_bf16(w) if w.dtype != np.uint16 else (w.astype(np.uint32) << 16).view(np.float32)).astype(np.float64)
    return xr @ wr.T


@pytest.mark.parametrize("b,d,m,wdtype,relu", [
    (300, 520, 1024, torch.float32, False),   # two tiles of inputs (ragged), four of outputs, ragged depth
    (70, 2048, 100, torch.bfloat16, True),    # fewer outputs than a tile: goes through the padded buffer
    (1, 64, 1, torch.float32, False),
    (600, 96, 300, torch.float32, True),
    (200, 32768, 1024, torch.bfloat16, False),  # four (input tile, output tile) units of great depth: stream-K
    (520, 22000, 512, torch.float32, True),     # stream-K over several input tiles, ragged depth
])
def test_projection_against_oracle(b, d, m, wdtype, relu):
    g = torch.Generator().manual_seed(31 + b + d + m)
    x = torch.randn(b, d, generator=g)
    w = (torch.randn(m, d, generator=g) / d ** 0.5).to(wdtype)
    bias = torch.randn(m, generator=g) * 0.1
    fc = binding.FreezeCache(1)
    try:
        fc.build_projection(0, w.cuda(), bias.cuda())
        y = fc.project(0, x.cuda(), relu)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        # a projection is not a cache
        with pytest.raises(binding.FreezeError):
            fc.lookup(0, x.cuda(), 1, 1)
    finally:
        fc.close()
    w_h = synth.bf16_bits(w) if wdtype == torch.bfloat16 else w.numpy()
    ref = fo.project(x.numpy(), w_h, bias.numpy(), relu)
    scale = _abs_scale(x.numpy(), w_h) + np.abs(bias.numpy())[None, :]
    # fp32 accumulation of exact bf16 x bf16 products in blocks: (log2(d) + 16) * 2^-24 of the magnitude sum
    assert got.shape == ref.shape
    assert (np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 4e-6 * scale + 1e-30).all()
    if relu:
        assert (got >= 0).all() and (got == 0).any()


def test_projection_then_lookup_matches_oracle_pipeline():
    # cache and queries are projected to 256 dimensions first, then looked up (Sec. 3.1: the cache
    # holds dimensionally reduced outputs); the look-up of the GPU's own projections must match the
    # oracle's look-up of the same values
    g = torch.Generator().manual_seed(5)
    n, b, d, m, classes = 3000, 200, 1024, 256, 6
    cent = torch.randn(classes, d, generator=g)
    cls = torch.randint(0, classes, (n,), generator=g)
    pts = cent[cls] + 0.7 * torch.randn(n, d, generator=g)
    qcls = torch.randint(0, classes, (b,), generator=g)
    q = cent[qcls] + 0.7 * torch.randn(b, d, generator=g)
    w = torch.randn(m, d, generator=g) / d ** 0.5
    bias = torch.zeros(m)
    fc = binding.FreezeCache(2)
    try:
        fc.build_projection(0, w.cuda(), bias.cuda())
        pts_r = fc.project(0, pts.cuda(), relu=True)
        q_r = fc.project(0, q.cuda(), relu=True)
        fc.build_layer(1, pts_r, cls.to(torch.int32).cuda(), classes)
        out = fc.lookup(1, q_r, 5, 4)
        torch.cuda.synchronize()
        res = fo.lookup(q_r.cpu().numpy(), pts_r.cpu().numpy(), cls.numpy().astype(np.int32), classes, 5, 4)
        assert np.array_equal(out["idx"].cpu().numpy(), res["idx"])
        assert np.array_equal(out["label"].cpu().numpy(), res["label"])
        assert np.array_equal(out["hit"].cpu().numpy(), res["hit"])
        # the random projection keeps the classes apart: most requests freeze with their own class
        assert (out["label"].cpu().numpy() == qcls.numpy()).mean() > 0.9
    finally:
        fc.close()
