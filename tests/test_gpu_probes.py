"""The measurement aids of sart_bench.h do what their declarations say (they are not part of the method, but
bench.py's roofline context rests on them): the read probe accepts its launch shapes and rejects bad ones, and
the matrix-core probe computes the products it claims to time."""
import numpy as np
import pytest

import paper_2505_13326_amd as sart

pytestmark = pytest.mark.gpu


def test_read_probe_shapes_and_argument_checks():
    import torch
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    order = torch.randperm(buf.numel() // 8192, device="cuda").to(torch.int32)
    sart.read_probe(buf)
    sart.read_probe(buf, order)
    for shape in ((256, 1, 0, 0), (2048, 8, 1, 1), (64, 2, 1, 0)):
        sart.read_probe(buf, order, shape=shape)
    torch.cuda.synchronize()
    for bad in ((0, 4, 0, 0), (256, 3, 0, 0), (256, 4, 2, 0)):
        with pytest.raises(sart.SartError):
            sart.read_probe(buf, shape=bad)


@pytest.mark.parametrize("shape", [0, 1])
def test_mfma_probe_sums_its_products(shape):
    """With every operand element equal to 0.5 a product contributes 0.25 per term: after `rounds` rounds every
    accumulator element holds a sum of exactly rounds * (terms per round) * 0.25, and a lane's result is the
    sum of its accumulator elements (all values are exact in fp32 at this size)."""
    import torch
    rounds, n_wg = 3, 4
    ops = torch.full((8192,), 0.5, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((n_wg * 256,), -1.0, dtype=torch.float32, device="cuda")
    sart.mfma_probe(ops, rounds, n_wg, sink, shape=shape)
    torch.cuda.synchronize()
    if shape == 0:
        # per round: 8 products of depth 16 into one 16-element accumulator, 2 into each of four others
        want = rounds * 0.25 * 16 * (8 * 16 + 4 * 2 * 16)
    else:
        # per round: 4 products of depth 32 into each of eight 4-element accumulators
        want = rounds * 0.25 * 32 * (8 * 4 * 4)
    got = sink.cpu().numpy()
    assert np.all(got == want), (got[:4], want)
    # the loop with the softmax: finite sums (weights 2^(s c - reference) of equal scores, whatever the reference)
    sart.mfma_probe(ops, rounds, n_wg, sink, shape=2)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(sink.cpu().numpy())) and np.all(sink.cpu().numpy() > 0)
    with pytest.raises(sart.SartError):
        sart.mfma_probe(ops, 0, n_wg, sink, shape=shape)
    with pytest.raises(sart.SartError):
        sart.mfma_probe(ops, rounds, n_wg, sink, shape=3)
