"""GPU: the matrix-core rate probe (measurement aid of the benchmark).  Its kernel adds the same 32x32x16 product to
an accumulator `iters` times: all-zero operands give zeros, and with the pseudo-random operands (bf16 magnitudes in
[0.5, 2), so a 16-term dot product is exact in fp32, and so are its first few multiples) the output is linear in
`iters`."""
import pytest
import torch

import paper_2104_05343_amd as opt

pytestmark = pytest.mark.gpu


def _run(wgs, iters, rnd):
    out = torch.full((wgs * 512,), float("nan"), dtype=torch.float32, device="cuda:0")
    opt.debug_mfma_rate(out, wgs, iters, rnd)
    torch.cuda.synchronize()
    return out


def test_probe_zero_operands_and_linearity():
    assert torch.count_nonzero(_run(3, 5, 0)).item() == 0
    one, two, four = _run(3, 1, 1), _run(3, 2, 1), _run(3, 4, 1)
    assert torch.isfinite(one).all() and torch.count_nonzero(one).item() > 0
    assert torch.equal(two, 2 * one) and torch.equal(four, 4 * one)
    # every workgroup computes the same thing
    assert torch.equal(one[:512], one[512:1024])


def test_probe_errors():
    out = torch.empty(512, dtype=torch.float32, device="cuda:0")
    for args, code in [((None, 1, 1, 0), opt.EINVAL), ((out, 0, 1, 0), opt.ESHAPE), ((out, 1, 0, 0), opt.ESHAPE),
                       ((out, 1 << 20, 1, 0), opt.ESHAPE)]:
        with pytest.raises(opt.OptimusError) as e:
            opt.debug_mfma_rate(*args)
        assert e.value.code == code
