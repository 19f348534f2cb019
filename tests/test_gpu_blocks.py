"""GPU: block addressing (row-major <-> block-major) is bit-exact against the oracle's partition."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import blocks

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("q", [1, 2, 4, 8])
@pytest.mark.parametrize("elem_bytes", [2, 4])
def test_pack_unpack_bit_exact(q, elem_bytes):
    R, C = 24 * q, 40 * q
    npdt, tdt = (np.int16, torch.int16) if elem_bytes == 2 else (np.int32, torch.int32)
    rng = np.random.default_rng(q)
    T = rng.integers(np.iinfo(npdt).min, np.iinfo(npdt).max, size=(R, C)).astype(npdt)
    src = torch.from_numpy(T.reshape(-1)).to("cuda:0")
    dst = torch.zeros(R * C, dtype=tdt, device="cuda:0")
    opt.pack_blocks(src, dst, R, C, q, elem_bytes)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), blocks.pack_block_major(T, q))
    back = torch.zeros(R * C, dtype=tdt, device="cuda:0")
    opt.unpack_blocks(dst, back, R, C, q, elem_bytes)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().reshape(R, C), T)


def test_pack_errors():
    a = torch.zeros(64, dtype=torch.int16, device="cuda:0")
    b = torch.zeros(64, dtype=torch.int16, device="cuda:0")
    for args, code in [((a, b, 6, 8, 4, 2), opt.ESHAPE), ((a, b, 8, 8, 2, 3), opt.EDTYPE), ((a, a, 8, 8, 2, 2), opt.EINVAL)]:
        with pytest.raises(opt.OptimusError) as e:
            opt.pack_blocks(*args)
        assert e.value.code == code
