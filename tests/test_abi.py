"""CPU-only: the C-ABI library loads and exports every symbol include/optimus.h declares;
host-side validation returns the documented error codes without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2104_05343_amd as opt
from paper_2104_05343_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "optimus.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(optimus_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = _declared_symbols()
    assert len(syms) >= 20
    L = ctypes.CDLL(binding.LIB_PATH)
    for s in syms:
        assert hasattr(L, s), s
    # the binding covers the same set
    assert set(binding.SIGNATURES) == set(syms)


def test_error_strings_and_version():
    assert opt.abi_version() == 2
    for code in range(7):
        assert isinstance(opt.error_string(code), str) and opt.error_string(code)
    assert "unknown" in opt.error_string(99)


def test_host_validation_without_gpu():
    L = opt.lib()
    one = ctypes.c_void_p(256)
    # shapes / coordinates / dtype are rejected before anything is enqueued (no GPU needed)
    assert L.optimus_summa_ab(one, one, one, 32, 64, 255, 2, 0, 0, 0, None, 0, None) == opt.ESHAPE
    assert L.optimus_summa_ab(one, one, one, 32, 64, 256, 2, 2, 0, 0, None, 0, None) == opt.ECOORD
    assert L.optimus_summa_ab(one, one, one, 32, 64, 256, 2, -1, 0, 0, None, 0, None) == opt.ECOORD
    assert L.optimus_summa_ab(None, one, one, 32, 64, 256, 2, 0, 0, 0, None, 0, None) == opt.EINVAL
    assert L.optimus_summa_abt(one, one, one, 32, 64, 256, 2, 0, 0, 7, None, 0, None) == opt.EDTYPE
    assert L.optimus_summa_atb(one, one, one, 0, 64, 256, 2, 0, 0, 0, None, 0, None) == opt.ESHAPE
    assert L.optimus_pack_blocks(one, ctypes.c_void_p(512), 6, 8, 4, 2, None) == opt.ESHAPE
    assert L.optimus_pack_blocks(one, ctypes.c_void_p(512), 8, 8, 4, 3, None) == opt.EDTYPE
    assert L.optimus_layernorm2d_stats(one, one, 8, 10, 4, 0, 0, 1, None) == opt.ESHAPE
    assert L.optimus_attention_fwd(one, one, one, 4, 64, 64, 4, 2, 0, 0, 1, 1, None, 0, None) == opt.EWORKSPACE
    assert L.optimus_attention_fwd(one, one, one, 3, 64, 64, 4, 2, 0, 0, 1, 1, one, 1 << 30, None) == opt.ESHAPE
    assert L.optimus_attention_fwd(one, one, one, 4, 64, 64, 4, 2, 0, 0, 1, 0, one, 1 << 30, None) == opt.EDTYPE
    assert L.optimus_attention_fused_fwd(one, one, one, 4, 64, 64, 4, 2, 0, 0, 1, 1, None) == opt.ESHAPE      # d = 16
    assert L.optimus_attention_fused_fwd(one, one, one, 4, 64, 128, 2, 2, 0, 0, 1, 0, None) == opt.EDTYPE
    assert L.optimus_attention_fused_fwd(one, one, one, 4, 64, 128, 2, 2, 2, 0, 1, 1, None) == opt.ECOORD
    assert L.optimus_attention_fused_bwd(one, one, one, one, one, 4, 64, 128, 2, 2, 0, 0, 1, 1, None, 0, None) == opt.EWORKSPACE
    assert L.optimus_attention_fused_workspace_bytes(4, 64, 128, 2, 2) >= 4 * 2 * 64 * 4
    assert L.optimus_attention_fused_workspace_bytes(4, 64, 64, 4, 2) == 0
    assert L.optimus_embedding_fwd(one, one, one, 64, 510, 128, 4, 0, 0, 1, None) == opt.ESHAPE
    assert L.optimus_embedding_bwd(one, one, one, 64, 512, 128, 4, 4, 0, 1, None) == opt.ECOORD
    assert L.optimus_cross_entropy2d(one, one, one, one, one, 64, 512, 4, 0, 0, 9, None) == opt.EDTYPE
    assert L.optimus_cross_entropy2d_bwd(one, one, one, None, 1.0, 64, 512, 4, 0, 0, 1, None) == opt.EINVAL
    assert L.optimus_summa_step(1, one, one, one, 32, 64, 256, 2, 0, 0, 2, 1, None) == opt.ECOORD
    assert L.optimus_summa_reduce(one, 0, one, 32, 64, 2, 0, 0, 1, None) == opt.ESHAPE


def test_stack_sizes_host_only():
    """Buffer sizes of the checkpointed stack (host arithmetic): the checkpoint region is L inputs of b*s*h bf16, the
    conjunction buffer two of them, and a bad configuration is refused."""
    cfg = opt.LayerCfg(8, 512, 1024, 16, 4, 1e-5, 1, opt.BF16)
    act = 8 * 512 * 1024 * 2
    sz = opt.stack_sizes(cfg, 24)
    assert sz.checkpoint == 24 * act and sz.conjunction == 2 * act
    # the stack runs the whole grid: its workspace is the layer's whole-grid size = the minimum plus attention scratch
    # for 15 more devices (8 matrices of 512 x 512, fp32 scores + bf16 gradient each; all 16 fit in 256 MiB)
    one = 8 * 512 * 512 * (4 + 2)
    assert sz.workspace == opt.layer_workspace_bytes_grid(cfg) == opt.layer_workspace_bytes(cfg) + 15 * one
    big = opt.LayerCfg(8, 1024, 4096, 32, 4, 1e-5, 1, opt.BF16)   # 16 matrices of 1024 x 1024 per device: two devices fit
    assert opt.layer_workspace_bytes_grid(big) == opt.layer_workspace_bytes(big) + 16 * 1024 * 1024 * 6
    assert sz.forward >= 12 * act + 16 * 2 * 4 * 512 * 512 * 2        # 12 activation-sized units + probabilities
    assert sz.backward >= 11 * act and sz.param_grad >= 12 * 1024 * 1024 * 4
    fused = opt.LayerCfg(8, 512, 1024, 16, 4, 1e-5, 1, opt.BF16, 1)
    assert opt.stack_sizes(fused, 24).forward < sz.forward
    assert opt.layer_workspace_bytes_grid(fused) == opt.layer_workspace_bytes(fused)   # no score scratch to batch
    for bad_cfg, L in ((opt.LayerCfg(3, 64, 128, 4, 2, 1e-5, 1, opt.BF16), 2), (cfg, 0)):
        with pytest.raises(opt.OptimusError) as e:
            opt.stack_sizes(bad_cfg, L)
        assert e.value.code == opt.ESHAPE


def test_flop_accounting_matches_table1():
    # forward = 2*(12 b s h^2 + 2 b s^2 h)/p flops, backward (no recompute) twice that
    cfg = opt.LayerCfg(8, 1024, 4096, 32, 4, 1e-5, 1, opt.BF16)
    b, s, h, p = 8, 1024, 4096, 16
    assert opt.layer_flops(cfg, 0) == 2 * (12 * b * s * h * h + 2 * b * s * s * h) // p
    assert opt.layer_flops(cfg, 1) == 2 * opt.layer_flops(cfg, 0)
    assert opt.gemm_flops(16384, 3072, 12288, 8) == 2 * 2048 * 3072 * 1536
    assert opt.gemm_flops(10, 3, 4, 4) == -1
    assert opt.layer_workspace_bytes(cfg) >= 16 * 1024 * 1024 * 6
    bad = opt.LayerCfg(8, 1024, 4096, 30, 4, 1e-5, 1, opt.BF16)   # n not divisible by q
    assert opt.layer_flops(bad, 0) == -1 and opt.layer_workspace_bytes(bad) == 0
