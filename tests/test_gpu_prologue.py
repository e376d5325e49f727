"""The fused input prologue (ReLU on the activation operand as it is loaded) against the oracle, on every path that
loads an operand: vector and element loads, transposes, every tile configuration (ring tiles take their
through-registers form), K slices, batched, the convolution in both weight orders and the 1x1 batched-GEMM form."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import (TOL, TORCH_DTYPE, applicable_configs, assert_elementwise, bias_axis_code, conv_scale, gemm_scale,
                     make_conv_workspace, make_workspace, oracle_bias_axis, sliceable_configs, to_f64, to_gpu, within_bound)

pytestmark = pytest.mark.gpu


def _gemm(c, config=-1, k_slices=None, relu=False, alpha=1.0):
    dt = c["dtype"]
    A, B = to_gpu(c["A"], dt), to_gpu(c["B"], dt)
    M, N, K = c["M"], c["N"], c["K"]
    Av = A[:, :M] if c["transA"] else A[:, :K]
    Bv = B[:, :K] if c["transB"] else B[:, :N]
    bias, res = to_gpu(c["bias"], dt), to_gpu(c["residual"], dt)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dt], device="cuda")
    epi = hb.make_epilogue(alpha=alpha, bias=bias, bias_axis=bias_axis_code(c["bias_axis"]), residual=res, relu=relu,
                           relu_input=True)
    if k_slices is None:
        hb.hidet_gemm(Av, Bv, C, transA=c["transA"], transB=c["transB"], epilogue=epi, config=config)
    else:
        hb.hidet_batched_gemm_splitk(Av, Bv, C, make_workspace(1, M, N, k_slices), k_slices=k_slices, transA=c["transA"],
                                     transB=c["transB"], epilogue=epi, config=config)
    torch.cuda.synchronize()
    A64, B64 = wl.widen(c["A"], dt), wl.widen(c["B"], dt)
    A64 = A64[:, :M] if c["transA"] else A64[:, :K]
    B64 = B64[:, :K] if c["transB"] else B64[:, :N]
    b64 = None if c["bias"] is None else wl.widen(c["bias"], dt)
    r64 = None if c["residual"] is None else wl.widen(c["residual"], dt)
    ref = oracle.gemm(A64, B64, transA=c["transA"], transB=c["transB"], alpha=alpha, bias=b64,
                      bias_axis=oracle_bias_axis(c["bias_axis"]), residual=r64, relu=relu, relu_input=True)
    got = to_f64(C)
    assert_elementwise(got, ref, gemm_scale(np.maximum(A64, 0.0), B64, c["transA"], c["transB"], alpha, b64, c["bias_axis"], r64),
                       dt, K, "prologue gemm %dx%dx%d %s config %d" % (M, N, K, dt, config))
    # the prologue must have done something: without it the result differs
    plain = oracle.gemm(A64, B64, transA=c["transA"], transB=c["transB"], alpha=alpha, bias=b64,
                        bias_axis=oracle_bias_axis(c["bias_axis"]), residual=r64, relu=relu)
    assert K == 0 or oracle.rel_frobenius(plain, ref) > 0.05
    return oracle.rel_frobenius(got, ref), ref


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False), (True, True)])
def test_prologue_shapes_and_transposes(dtype, transA, transB):
    for i, (M, N, K) in enumerate([(1, 17, 5), (31, 33, 7), (127, 129, 65), (200, 304, 72), (264, 328, 200)]):
        c = wl.gemm_case(9200 + i, M, N, K, dtype, transA=transA, transB=transB, bias="col", residual=(i % 2 == 0))
        err, ref = _gemm(c, relu=(i % 2 == 1), alpha=0.5)
        assert within_bound(err, ref, dtype), (M, N, K)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_prologue_on_every_config(dtype):
    for cfg in applicable_configs(dtype):
        c = wl.gemm_case(9300 + cfg, 283, 331, 203, dtype, bias="col")       # element loads
        err, ref = _gemm(c, config=cfg, relu=True)
        assert err <= TOL[dtype], cfg
        c = wl.gemm_case(9400 + cfg, 264, 328, 200, dtype, bias="row")       # vector loads (ring tiles: through registers)
        err, ref = _gemm(c, config=cfg)
        assert err <= TOL[dtype], cfg
    for cfg in sliceable_configs(dtype)[::3]:
        c = wl.gemm_case(9500 + cfg, 136, 264, 1000, dtype, residual=True)
        err, ref = _gemm(c, config=cfg, k_slices=3)
        assert err <= TOL[dtype], cfg


def test_prologue_large_ring_shape_and_batched():
    # a shape that the untuned choice gives to a ring tile: it must take the through-registers form
    c = wl.gemm_case(9600, 1024, 1024, 512, "f16", bias="col")
    err, _ = _gemm(c, relu=True)
    assert err <= TOL["f16"]
    g = wl.rng(9601)
    A = wl.normal(g, (5, 70, 96), "f16")
    B = wl.normal(g, (5, 96, 40), "f16")
    C = torch.empty((5, 70, 40), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm(to_gpu(A, "f16"), to_gpu(B, "f16"), C, epilogue=hb.make_epilogue(relu_input=True))
    torch.cuda.synchronize()
    ref = oracle.batched_gemm(wl.widen(A, "f16"), wl.widen(B, "f16"), relu_input=True)
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_prologue_on_convolutions(dtype):
    cases = [(2, 32, 13, 19, 24, 3, 3, 1, 1), (1, 64, 14, 14, 40, 3, 3, 2, 1), (3, 32, 9, 11, 20, 5, 5, 1, 2),
             (2, 64, 10, 12, 48, 1, 1, 1, 0)]  # the last one also has the batched-GEMM form
    for i, (Nb, IC, H, W, OC, KH, KW, s, p) in enumerate(cases):
        c = wl.conv_case(9700 + i, Nb, IC, H, W, OC, KH, KW, s, p, dtype, residual=(i % 2 == 0))
        x, w = to_gpu(c["x"], dtype), to_gpu(c["w"], dtype)
        bias, res = to_gpu(c["bias"], dtype), to_gpu(c["residual"], dtype)
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, residual=res, relu=True, relu_input=True)
        x64, w64 = wl.widen(c["x"], dtype), wl.widen(c["w"], dtype)
        b64 = wl.widen(c["bias"], dtype)
        r64 = None if c["residual"] is None else wl.widen(c["residual"], dtype)
        ref = oracle.conv2d(x64, w64, stride=(s, s), pad=(p, p), bias=b64, residual=r64, relu=True, relu_input=True)
        scale = conv_scale(np.maximum(x64, 0.0), w64, (s, s), (p, p), 1.0, b64, r64)
        y = torch.full(tuple(ref.shape), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
        wp = hb.hidet_conv2d_pack_weights(w)
        runs = {
            "untuned": lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, stride=(s, s), pad=(p, p), epilogue=epi),
            "gather": lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, stride=(s, s), pad=(p, p), epilogue=epi, config=8),
            "sliced": lambda: hb.hidet_conv2d_implicit_gemm_splitk(x, w, y, make_conv_workspace(y.shape, 3), k_slices=3,
                                                                   stride=(s, s), pad=(p, p), epilogue=epi),
            "packed": lambda: hb.hidet_conv2d_implicit_gemm_packed(x, wp, y, stride=(s, s), pad=(p, p), epilogue=epi),
        }
        for name, run in runs.items():
            y.fill_(float("nan"))
            run()
            torch.cuda.synchronize()
            got = to_f64(y)
            assert within_bound(oracle.rel_frobenius(got, ref), ref, dtype), (i, name)
            assert_elementwise(got, ref, scale, dtype, w64[0].size, "prologue conv %d %s" % (i, name))
